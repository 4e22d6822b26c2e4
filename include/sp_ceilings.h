/*
 * sp_ceilings — measurement aids for benchmarks, built into a shared object of their own
 * (libspceilings.so); the attention library (shiftattn.h) neither contains nor uses them.
 *
 * Two reference kernels that show what THIS chip delivers for the two resources the attention
 * kernels are bound by (the published peaks assume the full boost clock):
 *   mfma    a register-resident bf16 32x32x16 MFMA loop on every CU: 8 waves per CU, `iters`
 *           (positive, even) rounds of four MFMAs each.  random_operands == 0 multiplies the same
 *           two operand registers over and over; != 0 cycles through eight A and eight B
 *           registers of pseudo-random values, as a kernel working on real data does (more
 *           power, hence a lower sustained clock).  *host_flops (HOST pointer) receives the
 *           number of flops the launch performs.  `sink` is DEVICE scratch of at least
 *           16 + 4 * CUs bytes; after the launch its first two uint64 hold the shader-clock
 *           cycles and the ticks of the constant 100 MHz counter that workgroup 0 spent in the
 *           loop (their ratio is the clock the chip sustained under that load).
 *   stream  reads `bytes` (a positive multiple of 16) from DEVICE buffer `buf` once, 16 bytes per
 *           lane, nontemporal, with `blocks_per_cu` (1..32) workgroups of 256 lanes per CU and
 *           `unroll` (4 or 8) independent loads in flight per lane; `sink` is DEVICE scratch of
 *           at least 4 * 32 * CUs bytes.  A benchmark takes the best of several shapes.
 * Both only enqueue on `stream` (a hipStream_t passed as void*, NULL = default stream); the
 * caller times them.  Return value: 0, or a negative code: -1 NULL argument, -2 bad count,
 * -4 sink too small, -5 HIP error (spc_last_error() has the text).  The caller owns all buffers.
 */
#ifndef SP_CEILINGS_H
#define SP_CEILINGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int spc_ceiling_mfma(int32_t iters, int32_t random_operands, double *host_flops, void *sink,
                     size_t sink_bytes, void *stream);
int spc_ceiling_stream(const void *buf, size_t bytes, int32_t blocks_per_cu, int32_t unroll,
                       void *sink, size_t sink_bytes, void *stream);
const char *spc_last_error(void); /* thread-local text of the last failure */

#ifdef __cplusplus
}
#endif
#endif /* SP_CEILINGS_H */
