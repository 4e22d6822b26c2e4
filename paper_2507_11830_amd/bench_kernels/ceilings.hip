// Two reference kernels that measure what this chip delivers for the two resources the attention
// kernels are bound by, so that achieved figures can be read against the box as well as against
// the datasheet: a register-resident bf16 MFMA loop (no memory, no LDS, no VALU work) and a
// plain 16-byte-per-lane streaming read.  Measurement aids only, built into their own shared
// object (libspceilings.so, declared in include/sp_ceilings.h): the attention library neither
// contains nor uses them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdarg>
#include <cstdio>

#include "sp_ceilings.h"

namespace spc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

static thread_local char g_err[256] = "";
static int fail(int status, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}

// 8 waves per workgroup, each with four independent 32x32x16 accumulators.  RANDOM = false
// multiplies the same two operand registers over and over (what a peak-rate loop usually does);
// RANDOM = true cycles through eight A and eight B registers of pseudo-random bf16 values in
// +-[1, 2), the way a real kernel presents fresh data to the matrix pipe with every instruction.
// The second form draws visibly more power, and the chip answers with a lower clock: it is the
// honest ceiling for a kernel that multiplies real data.
template <bool RANDOM>
__global__ __launch_bounds__(512) void ceiling_mfma_kernel(int iters, float *sink, unsigned long long *clocks) {
  constexpr int NR = RANDOM ? 8 : 1;
  union {
    bf16x8 v;
    unsigned short s[8];
  } a[NR], b[NR];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (RANDOM) {
        h = h * 1664525u + 1013904223u;
        a[r].s[e] = (unsigned short)(0x3F80u | ((h >> 9) & 0x807Fu));   // sign and mantissa from the hash
        b[r].s[e] = (unsigned short)(0x3F80u | ((h >> 17) & 0x807Fu));
      } else {
        a[r].s[e] = (unsigned short)(0x3C00 + (threadIdx.x & 63) + e);
        b[r].s[e] = (unsigned short)(0x3B00 + e);
      }
    }
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; it += 2) {  // two rounds per trip: eight MFMAs, every operand register once
#pragma unroll
    for (int k = 0; k < 8; ++k)
      acc[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k % NR].v, b[(k * 3) % NR].v, acc[k & 3], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  if (threadIdx.x == 0) {
    sink[blockIdx.x] = s;
    if (blockIdx.x == 0) {
      clocks[0] = c1 - c0;  // shader clock cycles of the loop
      clocks[1] = w1 - w0;  // ticks of the constant 100 MHz counter over the same span
    }
  }
}

template <int UNROLL>
__global__ __launch_bounds__(256) void ceiling_stream_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  u32x4 x = {0, 0, 0, 0};
  for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {  // UNROLL independent loads in flight per lane
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) x ^= v[u];
  }
  for (; i < n16; i += stride) x ^= __builtin_nontemporal_load(src + i);
  const uint32_t r = x[0] ^ x[1] ^ x[2] ^ x[3];
  if (r == 0x9E3779B9u) sink[blockIdx.x] = r;  // keeps the loads alive; practically never taken
}

static int cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&p, dev) != hipSuccess) return 0;
    n = p.multiProcessorCount;
  }
  return n;
}

}  // namespace spc

using namespace spc;

extern "C" {

int spc_ceiling_mfma(int32_t iters, int32_t random_operands, double *host_flops, void *sink,
                          size_t sink_bytes, void *stream) {
  if (!host_flops || !sink) return fail(-1, "spc_ceiling_mfma: NULL argument");
  if (iters <= 0 || iters % 2 != 0) return fail(-2, "iters=%d must be positive and even", iters);
  const int cus = cu_count();
  if (cus <= 0) return fail(-5, "cannot read the device properties");
  const size_t need = (size_t)cus * sizeof(float) + 16;
  if (sink_bytes < need) return fail(-4, "sink: need %zu bytes, got %zu", need, sink_bytes);
  // layout of sink: two 64-bit clock readings, then one float per workgroup
  if (random_operands)
    hipLaunchKernelGGL(ceiling_mfma_kernel<true>, dim3(cus), dim3(512), 0, (hipStream_t)stream, iters,
                       (float *)((char *)sink + 16), (unsigned long long *)sink);
  else
    hipLaunchKernelGGL(ceiling_mfma_kernel<false>, dim3(cus), dim3(512), 0, (hipStream_t)stream, iters,
                       (float *)((char *)sink + 16), (unsigned long long *)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(-5, "ceiling launch: %s", hipGetErrorString(e));
  *host_flops = (double)cus * 8.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
  return 0;
}

int spc_ceiling_stream(const void *buf, size_t bytes, int32_t blocks_per_cu, int32_t unroll, void *sink,
                       size_t sink_bytes, void *stream) {
  if (!buf || !sink) return fail(-1, "spc_ceiling_stream: NULL argument");
  if (bytes < 16 || bytes % 16 != 0) return fail(-2, "bytes=%zu must be a positive multiple of 16", bytes);
  if (blocks_per_cu < 1 || blocks_per_cu > 32 || (unroll != 4 && unroll != 8))
    return fail(-2, "blocks_per_cu=%d (1..32), unroll=%d (4 or 8)", blocks_per_cu, unroll);
  const int cus = cu_count();
  if (cus <= 0) return fail(-5, "cannot read the device properties");
  const int grid = cus * blocks_per_cu;
  if (sink_bytes < (size_t)grid * 4) return fail(-4, "sink: need %zu bytes, got %zu", (size_t)grid * 4, sink_bytes);
  if (unroll == 4)
    hipLaunchKernelGGL(ceiling_stream_kernel<4>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)buf,
                       bytes / 16, (uint32_t *)sink);
  else
    hipLaunchKernelGGL(ceiling_stream_kernel<8>, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)buf,
                       bytes / 16, (uint32_t *)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(-5, "ceiling launch: %s", hipGetErrorString(e));
  return 0;
}

const char *spc_last_error(void) { return g_err; }

}  // extern "C"
