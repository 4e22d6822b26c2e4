// Local halves of the sequence-parallel head exchange (paper section on Arctic Sequence
// Parallelism; Figure 2: in the SP mode each GPU attends with its own heads over all tokens).
// A rank holds its T_loc tokens with all H heads; `pack` lays head slice j out contiguously as
// the block that goes to rank j, `unpack` is the inverse for the blocks that come back after
// attention.  With tokens distributed in contiguous slices in rank order these are the only
// non-trivial local steps: the received pre-attention blocks already form [T][H/P][d], the input
// layout of sp_kv_append and sp_attn_prefill.  Pure bit copies, one 16-byte chunk per lane,
// coalesced on both sides (a head row is d/8 consecutive chunks); HBM-bound, 2 x bytes moved.
#include "sp_common.h"

namespace sp {

// PACK:   dst[j][t][h'][c] = src[t][j * hp + h'][c];  UNPACK: the inverse.  Index space of the
// thread grid is the [T][H][chunks] order, so the [T][H][d] side is fully sequential.
template <bool PACK>
__global__ __launch_bounds__(256) void ulysses_permute_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                              int T_loc, int H, int hp, int cpr, long total) {
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= total) return;
  const int c = (int)(gid % cpr);
  const long th = gid / cpr;
  const int h = (int)(th % H);
  const long t = th / H;
  const int j = h / hp, hl = h - j * hp;
  const long blocked = (((long)j * T_loc + t) * hp + hl) * cpr + c;
  if (PACK) dst[blocked] = __builtin_nontemporal_load(src + gid);
  else dst[gid] = __builtin_nontemporal_load(src + blocked);
}

int launch_ulysses(bool pack, const void *src, void *dst, int T_loc, int H, int d, int P, hipStream_t stream) {
  const int cpr = d / 8;
  const long total = (long)T_loc * H * cpr;
  const long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffL) return fail(SP_ERR_BAD_SHAPE, "ulysses permute: too many elements for one launch");
  if (pack)
    hipLaunchKernelGGL(ulysses_permute_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, (const u32x4 *)src,
                       (u32x4 *)dst, T_loc, H, H / P, cpr, total);
  else
    hipLaunchKernelGGL(ulysses_permute_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, (const u32x4 *)src,
                       (u32x4 *)dst, T_loc, H, H / P, cpr, total);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "ulysses permute launch: %s", hipGetErrorString(e));
  return SP_OK;
}

}  // namespace sp
