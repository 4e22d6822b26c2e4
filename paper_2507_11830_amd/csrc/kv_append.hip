// KV append: scatter the new tokens' K and V rows into their 16-token pages.
// This is the step that keeps ONE cache image valid for both the sequence-parallel prefill
// and the tensor-parallel decode (the invariant KV layout of the paper's section
// "Introducing Shift Parallelism").  Pure bit copy with exact int32 page indexing.
//
// Work decomposition: one lane moves one 16-byte chunk of K and the matching chunk of V.
// A token row of one KV head (head_dim bf16) is head_dim/8 chunks, so at head_dim 128
// sixteen adjacent lanes read and write one contiguous 256-byte row: fully coalesced on both
// sides.  HBM-bound: 4 * head_dim bytes read + the same written per (token, kv head).
#include "sp_common.h"

namespace sp {

// The chain of dependent memory round trips decides the time of a small append (a decode step
// moves a few KiB): the new rows are requested first, the per-sequence prefix sums are staged
// in LDS with one cooperative load (so the search for a token's sequence costs no further round
// trips), and only the block-table lookup remains between them and the store.
constexpr int kCuInLds = 2048;  // prefix sums staged in LDS; longer batches search global memory

__global__ __launch_bounds__(256) void kv_append_kernel(
    u32x4 *__restrict__ k_pages, u32x4 *__restrict__ v_pages, const u32x4 *__restrict__ k_new,
    const u32x4 *__restrict__ v_new, const int32_t *__restrict__ cu_new,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ block_table, int batch,
    int max_pages, int num_pages, int chunks_per_head, int num_kv_heads, long total_chunks) {
  __shared__ int32_t s_cu[kCuInLds];
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = gid < total_chunks;
  u32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
  if (live) {
    kv = __builtin_nontemporal_load(k_new + gid);
    vv = __builtin_nontemporal_load(v_new + gid);
  }
  const bool staged = batch + 1 <= kCuInLds;
  if (staged) {
    for (int i = threadIdx.x; i <= batch; i += blockDim.x) s_cu[i] = cu_new[i];
    __syncthreads();
  }
  if (!live) return;
  const int chunks_per_token = chunks_per_head * num_kv_heads;
  const int tok = (int)(gid / chunks_per_token);
  const int rem = (int)(gid - (long)tok * chunks_per_token);
  const int g = rem / chunks_per_head;
  const int c = rem - g * chunks_per_head;

  // Largest s with cu_new[s] <= tok (sequences with no new tokens are skipped over).
  int lo = 0, hi = batch;
  if (staged) {
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (s_cu[mid] <= tok) lo = mid; else hi = mid;
    }
  } else {
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (cu_new[mid] <= tok) lo = mid; else hi = mid;
    }
  }
  const int s = lo;
  // A call on a sub-range of a batch's sequences passes prefix sums that start above 0 and end
  // below total_new_tokens: tokens outside [cu_new[0], cu_new[batch]) belong to other calls.
  const int cu_lo = staged ? s_cu[0] : cu_new[0], cu_hi = staged ? s_cu[batch] : cu_new[batch];
  if (tok < cu_lo || tok >= cu_hi) return;
  const int pos = ctx_lens[s] + (tok - (staged ? s_cu[s] : cu_new[s]));
  const int logical = pos >> 4;
  if (pos < 0 || logical >= max_pages) return;
  const int page = block_table[(long)s * max_pages + logical];
  if (page < 0 || page >= num_pages) return;  // bad metadata must not turn into a wild store
  const long dst = (((long)page * num_kv_heads + g) * kPage + (pos & 15)) * chunks_per_head + c;
  k_pages[dst] = kv;
  v_pages[dst] = vv;
}

int launch_kv_append(const sp_cache_desc &c, const void *k_new, const void *v_new,
                     const int32_t *cu_new, const int32_t *ctx_lens, const int32_t *block_table,
                     int batch, int max_pages, int total_new, hipStream_t stream) {
  int chunks_per_head = c.head_dim / 8;
  long total_chunks = (long)total_new * c.num_kv_heads * chunks_per_head;
  long blocks = (total_chunks + 255) / 256;
  if (blocks > 0x7fffffffL) return fail(SP_ERR_BAD_SHAPE, "sp_kv_append: too many tokens for one launch");
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     (u32x4 *)c.k_pages, (u32x4 *)c.v_pages, (const u32x4 *)k_new,
                     (const u32x4 *)v_new, cu_new, ctx_lens, block_table, batch, max_pages,
                     c.num_pages, chunks_per_head, c.num_kv_heads, total_chunks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "kv_append launch: %s", hipGetErrorString(e));
  return SP_OK;
}

}  // namespace sp
