// Single-token (decode) GQA attention over the paged KV cache, split over the key range, with
// a log-sum-exp combine pass (sp_attn_decode): the attention each GPU runs on its head shard
// in the tensor-parallel mode.  Same cache, same block table, same arithmetic as the prefill
// kernel (paper section "Introducing Shift Parallelism": the computation and data mapping of
// attention are identical in both modes), only with one query token per sequence.
//
// Split kernel.  One WAVE owns one split — `chunk` consecutive keys — of one
// (sequence, KV-head group).  The group's query heads (<= 32) are the columns of a 32-wide
// MFMA tile, so every K/V byte is read from HBM exactly once for all heads that share it.
// The wave walks its keys in blocks of 32 tokens (2 pages): global -> registers -> its own
// LDS region, with the next block's loads in flight while the current block runs
// S^T = K Q^T, the online softmax and O^T += V^T P^T.  Waves never wait for each other, so
// the memory system sees (waves per CU) x 16 KiB in flight.  Each split writes an
// un-normalised fp32 partial (o, m, l) per (sequence, head, split).
// Combine kernel: out = sum_k 2^(m_k - M) o_k / sum_k 2^(m_k - M) l_k in fixed split order,
// one round-to-nearest-even to bf16.
//
// Bound: HBM bandwidth.  Algorithmic bytes: 4 * head_dim per cached token per KV head.
#include "attn_tile.h"

namespace sp {

constexpr int kDecMinChunk = 128;
constexpr int kDecMaxChunk = 1024;  // <= 64 pages, so one lane can hold each page id of a split

struct DecodeArgs {
  const char *k_pages, *v_pages, *q;
  const int32_t *seq_lens, *block_table;
  float *part_o;   // [batch][Hq][nsplit][D]
  float *part_ml;  // [batch][Hq][nsplit][2]  (m in log2 units, l)
  int max_pages, num_pages, Hq, Hkv, group, geff, n_hgroups, chunk, nsplit;
  float sl2e;
};

static int g_chunk_override = 0;  // tuning hook (sp_debug_set_tuning), 0 = heuristic

static int pick_chunk(int batch, int num_q_heads, int max_seq_len) {
  if (g_chunk_override > 0) return g_chunk_override;
  // Largest chunk that still yields a few thousand splits (one wave each), assuming ~8 query
  // heads per split and a mean length of half the maximum.  Depends only on host-side shape so
  // the workspace size is known without reading device memory.
  long est128 = (long)batch * ((num_q_heads + 7) / 8) * ((long)max_seq_len / 2 + 127) / 128;
  int chunk = kDecMinChunk;
  while (chunk < kDecMaxChunk && est128 / (2 * chunk / kDecMinChunk) >= 4096) chunk *= 2;
  return chunk;
}

void set_decode_chunk(int chunk) { g_chunk_override = chunk; }

size_t decode_workspace_bytes(int batch, int max_seq_len, int num_q_heads, int head_dim) {
  if (max_seq_len <= 0) return 0;
  int chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  size_t nsplit = (size_t)(max_seq_len + chunk - 1) / chunk;
  return (size_t)batch * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

// One wave per split.  No workgroup barrier anywhere: the wave stages its own 32-key blocks
// global -> registers -> its private LDS region (next block's loads in flight during the
// current block's MFMAs) and writes its own un-normalised partial.
template <int D>
__global__ __launch_bounds__(64, 2) void decode_split_kernel(DecodeArgs a) {
  using G = TileGeom<D>;
  constexpr int CPR = G::kChunksPerRow;
  constexpr int NCH = 32 * CPR / 64;        // 16-byte chunks per lane per matrix per block
  constexpr int ROWS_PER_LOAD = 64 / CPR;   // key rows covered by one wave-wide load
  constexpr int KBYTES = 32 * G::kKStride, VBYTES = 32 * G::kVStride;
  __shared__ __align__(16) char smem_raw[KBYTES + VBYTES];
  lds_char *kb = (lds_char *)smem_raw, *vb = kb + KBYTES;

  const int lane = threadIdx.x;
  const int col = lane & 31, half = lane >> 5;
  const int seq = blockIdx.y / a.n_hgroups, hg = blockIdx.y - seq * a.n_hgroups;
  const int split = blockIdx.x;
  const int L = a.seq_lens[seq];
  const int kv0 = split * a.chunk;
  if (kv0 >= L) return;
  const int kv1 = min(L, kv0 + a.chunk);
  const int head0 = hg * a.geff;
  const int kvh = head0 / a.group;
  const int ncols = min(a.geff, a.Hq - head0);  // valid columns (heads) of this tile
  const int32_t *bt_row = a.block_table + (long)seq * a.max_pages;

  // Page ids of the whole split, one per lane (chunk <= 64 pages); later broadcast by readlane.
  const int npages = (kv1 - kv0 + kPage - 1) >> 4;
  int my_page = lane < npages ? bt_row[(kv0 >> 4) + lane] : -1;
  if (my_page >= a.num_pages) my_page = -1;  // bad metadata must not become a wild load

  bf16x8 qreg[G::kDSteps];
  {
    const char *qrow = a.q + ((long)seq * a.Hq + head0 + col) * (D * 2);
#pragma unroll
    for (int s = 0; s < G::kDSteps; ++s) {
      if (col < ncols) {
        qreg[s] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * s + 16 * half);
      } else {
        u32x4 z = {0, 0, 0, 0};
        qreg[s] = *reinterpret_cast<bf16x8 *>(&z);
      }
    }
  }
  f32x16 o[G::kDBlocks];
#pragma unroll
  for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  u32x4 kreg[NCH], vreg[NCH];
  auto issue_loads = [&](int base) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = lane + i * 64;
      int row = id / CPR, cc = id % CPR;
      int kvpos = base + row;
      // all lanes of load i sit in one page: its id comes from the lane that fetched it
      int pg = __builtin_amdgcn_readlane(my_page, ((base - kv0) >> 4) + (i * ROWS_PER_LOAD) / kPage);
      if (pg >= 0 && kvpos < kv1) {
        long off = (((long)pg * a.Hkv + kvh) * kPage + (kvpos & 15)) * (D * 2) + cc * 16;
        kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.k_pages + off));
        vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.v_pages + off));
      } else {  // past the split end: zeros, so zero weights never meet NaN payloads
        kreg[i] = (u32x4){0, 0, 0, 0};
        vreg[i] = (u32x4){0, 0, 0, 0};
      }
    }
  };
  auto write_lds = [&]() {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = lane + i * 64;
      int row = id / CPR, cc = id % CPR;
      *(lds_u32x4 *)(kb + row * G::kKStride + cc * 16) = kreg[i];
      *(lds_u32x4 *)(vb + row * G::kVStride + cc * 16) = vreg[i];
    }
  };

  issue_loads(kv0);
  for (int base = kv0; base < kv1; base += 32) {
    write_lds();
    __syncthreads();  // single-wave workgroup: orders the LDS writes before the reads, no s_barrier wait
    if (base + 32 < kv1) issue_loads(base + 32);
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < G::kDSteps; ++s) {
      bf16x8 kop = lds_read_k_operand(kb, G::kKStride, col, 2 * s + half);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[s], sacc, 0, 0, 0);
    }
    if (base + 32 > kv1) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int kv = base + 8 * (r >> 2) + 4 * half + (r & 3);
        if (kv >= kv1) sacc[r] = -INFINITY;
      }
    }
    float mx = sacc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
    mx = fmaxf(mx, other_half(mx));
    const float m_new = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * a.sl2e);
    const float msc = m_new * a.sl2e;
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[r], a.sl2e, -msc));
      sacc[r] = p;
      lsum += p;
    }
    l = l * alpha + lsum;
    m = m_new;
    bf16x8 pop[2] = {pack8(sacc, 0), pack8(sacc, 8)};
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db) {
        bf16x8 vop = lds_read_vt_operand(vb, G::kVStride, 16 * ks + 4 * half, 32 * db, lane);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[ks], o[db], 0, 0, 0);
      }
    __syncthreads();  // reads of this block done before the next block overwrites the region
  }

  // ---- the split's un-normalised partial: a lane holds 4-channel runs of its column
  l += other_half(l);
  if (col < ncols) {
    long pidx = ((long)seq * a.Hq + head0 + col) * a.nsplit + split;
    float *po = a.part_o + pidx * D;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<f32x4 *>(po + 32 * db + 8 * r4 + 4 * half) =
            (f32x4){o[db][4 * r4], o[db][4 * r4 + 1], o[db][4 * r4 + 2], o[db][4 * r4 + 3]};
    if (half == 0) *reinterpret_cast<f32x2 *>(a.part_ml + pidx * 2) = (f32x2){m * a.sl2e, l};
  }
}

// Broadcast of lane k's float (k wave-uniform); the builtin is integer-typed, so bit-cast.
__device__ __forceinline__ float lane_bcast(float x, int k) {
  return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), k));
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// One wave per (sequence, head).  Lane k holds the weight of split k (64 splits per round);
// every lane owns two output channels and accumulates the splits in index order.
template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const float *__restrict__ part_o,
                                                             const float *__restrict__ part_ml,
                                                             const int32_t *__restrict__ seq_lens,
                                                             char *__restrict__ out, int Hq, int chunk,
                                                             int nsplit) {
  const int row = blockIdx.x;  // seq * Hq + head
  const int seq = row / Hq;
  const int L = seq_lens[seq];
  const int lane = threadIdx.x;
  const int ch = (lane % (D / 2)) * 2;
  const bool writer = lane < D / 2;
  bf16x2 *dst = reinterpret_cast<bf16x2 *>(out + ((long)row * D + ch) * 2);
  if (L <= 0 || part_o == nullptr) {
    if (writer) *dst = __builtin_convertvector((f32x2){0.f, 0.f}, bf16x2);
    return;
  }
  // a too-small max_seq_len hint must not read past the workspace
  const int n = min((L + chunk - 1) / chunk, nsplit);
  const f32x2 *ml = reinterpret_cast<const f32x2 *>(part_ml) + (long)row * nsplit;
  const float *po = part_o + (long)row * nsplit * D + ch;
  float M = -INFINITY;
  for (int k = lane; k < n; k += 64) M = fmaxf(M, ml[k][0]);
  M = wave_max(M);
  float a0 = 0.f, a1 = 0.f, den = 0.f;
  for (int base = 0; base < n; base += 64) {
    const int cnt = min(64, n - base);
    float f = 0.f;
    if (lane < cnt) {
      f32x2 v = ml[base + lane];
      f = __builtin_amdgcn_exp2f(v[0] - M);
      den += f * v[1];
    }
    int k = 0;
    for (; k + 4 <= cnt; k += 4) {
      f32x2 v0 = *reinterpret_cast<const f32x2 *>(po + (long)(base + k) * D);
      f32x2 v1 = *reinterpret_cast<const f32x2 *>(po + (long)(base + k + 1) * D);
      f32x2 v2 = *reinterpret_cast<const f32x2 *>(po + (long)(base + k + 2) * D);
      f32x2 v3 = *reinterpret_cast<const f32x2 *>(po + (long)(base + k + 3) * D);
      float f0 = lane_bcast(f, k), f1 = lane_bcast(f, k + 1);
      float f2 = lane_bcast(f, k + 2), f3 = lane_bcast(f, k + 3);
      a0 += f0 * v0[0]; a1 += f0 * v0[1];
      a0 += f1 * v1[0]; a1 += f1 * v1[1];
      a0 += f2 * v2[0]; a1 += f2 * v2[1];
      a0 += f3 * v3[0]; a1 += f3 * v3[1];
    }
    for (; k < cnt; ++k) {
      f32x2 v0 = *reinterpret_cast<const f32x2 *>(po + (long)(base + k) * D);
      float f0 = lane_bcast(f, k);
      a0 += f0 * v0[0]; a1 += f0 * v0[1];
    }
  }
  den = wave_sum(den);
  float inv = 1.0f / den;
  if (writer) *dst = __builtin_convertvector((f32x2){a0 * inv, a1 * inv}, bf16x2);
}

template <int D>
static int launch_decode_d(DecodeArgs &a, char *out, int batch, hipStream_t stream) {
  long gy = (long)batch * a.n_hgroups;
  if (gy > 65535) return fail(SP_ERR_BAD_SHAPE, "sp_attn_decode: batch * head groups = %ld exceeds 65535", gy);
  hipLaunchKernelGGL(decode_split_kernel<D>, dim3(a.nsplit, (unsigned)gy), dim3(64), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "decode split launch: %s", hipGetErrorString(e));
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(batch * a.Hq), dim3(64), 0, stream, a.part_o, a.part_ml,
                     a.seq_lens, out, a.Hq, a.chunk, a.nsplit);
  e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "decode combine launch: %s", hipGetErrorString(e));
  return SP_OK;
}

int launch_decode(const sp_cache_desc &c, const void *q, void *out, const int32_t *seq_lens,
                  const int32_t *block_table, int batch, int max_pages, int max_seq_len,
                  int num_q_heads, float scale, void *workspace, size_t workspace_bytes,
                  hipStream_t stream) {
  (void)workspace_bytes;
  DecodeArgs a;
  a.k_pages = (const char *)c.k_pages;
  a.v_pages = (const char *)c.v_pages;
  a.q = (const char *)q;
  a.seq_lens = seq_lens;
  a.block_table = block_table;
  a.max_pages = max_pages;
  a.num_pages = c.num_pages;
  a.Hq = num_q_heads;
  a.Hkv = c.num_kv_heads;
  a.group = num_q_heads / c.num_kv_heads;
  a.geff = a.group < 32 ? a.group : 32;
  if (a.group % a.geff != 0) a.geff = 1;  // odd large groups: one head per tile
  a.n_hgroups = num_q_heads / a.geff;
  a.sl2e = scale * 1.44269504088896340736f;
  if (max_seq_len <= 0) {
    // every sequence is empty: the combine kernel alone writes the zero rows
    a.chunk = kDecMinChunk;
    a.nsplit = 1;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    if (c.head_dim == 128)
      hipLaunchKernelGGL(decode_combine_kernel<128>, dim3(batch * a.Hq), dim3(64), 0, stream, a.part_o,
                         a.part_ml, seq_lens, (char *)out, a.Hq, a.chunk, a.nsplit);
    else
      hipLaunchKernelGGL(decode_combine_kernel<64>, dim3(batch * a.Hq), dim3(64), 0, stream, a.part_o,
                         a.part_ml, seq_lens, (char *)out, a.Hq, a.chunk, a.nsplit);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SP_ERR_HIP, "decode combine launch: %s", hipGetErrorString(e));
    return SP_OK;
  }
  a.chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  a.nsplit = (max_seq_len + a.chunk - 1) / a.chunk;
  a.part_o = (float *)workspace;
  a.part_ml = a.part_o + (size_t)batch * num_q_heads * a.nsplit * c.head_dim;
  if (c.head_dim == 128) return launch_decode_d<128>(a, (char *)out, batch, stream);
  return launch_decode_d<64>(a, (char *)out, batch, stream);
}

}  // namespace sp
