// Single-token (decode) GQA attention over the paged KV cache, split over the key range, with
// a log-sum-exp combine pass (sp_attn_decode): the attention each GPU runs on its head shard
// in the tensor-parallel mode.  Same cache, same block table, same arithmetic as the prefill
// kernel (paper section "Introducing Shift Parallelism": the computation and data mapping of
// attention are identical in both modes), only with one query token per sequence.
//
// Split kernel.  One workgroup (4 waves) owns one split — `chunk` consecutive keys — of one
// (sequence, KV-head group).  The group's query heads (<= 32) are the columns of a 32-wide
// MFMA tile, so every K/V byte is read from HBM exactly once for all heads that share it.
// Keys are walked in tiles of 128 tokens (8 pages): the whole workgroup stages the tile
// global -> registers -> LDS with the next tile's loads in flight, then wave w works on key
// rows 32w..32w+31 of the tile with its own running (max, sum, O^T).  The four waves' states
// are merged through LDS at the end and written as an un-normalised fp32 partial
// (o, m, l) per (sequence, head, split).
// Combine kernel: out = sum_k 2^(m_k - M) o_k / sum_k 2^(m_k - M) l_k in fixed split order,
// one round-to-nearest-even to bf16.
//
// Bound: HBM bandwidth.  Algorithmic bytes: 4 * head_dim per cached token per KV head.
#include "attn_tile.h"

namespace sp {

constexpr int kDecWaves = 4;
constexpr int kDecTile = 32 * kDecWaves;  // keys per workgroup tile
constexpr int kDecMinChunk = 256;
constexpr int kDecMaxChunk = 1024;

struct DecodeArgs {
  const char *k_pages, *v_pages, *q;
  const int32_t *seq_lens, *block_table;
  float *part_o;   // [batch][Hq][nsplit][D]
  float *part_ml;  // [batch][Hq][nsplit][2]  (m in log2 units, l)
  int max_pages, num_pages, Hq, Hkv, group, geff, n_hgroups, chunk, nsplit;
  float sl2e;
};

static int pick_chunk(int batch, int num_q_heads, int max_seq_len) {
  // Aim for a few thousand workgroups; assumes ~8 query heads per workgroup and mean length
  // about half the maximum.  Depends only on host-side shape so the workspace size is known.
  long est = (long)batch * num_q_heads * (long)max_seq_len / (8L * 2 * 2048);
  int chunk = kDecMinChunk;
  while (chunk * 2 <= est && chunk < kDecMaxChunk) chunk *= 2;
  return chunk;
}

size_t decode_workspace_bytes(int batch, int max_seq_len, int num_q_heads, int head_dim) {
  if (max_seq_len <= 0) return 0;
  int chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  size_t nsplit = (size_t)(max_seq_len + chunk - 1) / chunk;
  return (size_t)batch * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

template <int D>
__global__ __launch_bounds__(kDecWaves * 64, 2) void decode_split_kernel(DecodeArgs a) {
  using G = TileGeom<D>;
  constexpr int NT = kDecWaves * 64;
  constexpr int KVT = kDecTile;
  constexpr int KBYTES = KVT * G::kKStride, VBYTES = KVT * G::kVStride;
  constexpr int CPR = G::kChunksPerRow;
  constexpr int NCH = KVT * CPR / NT;
  extern __shared__ __align__(16) char smem_raw[];
  lds_char *smem = (lds_char *)smem_raw;
  lds_char *kb = smem, *vb = smem + KBYTES;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
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
      int id = tid + i * NT;
      int kvpos = base + id / CPR, cc = id % CPR;
      int pg = kvpos < kv1 ? bt_row[kvpos >> 4] : -1;
      if (pg >= 0 && pg < a.num_pages) {
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
      int id = tid + i * NT;
      int row = id / CPR, cc = id % CPR;
      *(lds_u32x4 *)(kb + row * G::kKStride + cc * 16) = kreg[i];
      *(lds_u32x4 *)(vb + row * G::kVStride + cc * 16) = vreg[i];
    }
  };

  issue_loads(kv0);
  for (int base = kv0; base < kv1; base += KVT) {
    write_lds();
    __syncthreads();
    if (base + KVT < kv1) issue_loads(base + KVT);
    const int rbase = base + 32 * w;  // first key row of this wave's block
    if (rbase < kv1) {
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < G::kDSteps; ++s) {
        bf16x8 kop = lds_read_k_operand(kb, G::kKStride, 32 * w + col, 2 * s + half);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[s], sacc, 0, 0, 0);
      }
      if (rbase + 32 > kv1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int kv = rbase + 8 * (r >> 2) + 4 * half + (r & 3);
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
          bf16x8 vop = lds_read_vt_operand(vb, G::kVStride, 32 * w + 16 * ks + 4 * half, 32 * db, lane);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[ks], o[db], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // ---- merge the four waves' running states through LDS (the tile buffers are free now)
  // layout: ml[w][col][2] floats, then ow[w][col][D] floats
  constexpr int OS = D + 1;  // odd row stride keeps the column-strided stores off one bank
  lds_float *ml = (lds_float *)smem;
  lds_float *ow = ml + kDecWaves * 32 * 2;
  l += other_half(l);
  if (col < ncols) {
    if (half == 0) {
      ml[(w * 32 + col) * 2 + 0] = m * a.sl2e;  // log2 units; -inf if the wave saw no key
      ml[(w * 32 + col) * 2 + 1] = l;
    }
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        ow[(w * 32 + col) * OS + 32 * db + 8 * (r >> 2) + 4 * half + (r & 3)] = o[db][r];
  }
  __syncthreads();
  // thread -> (column, channel) pairs; fixed wave order keeps the sum reproducible
  for (int idx = tid; idx < ncols * D; idx += NT) {
    int c = idx / D, ch = idx - c * D;
    float M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < kDecWaves; ++ww) M = fmaxf(M, ml[(ww * 32 + c) * 2]);
    float acc = 0.f, lt = 0.f;
#pragma unroll
    for (int ww = 0; ww < kDecWaves; ++ww) {
      float f = __builtin_amdgcn_exp2f(ml[(ww * 32 + c) * 2] - M);
      acc += f * ow[(ww * 32 + c) * OS + ch];
      lt += f * ml[(ww * 32 + c) * 2 + 1];
    }
    long pidx = ((long)seq * a.Hq + head0 + c) * a.nsplit + split;
    a.part_o[pidx * D + ch] = acc;
    if (ch == 0) {
      a.part_ml[pidx * 2] = M;
      a.part_ml[pidx * 2 + 1] = lt;
    }
  }
}

// One workgroup of D/2 threads per (sequence, head); every thread owns two channels.
template <int D>
__global__ __launch_bounds__(D / 2) void decode_combine_kernel(const float *__restrict__ part_o,
                                                               const float *__restrict__ part_ml,
                                                               const int32_t *__restrict__ seq_lens,
                                                               char *__restrict__ out, int Hq, int chunk,
                                                               int nsplit) {
  const int row = blockIdx.x;  // seq * Hq + head
  const int seq = row / Hq;
  const int L = seq_lens[seq];
  const int ch = threadIdx.x * 2;
  bf16x2 *dst = reinterpret_cast<bf16x2 *>(out + ((long)row * D + ch) * 2);
  if (L <= 0 || part_o == nullptr) {
    *dst = __builtin_convertvector((f32x2){0.f, 0.f}, bf16x2);
    return;
  }
  const int n = min((L + chunk - 1) / chunk, nsplit);  // a too-small max_seq_len hint must not read past the workspace
  const float *ml = part_ml + (long)row * nsplit * 2;
  const float *po = part_o + (long)row * nsplit * D + ch;
  float M = -INFINITY;
  for (int k = 0; k < n; ++k) M = fmaxf(M, ml[2 * k]);
  float a0 = 0.f, a1 = 0.f, den = 0.f;
  for (int k = 0; k < n; ++k) {
    float f = __builtin_amdgcn_exp2f(ml[2 * k] - M);
    f32x2 v = *reinterpret_cast<const f32x2 *>(po + (long)k * D);
    a0 += f * v[0];
    a1 += f * v[1];
    den += f * ml[2 * k + 1];
  }
  float inv = 1.0f / den;
  *dst = __builtin_convertvector((f32x2){a0 * inv, a1 * inv}, bf16x2);
}

template <int D>
static int launch_decode_d(DecodeArgs &a, char *out, int batch, hipStream_t stream) {
  using G = TileGeom<D>;
  size_t tile_bytes = (size_t)kDecTile * (G::kKStride + G::kVStride);
  size_t merge_bytes = (size_t)kDecWaves * 32 * (2 + D + 1) * sizeof(float);
  size_t smem = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)decode_split_kernel<D>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return fail(SP_ERR_HIP, "decode smem attribute: %s", hipGetErrorString(e));
    attr_set = true;
  }
  long gy = (long)batch * a.n_hgroups;
  if (gy > 65535) return fail(SP_ERR_BAD_SHAPE, "sp_attn_decode: batch * head groups = %ld exceeds 65535", gy);
  hipLaunchKernelGGL(decode_split_kernel<D>, dim3(a.nsplit, (unsigned)gy), dim3(kDecWaves * 64), smem, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "decode split launch: %s", hipGetErrorString(e));
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(batch * a.Hq), dim3(D / 2), 0, stream, a.part_o, a.part_ml,
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
      hipLaunchKernelGGL(decode_combine_kernel<64>, dim3(batch * a.Hq), dim3(32), 0, stream, a.part_o,
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
