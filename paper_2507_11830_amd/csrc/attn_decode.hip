// Single-token (decode) GQA attention over the paged KV cache, split over the key range, with
// a log-sum-exp combine pass (sp_attn_decode): the attention each GPU runs on its head shard
// in the tensor-parallel mode.  Same cache, same block table, same arithmetic as the prefill
// kernel (paper section "Introducing Shift Parallelism": the computation and data mapping of
// attention are identical in both modes), only with one query token per sequence.
//
// Split kernel.  One workgroup of four waves owns one split — `chunk` consecutive keys — of
// one (sequence, KV-head group); the split is cut into four contiguous quarters, one per WAVE.
// The group's query heads (<= 32) are the columns of a 32-wide MFMA tile, so every K/V byte is
// read from HBM exactly once for all heads that share it.  A wave walks its keys in blocks of
// 32 tokens (2 pages): global -> registers -> its own LDS region, with the next block's loads
// in flight while the current block runs S^T = K Q^T, the online softmax and O^T += V^T P^T.
// Waves never wait for each other inside the loop (no workgroup barrier), so the memory system
// sees (waves per CU) x 16 KiB in flight.  At the end the four running states are merged
// through LDS into one un-normalised fp32 partial (o, m, l) per (sequence, head, split).
// Combine kernel: out = sum_k 2^(m_k - M) o_k / sum_k 2^(m_k - M) l_k in fixed split order,
// one round-to-nearest-even to bf16.
//
// Bound: HBM bandwidth.  Algorithmic bytes: 4 * head_dim per cached token per KV head.
#include "attn_tile.h"

namespace sp {

constexpr int kDecWaves = 4;
constexpr int kDecMinChunk = 512;
constexpr int kDecMaxChunk = 4096;  // a wave's quarter is <= 64 pages: one lane holds each page id

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
  // Fewer, longer splits win as long as the grid still has on the order of a hundred
  // workgroups: a wave's fixed costs (first loads, final merge, its partial) are amortised over
  // more keys.  Estimate with ~8 query heads per split and a mean length of half the maximum;
  // only host-side shape is used, so the workspace size is known without reading device memory.
  int chunk = kDecMaxChunk;
  while (chunk > kDecMinChunk) {
    long est = (long)batch * ((num_q_heads + 7) / 8) * ((long)max_seq_len / 2) / chunk;
    if (est >= 128) break;
    chunk /= 2;
  }
  return chunk;
}

void set_decode_chunk(int chunk) { g_chunk_override = chunk; }

size_t decode_workspace_bytes(int batch, int max_seq_len, int num_q_heads, int head_dim) {
  if (max_seq_len <= 0) return 0;
  int chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  size_t nsplit = (size_t)(max_seq_len + chunk - 1) / chunk;
  return (size_t)batch * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

// Orders a wave's own LDS writes before its later LDS reads (and vice versa) without a
// workgroup barrier: the hardware runs one wave's LDS operations in order, so only the
// compiler has to be stopped from moving them across this point.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D>
__global__ __launch_bounds__(kDecWaves * 64, 2) void decode_split_kernel(DecodeArgs a) {
  using G = TileGeom<D>;
  constexpr int CPR = G::kChunksPerRow;
  constexpr int NCH = 32 * CPR / 64;        // 16-byte chunks per lane per matrix per block
  constexpr int ROWS_PER_LOAD = 64 / CPR;   // key rows covered by one wave-wide load
  constexpr int KBYTES = 32 * G::kKStride, VBYTES = 32 * G::kVStride, WBYTES = KBYTES + VBYTES;
  constexpr int OS = D + 1;                 // odd row stride of the merge buffer
  static_assert(32 * (2 + OS) * 4 <= WBYTES, "merge state must fit the wave's tile region");
  __shared__ __align__(16) char smem_raw[kDecWaves * WBYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  lds_char *kb = (lds_char *)smem_raw + w * WBYTES, *vb = kb + KBYTES;
  const int seq = blockIdx.y / a.n_hgroups, hg = blockIdx.y - seq * a.n_hgroups;
  const int split = blockIdx.x;
  // A wave's quarter starts at a position that does not depend on the sequence length, so its
  // page ids and query rows are requested in the same memory round trip as the length itself.
  const int s0 = split * a.chunk;
  const int per_wave = a.chunk / kDecWaves;  // a multiple of 32
  const int kv0 = s0 + w * per_wave;
  const int head0 = hg * a.geff;
  const int kvh = head0 / a.group;
  const int ncols = min(a.geff, a.Hq - head0);  // valid columns (heads) of this tile
  const int32_t *bt_row = a.block_table + (long)seq * a.max_pages;
  // Page ids of the wave's keys, one per lane (<= 64 pages); later broadcast by readlane.
  // Entries past the sequence end are fetched too (index clamped to the table) and never used.
  int my_page = bt_row[min((kv0 >> 4) + lane, a.max_pages - 1)];
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
  const int L = a.seq_lens[seq];
  if (s0 >= L) return;  // whole workgroup
  const int kv1 = min(min(L, s0 + a.chunk), kv0 + per_wave);
  if (my_page >= a.num_pages) my_page = -1;  // bad metadata must not become a wild load

  f32x16 o[G::kDBlocks];
#pragma unroll
  for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  if (kv0 < kv1) {
    u32x4 kreg[NCH], vreg[NCH];
    // Blocks that lie fully inside the range are loaded without any branch (a conditional load
    // forces a full vmcnt(0) at the join, which would expose a memory round trip per block);
    // only the last, partial block takes the guarded path that zero-fills rows past the end, so
    // zero weights never meet NaN payloads of unwritten cache slots.
    auto issue_loads = [&](int base) {
      const int pslot = (base - kv0) >> 4;
      if (base + 32 <= kv1) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          int id = lane + i * 64;
          int row = id / CPR, cc = id % CPR;
          // all lanes of load i sit in one page: its id comes from the lane that fetched it
          int pg = max(__builtin_amdgcn_readlane(my_page, pslot + (i * ROWS_PER_LOAD) / kPage), 0);
          long off = (((long)pg * a.Hkv + kvh) * kPage + ((base + row) & 15)) * (D * 2) + cc * 16;
          kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.k_pages + off));
          vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.v_pages + off));
        }
      } else {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          int id = lane + i * 64;
          int row = id / CPR, cc = id % CPR;
          int kvpos = base + row;
          int pg = __builtin_amdgcn_readlane(my_page, pslot + (i * ROWS_PER_LOAD) / kPage);
          if (pg >= 0 && kvpos < kv1) {
            long off = (((long)pg * a.Hkv + kvh) * kPage + (kvpos & 15)) * (D * 2) + cc * 16;
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.k_pages + off));
            vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.v_pages + off));
          } else {
            kreg[i] = (u32x4){0, 0, 0, 0};
            vreg[i] = (u32x4){0, 0, 0, 0};
          }
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
      wave_lds_fence();
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
      if (L <= 64) {  // very short sequences: weights as hi + lo, so bf16 rounding of P stays out of the tolerance
        bf16x8 plo[2] = {pack8_residual(sacc, 0, pop[0]), pack8_residual(sacc, 8, pop[1])};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int db = 0; db < G::kDBlocks; ++db) {
            bf16x8 vop = lds_read_vt_operand(vb, G::kVStride, 16 * ks + 4 * half, 32 * db, lane);
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, plo[ks], o[db], 0, 0, 0);
          }
      }
      wave_lds_fence();  // reads of this block done before the next block overwrites the region
    }
  }

  // ---- merge the four waves' running states through LDS (each wave reuses its own region)
  // layout per wave: ml[col][2] floats, then ow[col][OS] floats
  l += other_half(l);
  {
    lds_float *ml = (lds_float *)kb;
    lds_float *ow = ml + 32 * 2;
    if (col < ncols) {
      if (half == 0) {
        ml[col * 2 + 0] = m * a.sl2e;  // log2 units; -inf if the wave had no key
        ml[col * 2 + 1] = l;
      }
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) ow[col * OS + 32 * db + 8 * (r >> 2) + 4 * half + (r & 3)] = o[db][r];
    }
  }
  __syncthreads();
  // thread -> (column, channel); fixed wave order keeps the sum reproducible
  for (int idx = tid; idx < ncols * D; idx += kDecWaves * 64) {
    const int c = idx / D, ch = idx - c * D;
    float mw[kDecWaves], M = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < kDecWaves; ++ww) {
      mw[ww] = ((lds_float *)((lds_char *)smem_raw + ww * WBYTES))[c * 2];
      M = fmaxf(M, mw[ww]);
    }
    float acc = 0.f, lt = 0.f;
#pragma unroll
    for (int ww = 0; ww < kDecWaves; ++ww) {
      lds_float *wml = (lds_float *)((lds_char *)smem_raw + ww * WBYTES);
      float f = __builtin_amdgcn_exp2f(mw[ww] - M);  // wave 0 always has a key, so M is finite
      acc += f * wml[64 + c * OS + ch];
      lt += f * wml[c * 2 + 1];
    }
    const long pidx = ((long)seq * a.Hq + head0 + c) * a.nsplit + split;
    a.part_o[pidx * D + ch] = acc;
    if (ch == 0) *reinterpret_cast<f32x2 *>(a.part_ml + pidx * 2) = (f32x2){M, lt};
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
    for (; k + 8 <= cnt; k += 8) {  // eight independent loads in flight per lane
      f32x2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x2 *>(po + (long)(base + k + u) * D);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float fu = lane_bcast(f, k + u);
        a0 += fu * v[u][0];
        a1 += fu * v[u][1];
      }
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
  hipLaunchKernelGGL(decode_split_kernel<D>, dim3(a.nsplit, (unsigned)gy), dim3(kDecWaves * 64), 0, stream, a);
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
