// Causal GQA flash attention over the paged KV cache for packed varlen query chunks
// (sp_attn_prefill): the attention each GPU runs on its head shard in the sequence-parallel
// mode after the sequence->head exchange, and for chunked prefill against a cached prefix.
// Per the paper's section "Introducing Shift Parallelism" this computation and its data
// mapping are the same in both parallel modes; only the query count per sequence differs.
//
// Decomposition.  One workgroup owns a tile of NW*QB*32 query COLUMNS of one
// (sequence, KV head).  The G = Hq/Hkv query heads that share the KV head are stacked into the
// column dimension (column = token * G + head), so a K/V tile staged in LDS is reused by all
// G heads and all columns of a wave have nearly the same causal bound.  Each wave owns QB
// blocks of 32 columns; the workgroup walks the visible keys in tiles of KVT tokens
// (KVT/16 pages, looked up in the block table), double-buffered in LDS with the next tile's
// global loads in flight during the current tile's MFMAs.
//
// Bound: bf16 MFMA (4 * head_dim flops per visible (query, key) pair per head).  K/V HBM
// traffic is ~1/(8*columns) of that in bytes and is served mostly from L2.
#include "attn_tile.h"

namespace sp {

struct PrefillArgs {
  const char *k_pages, *v_pages, *q;
  char *out;
  const int32_t *cu_q, *ctx_lens, *block_table;
  int max_pages, num_pages, Hq, Hkv, gshift, n_hgroups, ntiles_x;
  float sl2e;  // scale * log2(e)
};

template <int D, int NW, int QB, int KVT>
__global__ __launch_bounds__(NW * 64) void prefill_kernel(PrefillArgs a) {
  using G = TileGeom<D>;
  constexpr int NT = NW * 64;
  constexpr int COLS = NW * QB * 32;
  constexpr int KB = KVT / 32;
  constexpr int KBYTES = KVT * G::kKStride, VBYTES = KVT * G::kVStride, STAGE = KBYTES + VBYTES;
  constexpr int CPR = G::kChunksPerRow;
  constexpr int NCH = KVT * CPR / NT;
  static_assert(KVT * CPR % NT == 0 && NCH >= 1, "tile does not divide over the workgroup");
  extern __shared__ __align__(16) char smem_raw[];
  lds_char *smem = (lds_char *)smem_raw;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int seq = blockIdx.y / a.n_hgroups, hg = blockIdx.y - seq * a.n_hgroups;
  const int tile = a.ntiles_x - 1 - (int)blockIdx.x;  // longest key ranges are dispatched first
  const int tpt = COLS >> a.gshift;                   // tokens per tile
  const int q0 = a.cu_q[seq];
  const int q_len = a.cu_q[seq + 1] - q0;
  const int tok0 = tile * tpt;
  if (tok0 >= q_len) return;
  const int ctx = a.ctx_lens[seq];
  const int kv_end = ctx + min(q_len, tok0 + tpt);
  const int kvh = (hg << a.gshift) / (a.Hq / a.Hkv);
  const int32_t *bt_row = a.block_table + (long)seq * a.max_pages;
  const int gmask = (1 << a.gshift) - 1;

  // ---- per-column state and the resident Q^T operands
  bf16x8 qreg[QB][G::kDSteps];
  int lim[QB];
  bool valid[QB];
  long out_off[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int C = (w * QB + qb) * 32 + col;
    int token = tok0 + (C >> a.gshift);
    int head = (hg << a.gshift) | (C & gmask);
    valid[qb] = token < q_len;
    lim[qb] = valid[qb] ? ctx + token + 1 : 1;
    long row = ((long)(q0 + token) * a.Hq + head) * (D * 2);
    out_off[qb] = row;
#pragma unroll
    for (int s = 0; s < G::kDSteps; ++s) {
      if (valid[qb]) {
        qreg[qb][s] = *reinterpret_cast<const bf16x8 *>(a.q + row + 32 * s + 16 * half);
      } else {
        u32x4 z = {0, 0, 0, 0};
        qreg[qb][s] = *reinterpret_cast<bf16x8 *>(&z);
      }
    }
  }
  // Causal bounds of this wave's columns (wave-uniform).
  const int wtok_first = tok0 + ((w * QB * 32) >> a.gshift);
  const int wtok_last = tok0 + (((w + 1) * QB * 32 - 1) >> a.gshift);
  const int wlim_max = wtok_first < q_len ? ctx + min(wtok_last, q_len - 1) + 1 : 0;
  const int wlim_min = wtok_last < q_len ? ctx + wtok_first + 1 : 1;

  f32x16 o[QB][G::kDBlocks];
  float m[QB], l[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m[qb] = -INFINITY;
    l[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
  }

  // ---- cooperative K/V tile staging: global -> registers -> LDS
  u32x4 kreg[NCH], vreg[NCH];
  int pg[NCH];
  auto load_pages = [&](int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int kvpos = t * KVT + (tid + i * NT) / CPR;
      pg[i] = kvpos < kv_end ? bt_row[kvpos >> 4] : -1;
    }
  };
  auto issue_loads = [&](int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = tid + i * NT;
      int kvpos = t * KVT + id / CPR, cc = id % CPR;
      if (pg[i] >= 0 && pg[i] < a.num_pages) {
        long off = (((long)pg[i] * a.Hkv + kvh) * kPage + (kvpos & 15)) * (D * 2) + cc * 16;
        kreg[i] = *reinterpret_cast<const u32x4 *>(a.k_pages + off);
        vreg[i] = *reinterpret_cast<const u32x4 *>(a.v_pages + off);
      } else {  // rows past the sequence end: zeros, so masked weights never meet NaN payloads
        kreg[i] = (u32x4){0, 0, 0, 0};
        vreg[i] = (u32x4){0, 0, 0, 0};
      }
    }
  };
  auto write_lds = [&](int buf) {
    lds_char *kb = smem + buf * STAGE, *vb = kb + KBYTES;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int id = tid + i * NT;
      int row = id / CPR, cc = id % CPR;
      *(lds_u32x4 *)(kb + row * G::kKStride + cc * 16) = kreg[i];
      *(lds_u32x4 *)(vb + row * G::kVStride + cc * 16) = vreg[i];
    }
  };

  const int ntiles = (kv_end + KVT - 1) / KVT;
  load_pages(0);
  issue_loads(0);
  if (ntiles > 1) load_pages(1);
  write_lds(0);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const bool more = t + 1 < ntiles;
    if (more) {
      issue_loads(t + 1);
      if (t + 2 < ntiles) load_pages(t + 2);
    }
    const int base = t * KVT;
    if (base < wlim_max) {
      const lds_char *kb = smem + (t & 1) * STAGE, *vb = kb + KBYTES;
      // ---- S^T = K Q^T
      f32x16 sacc[QB][KB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[qb][b][r] = 0.f;
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int s = 0; s < G::kDSteps; ++s) {
          bf16x8 kop = lds_read_k_operand(kb, G::kKStride, 32 * b + col, 2 * s + half);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            sacc[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[qb][s], sacc[qb][b], 0, 0, 0);
        }
      // ---- online softmax per column, P packed straight into the PV operand layout
      bf16x8 pop[QB][KB][2];
      const bool need_mask = base + KVT > wlim_min;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (need_mask) {
#pragma unroll
          for (int b = 0; b < KB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int kv = base + 32 * b + 8 * (r >> 2) + 4 * half + (r & 3);
              if (kv >= lim[qb]) sacc[qb][b][r] = -INFINITY;
            }
        }
        float mx = sacc[qb][0][0];
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[qb][b][r]);
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f((m[qb] - m_new) * a.sl2e);
        const float msc = m_new * a.sl2e;
        float lsum = 0.f;
#pragma unroll
        for (int b = 0; b < KB; ++b) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][b][r], a.sl2e, -msc));
            sacc[qb][b][r] = p;
            lsum += p;
          }
          pop[qb][b][0] = pack8(sacc[qb][b], 0);
          pop[qb][b][1] = pack8(sacc[qb][b], 8);
        }
        l[qb] = l[qb] * alpha + lsum;
        m[qb] = m_new;
#pragma unroll
        for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int db = 0; db < G::kDBlocks; ++db) {
            bf16x8 vop = lds_read_vt_operand(vb, G::kVStride, 32 * b + 16 * ks + 4 * half, 32 * db, lane);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[qb][b][ks], o[qb][db], 0, 0, 0);
          }
    }
    if (more) write_lds((t + 1) & 1);
    __syncthreads();
  }

  // ---- normalise and store: a lane holds, per d-block, 4 runs of 4 consecutive channels
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    float lt = l[qb] + other_half(l[qb]);
    float inv = 1.0f / lt;
    if (valid[qb]) {
      char *dst = a.out + out_off[qb];
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          store4_bf16(dst + (32 * db + 8 * r4 + 4 * half) * 2, o[qb][db][4 * r4] * inv,
                      o[qb][db][4 * r4 + 1] * inv, o[qb][db][4 * r4 + 2] * inv,
                      o[qb][db][4 * r4 + 3] * inv);
    }
  }
}

template <int D, int NW, int QB, int KVT>
static int launch_cfg(const PrefillArgs &a0, int batch, int max_q_len, hipStream_t stream) {
  using G = TileGeom<D>;
  PrefillArgs a = a0;
  constexpr int COLS = NW * QB * 32;
  int tpt = COLS >> a.gshift;
  a.ntiles_x = (max_q_len + tpt - 1) / tpt;
  size_t smem = 2 * (size_t)KVT * (G::kKStride + G::kVStride);
  static bool attr_set = false;  // per instantiation; benign if two threads race
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)prefill_kernel<D, NW, QB, KVT>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return fail(SP_ERR_HIP, "prefill smem attribute: %s", hipGetErrorString(e));
    attr_set = true;
  }
  long gy = (long)batch * a.n_hgroups;
  if (gy > 65535) return fail(SP_ERR_BAD_SHAPE, "sp_attn_prefill: batch * head groups = %ld exceeds 65535", gy);
  hipLaunchKernelGGL((prefill_kernel<D, NW, QB, KVT>), dim3(a.ntiles_x, (unsigned)gy), dim3(NW * 64), smem,
                     stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "prefill launch: %s", hipGetErrorString(e));
  return SP_OK;
}

int launch_prefill(const sp_cache_desc &c, const void *q, void *out, const int32_t *cu_q,
                   const int32_t *ctx_lens, const int32_t *block_table, int batch, int max_pages,
                   int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                   hipStream_t stream) {
  (void)total_q;
  (void)max_kv_len;
  PrefillArgs a;
  a.k_pages = (const char *)c.k_pages;
  a.v_pages = (const char *)c.v_pages;
  a.q = (const char *)q;
  a.out = (char *)out;
  a.cu_q = cu_q;
  a.ctx_lens = ctx_lens;
  a.block_table = block_table;
  a.max_pages = max_pages;
  a.num_pages = c.num_pages;
  a.Hq = num_q_heads;
  a.Hkv = c.num_kv_heads;
  int group = num_q_heads / c.num_kv_heads;
  // Stack the heads of a group into the column dimension when the group size is a power of
  // two (<= 32); otherwise every query head gets its own tiles.
  int gshift = 0;
  if ((group & (group - 1)) == 0)
    while ((1 << gshift) < group && gshift < 5) ++gshift;
  a.gshift = gshift;
  a.n_hgroups = num_q_heads >> gshift;
  a.ntiles_x = 0;
  a.sl2e = scale * 1.44269504088896340736f;
  if (c.head_dim == 128) return launch_cfg<128, 8, 1, 64>(a, batch, max_q_len, stream);
  return launch_cfg<64, 8, 1, 64>(a, batch, max_q_len, stream);
}

}  // namespace sp
