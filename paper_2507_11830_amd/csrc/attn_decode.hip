// Single-token (decode) GQA attention over the paged KV cache, split over the key range, with
// a log-sum-exp combine pass (sp_attn_decode): the attention each GPU runs on its head shard
// in the tensor-parallel mode.  Same cache, same block table, same arithmetic as the prefill
// kernel (paper section "Introducing Shift Parallelism": the computation and data mapping of
// attention are identical in both modes), only with one query token per sequence.
//
// Split kernel.  One WAVE (a 64-thread workgroup) owns one split — `chunk` consecutive keys —
// of one (sequence, KV-head group).  The group's query heads (<= 32) are the columns of a
// 32-wide MFMA tile, so every K/V byte is read from HBM exactly once for all heads that share
// it.  The wave walks its keys in blocks of 32 tokens (2 pages) through a private ring of NB
// LDS slots that are filled by direct global -> LDS loads: while block i runs S^T = K Q^T, the
// online softmax and O^T += V^T P^T, the loads of blocks i+1 .. i+NB-1 are in flight.  The
// kernel is latency-bound unless every CU has several blocks outstanding at all times, and
// LDS (160 KiB per CU) holds far more in-flight data than registers can; nothing in the loop
// synchronises with another wave.  Each wave writes one un-normalised fp32 partial (o, m, l)
// per head.  Combine kernel: out = sum_k 2^(m_k - M) o_k / sum_k 2^(m_k - M) l_k in a fixed
// summation order, one round-to-nearest-even to bf16.
//
// Bound: HBM bandwidth.  Algorithmic bytes: 4 * head_dim per cached token per KV head.
#include <atomic>
#include <mutex>

#include "attn_tile.h"

namespace sp {

constexpr int kDecMinChunk = 128;
constexpr int kDecMaxChunk = 1024;  // <= 64 pages per wave: one lane holds each page id

struct DecodeArgs {
  const char *k_pages, *v_pages, *q;
  const char *k_new, *v_new;  // APPEND kernels: this step's K/V rows, bf16 [tokens][Hkv][D] (one token per sequence unless MQ)
  const int32_t *seq_lens, *block_table;
  const int32_t *cu_q, *ctx_lens;  // MQ kernels: query-token prefix sums [batch + 1], cached lengths [batch]
  float *part_o;   // [row][nsplit][D], row = token * Hq + head (one token per sequence unless MQ)
  float *part_ml;  // [row][nsplit][2]  (m in log2 units, l)
  int max_pages, num_pages, Hq, Hkv, group, geff, n_hgroups, chunk, nsplit;
  int q_cap;  // MQ kernels: query tokens per tile (32 / geff)
  int route_cap;  // MQ kernels: 0, or (mixed batches) only sequences with at most this many query tokens are
                  // served, and the partials are indexed [sequence][route_cap tokens][head] instead of by token row
  int32_t *arrive;  // FUSE kernels: one arrival counter per (sequence, head group), zero between launches
  char *out;        // FUSE kernels: bf16 [batch][Hq][D]
  float sl2e;
  float tau;  // lazy-rescale threshold in raw score units (8 / sl2e)
};

static thread_local int g_chunk_override = 0;  // tuning hooks of the calling thread (sp_debug_set_tuning), 0 = heuristic
static thread_local int g_ring_override = 0;

static int pick_chunk(int batch, int num_q_heads, int max_seq_len, int q_len = 1) {
  if (g_chunk_override > 0) return g_chunk_override;
  // Longer splits amortise a wave's fixed costs (first loads, its partial, the combine pass),
  // shorter ones fill and balance the chip: aim for a few waves per CU.  Estimate with ~8 query
  // heads per split and a mean length of half the maximum; only host-side shape is used, so
  // the workspace size is known without reading device memory.  With several query tokens per
  // sequence a split's partial is that many times larger against the same keys read, so the
  // balance moves towards longer splits (measured on batches of 16 to 256 sequences).
  const long tiles = (long)batch * ((num_q_heads + 7) / 8);
  if (q_len == 1) {
    // Single tokens: when the whole batch fits one round of resident waves (four per CU, by LDS)
    // with splits of at most 512 keys, make it exactly one round — a second, sparsely filled
    // round runs at a fraction of the bandwidth (C3: 1083 waves of 256 keys on 1024 slots take
    // 34.5 us, 870 waves of 320 keys 33.0).  With longer splits the serial chain of a wave's
    // blocks costs more than the second round (measured), and the rule below decides.
    const long slots = 4 * 256 * 85 / 100;  // resident waves of the chip, with a margin for the estimate
    const long one_round = (tiles * (max_seq_len / 2) / slots + 31) / 32 * 32;
    if (one_round <= 512) return (int)(one_round < kDecMinChunk ? kDecMinChunk : one_round);
  }
  const long enough = q_len > 1 ? 256 : 512;
  int chunk = kDecMaxChunk;
  while (chunk > kDecMinChunk) {
    long est = tiles * ((long)max_seq_len / 2) / chunk;
    if (est >= enough) break;
    chunk /= 2;
  }
  return chunk;
}

void set_decode_chunk(int chunk) { g_chunk_override = chunk; }
void set_decode_ring(int slots) { g_ring_override = slots; }

size_t decode_workspace_bytes(int batch, int max_seq_len, int num_q_heads, int head_dim) {
  if (max_seq_len <= 0) return 0;
  int chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  size_t nsplit = (size_t)(max_seq_len + chunk - 1) / chunk;
  return (size_t)batch * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

// Orders a wave's own LDS writes before its later LDS reads without a workgroup barrier: the
// hardware runs one wave's LDS operations in order, so only the compiler has to be stopped from
// moving them across this point.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// s_waitcnt on the vector-memory counter only (the other counters are not named, so they are
// left alone).  The "memory" clobber keeps the compiler from moving LDS reads of the awaited
// block above it.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Fused combine (FUSE forms of the split kernel; OFF by default, tuning key "decode_fuse").  Every
// wave of a (sequence, head group) — the ones without keys too — announces itself on that pair's
// arrival counter after its partial is visible device-wide; the wave that arrives last merges
// the pair's partials and writes the output rows, so the decode step is ONE launch.
// Measured, it loses badly on this chip: the partials of one sequence are written on all eight
// XCDs, whose L2 caches are not coherent with each other, so every wave needs a device-scope
// release (an L2 write-back) in front of its arrival, and with hundreds of waves executing one
// each the 64-sequence decode batch takes 106 us against 33 us for split + combine as two
// launches — the kernel boundary is the cheap device-wide release here.  Plain write-through
// stores plus a wait instead of the fence are not enough (seen: a merging wave reading a slot
// before the other XCD's store had landed).  The counters live in a device array of the
// library, start at zero and are reset by the merging wave, i.e. they are zero again when the
// kernel ends; nothing has to be cleared between launches.
//
// The merge itself: eight lanes per head (eight heads per pass), lane j of a head holds the
// (m, l) pairs of the splits j, j + 8, ... (at most four: the form is used up to 32 splits) and
// 16 channels of the output row.  Weights are exchanged inside the eight-lane groups; the partial
// rows are requested eight splits at a time, all of them before the first is used.  Summation
// order is fixed (split index ascending), so the result does not depend on which wave merges.
template <int D>
__device__ __forceinline__ void arrive_and_merge(const DecodeArgs &a, int lane, int seq, int head0, int ncols) {
  static_assert(D == 128 || D == 64, "head_dim");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // this wave's partial is visible to the whole device before its arrival is
  int old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(a.arrive + blockIdx.y, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != (int)gridDim.x - 1) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // every other wave's partial is visible to this one
  if (lane == 0) a.arrive[blockIdx.y] = 0;  // clean for the next launch
  const int nsplit = a.nsplit;  // <= 32
  constexpr int CPL = D / 8;    // channels per lane
  const int j = lane & 7;
  for (int h0 = 0; h0 < ncols; h0 += 8) {  // uniform
    const int hh = h0 + (lane >> 3);
    const bool hv = hh < ncols;
    const long row = (long)seq * a.Hq + head0 + (hv ? hh : 0);
    const f32x2 *ml = reinterpret_cast<const f32x2 *>(a.part_ml) + row * nsplit;
    const float *po = a.part_o + row * nsplit * D + j * CPL;
    f32x2 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = ml[min(8 * u + j, nsplit - 1)];
    // the first eight partial rows go out with the (m, l) pairs: one round trip for small split counts
    f32x4 v[8][CPL / 4];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int c = 0; c < CPL / 4; ++c) v[k][c] = *reinterpret_cast<const f32x4 *>(po + (long)min(k, nsplit - 1) * D + 4 * c);
    float M = -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) M = fmaxf(M, 8 * u + j < nsplit ? w[u][0] : -INFINITY);
#pragma unroll
    for (int o = 1; o <= 4; o <<= 1) M = fmaxf(M, __shfl_xor(M, o));
    float f[4], den = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool live = 8 * u + j < nsplit && w[u][0] != -INFINITY;
      f[u] = live ? __builtin_amdgcn_exp2f(w[u][0] - M) : 0.f;
      den += live ? f[u] * w[u][1] : 0.f;
    }
#pragma unroll
    for (int o = 1; o <= 4; o <<= 1) den += __shfl_xor(den, o);
    f32x4 acc[CPL / 4];
#pragma unroll
    for (int c = 0; c < CPL / 4; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (8 * u >= nsplit) break;  // uniform
      if (u > 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
          for (int c = 0; c < CPL / 4; ++c)
            v[k][c] = *reinterpret_cast<const f32x4 *>(po + (long)min(8 * u + k, nsplit - 1) * D + 4 * c);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float fk = __shfl(f[u], (lane & ~7) | k);  // weight of split 8u + k (0 past the end or empty)
#pragma unroll
        for (int c = 0; c < CPL / 4; ++c)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[c][e] += fk != 0.f ? fk * v[k][c][e] : 0.f;
      }
    }
    if (hv) {
      const float inv = M == -INFINITY ? 0.f : 1.0f / den;  // a row without keys: zeros
      char *dst = a.out + (row * D + j * CPL) * 2;
#pragma unroll
      for (int c = 0; c < CPL / 4; ++c)
        *reinterpret_cast<bf16x4 *>(dst + 8 * c) =
            __builtin_convertvector(M == -INFINITY ? (f32x4){0.f, 0.f, 0.f, 0.f} : acc[c] * inv, bf16x4);
    }
  }
}

// APPEND = true is the fused decode step: seq_lens counts a new token whose K/V row is NOT in the
// cache yet but in k_new / v_new.  The wave whose range holds that position writes the row into
// its page (for later steps) and patches it into its own LDS copy of the last block (for this
// step), so the separate append launch in front of every decode step disappears.
//
// MQ = true serves short query chunks (speculative-decoding verification: a handful of draft
// tokens per sequence on a long cached prefix, causal inside the chunk; the paper combines Shift
// Parallelism with speculative decoding in its "Arctic Inference" section).  The 32 tile columns
// then hold q_cap tokens x geff heads, each column with its own causal limit, the inputs are the
// ragged ones of sp_attn_prefill (cu_q, ctx_lens), and K/V are still read once for all of them.
// With APPEND as well (sp_chunk_step) the chunk's K/V rows are not in the cache yet: the waves
// whose key range reaches into the chunk fetch them from k_new / v_new, patch them into their
// LDS blocks and store them to their pages.
//
// NT = 2 (MQ only) gives the wave two column tiles, i.e. chunks of up to 2 * q_cap tokens, on the
// same single read of K and V: every K / V operand taken from LDS feeds one multiply per tile.
// The second set of accumulators costs nothing in residency: LDS already limits a CU to four of
// these waves, one per SIMD, so each may use the whole register file.
//
// FUSE = true (single-token forms only) folds the combine pass into this kernel: see arrive_and_merge.
template <int D, int NB, bool APPEND, bool MQ, int NT = 1, bool FUSE = false>
__global__ __launch_bounds__(64, NT > 1 ? 1 : 2) void decode_split_kernel(DecodeArgs a) {
  static_assert(NT == 1 || MQ, "several column tiles only make sense with several query tokens");
  static_assert(!FUSE || !MQ, "the fused combine serves the single-token forms");
  using G = TileGeom<D>;
  using Z = SwzTile<D>;
  constexpr int ROWB = D * 2;           // bytes of one K or V row
  constexpr int MBYTES = 32 * ROWB;     // one 32-key block of K or of V in LDS (swizzled, unpadded)
  constexpr int SLOT = 2 * MBYTES;      // K block, then V block
  constexpr int NI = MBYTES / 1024;     // 1 KiB load instructions per matrix and block
  constexpr int RPI = 1024 / ROWB;      // key rows per load instruction
  constexpr int LPB = 2 * NI;           // load instructions per block
  // NB = 1 is the "one and a half slot" form: two K blocks but a single V block in LDS (24 KiB
  // at head_dim 128 instead of 32; LDS is granted in 1280-byte granules, so that is six resident
  // waves per CU instead of four).  Measured: no faster, the kernel is bandwidth-bound either way.  V of block
  // i + 1 is requested right after the last read of V of block i and has the next block's
  // K Q^T and softmax to land.
  constexpr bool VS = NB == 1;
  static_assert((NB - 1) * LPB < 64, "outstanding loads must fit the vmcnt counter");
  extern __shared__ __align__(16) char smem_raw[];
  lds_char *smem = (lds_char *)smem_raw;

  const int lane = threadIdx.x;
  const int col = lane & 31, half = lane >> 5;
  const int seq = blockIdx.y / a.n_hgroups, hg = blockIdx.y - seq * a.n_hgroups;
  // Consecutive workgroup ids go round-robin over the 8 XCDs; rotating the split index by the
  // row index keeps the high splits (which only long sequences have) from piling onto the same
  // XCDs whenever the split count is a multiple of 8.
  const int split = (int)((blockIdx.x + blockIdx.y) % gridDim.x);
  // A split starts at a position that does not depend on the sequence length, so its page ids
  // and query rows are requested in the same memory round trip as the length itself.
  const int kv0 = split * a.chunk;  // a multiple of 32
  const int head0 = hg * a.geff;
  const int kvh = head0 / a.group;
  const int ncols = min(a.geff, a.Hq - head0);  // valid columns (heads) of this tile
  const int32_t *bt_row = a.block_table + (long)seq * a.max_pages;
  // Page ids of the wave's keys, one per lane (<= 64 pages); later broadcast by readlane.
  // Entries past the sequence end are fetched too (index clamped to the table) and never used.
  int my_page = bt_row[min((kv0 >> 4) + lane, a.max_pages - 1)];
  // Column -> (query token, head) of the tile, and the row of q / out / the partials it stands for.
  int L, ctx = 0, kv_end, lim_min = 0, lim_col[NT];
  bool col_valid[NT];
  long row_col[NT], prow_col[NT];  // row of q / out, and row of the partials (the same unless routed)
  if (MQ) {
    const int tok0 = a.cu_q[seq];
    const int qn = a.cu_q[seq + 1] - tok0;
    ctx = a.ctx_lens[seq];
    if (qn <= 0) return;  // no query token: no output row, no partial
    if (a.route_cap > 0 && qn > a.route_cap) return;  // mixed batch: the prefill kernel serves this sequence
    L = ctx + qn;
    kv_end = L;          // keys visible to the chunk's last token
    lim_min = ctx + 1;   // keys visible to its first token
    const int t0 = col / a.geff, h_col = col - t0 * a.geff;  // the host made sure that qn <= NT * q_cap
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int t = nt * a.q_cap + t0;  // tile nt holds the tokens nt * q_cap .. (nt + 1) * q_cap - 1
      col_valid[nt] = t0 < a.q_cap && t < qn && h_col < ncols;
      row_col[nt] = (long)(tok0 + t) * a.Hq + head0 + h_col;
      prow_col[nt] = a.route_cap > 0 ? ((long)seq * a.route_cap + t) * a.Hq + head0 + h_col : row_col[nt];
      lim_col[nt] = col_valid[nt] ? ctx + t + 1 : kv_end;
    }
  } else {
    col_valid[0] = col < ncols;
    row_col[0] = (long)seq * a.Hq + head0 + col;
    prow_col[0] = row_col[0];
    lim_col[0] = 0;
    L = 0;  // loaded below, after the query rows are requested
    kv_end = 0;
  }
  bf16x8 qreg[NT][G::kDSteps];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const char *qrow = a.q + row_col[nt] * (D * 2);
#pragma unroll
    for (int s = 0; s < G::kDSteps; ++s) {
      if (col_valid[nt]) {
        qreg[nt][s] = *reinterpret_cast<const bf16x8 *>(qrow + 32 * s + 16 * half);
      } else {
        u32x4 z = {0, 0, 0, 0};
        qreg[nt][s] = *reinterpret_cast<bf16x8 *>(&z);
      }
    }
  }
  // this step's new K/V row, one 16-byte chunk per lane (64 / CPR copies of the row per wave);
  // requested by every wave, used by the one that owns the position
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  u32x4 knew = {0, 0, 0, 0}, vnew = {0, 0, 0, 0};
  if (APPEND && !MQ) {
    const size_t noff = (((size_t)seq * a.Hkv + kvh) * CPR + (lane % CPR)) * 16;
    knew = *reinterpret_cast<const u32x4 *>(a.k_new + noff);
    vnew = *reinterpret_cast<const u32x4 *>(a.v_new + noff);
  }
  if (!MQ) {
    L = a.seq_lens[seq];
    kv_end = L;
  }
  if (kv0 >= kv_end) {  // nothing to attend to: an empty partial, so the combine pass needs no lengths
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (lane < 32 && col_valid[nt])
        *reinterpret_cast<f32x2 *>(a.part_ml + (prow_col[nt] * a.nsplit + split) * 2) = (f32x2){-INFINITY, 0.f};
    if (FUSE) arrive_and_merge<D>(a, lane, seq, head0, ncols);
    return;
  }
  const int kv1 = min(kv_end, kv0 + a.chunk);
  const int nb = (kv1 - kv0 + 31) >> 5;  // blocks of this wave, >= 1
  // Bad metadata must not become a wild access: loads go through the clamped page id (finite
  // garbage, as sp_attn_decode documents for unvalidated metadata), the fused-append stores
  // through the raw one, and are skipped when it lies outside the pool or past the table row
  // (the same rows sp_kv_append skips).
  const int my_page_raw = (kv0 >> 4) + lane < a.max_pages ? my_page : -1;
  my_page = min(max(my_page, 0), a.num_pages - 1);

  // ---- block loads.  Instruction j of a matrix covers RPI rows: lane l fills chunk slot l % 16
  // of line 4j + l / 16 of the block and fetches whichever global chunk the swizzle assigns to
  // that slot.  Rows past the end of the range are redirected to its last row (finite data;
  // their scores are masked).
  const int last_row = kv1 - 1 - kv0;  // relative to kv0
  const int dq = lane >> 4, dslot = lane & 15;
  constexpr int IPP = NI / 2;  // load instructions per page and matrix
  unsigned voff_k[IPP], voff_v[IPP];  // this lane's byte offset inside a (page, kv head) block, per instruction
#pragma unroll
  for (int jj = 0; jj < IPP; ++jj) {
    const int line = 4 * jj + dq;
    const int clk = dslot ^ Z::gk(line), clv = dslot ^ Z::gv(line);
    voff_k[jj] = (unsigned)(((D == 128 ? line : 2 * line + (clk >> 3)) & 15) * ROWB + (D == 128 ? clk : (clk & 7)) * 16);
    voff_v[jj] = (unsigned)(((D == 128 ? line : 2 * line + (clv >> 3)) & 15) * ROWB + (D == 128 ? clv : (clv & 7)) * 16);
  }
  const size_t page_stride = (size_t)a.Hkv * (kPage * ROWB);
  const char *kpool = a.k_pages + (size_t)kvh * (kPage * ROWB), *vpool = a.v_pages + (size_t)kvh * (kPage * ROWB);
  // K (isv = false) or V block bi of the wave's range into the LDS bytes [dst0, dst0 + MBYTES).
  // The "memory" clobber keeps LDS reads of the bytes being replaced on the near side of the request.
  auto issue_mat = [&](int bi, bool isv, unsigned dst0) {
    const char *pool = isv ? vpool : kpool;
    if (32 * bi + 31 <= last_row) {
      // both pages of the block lie inside the range: two page bases, precomputed lane offsets
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        const char *pb = pool + (size_t)(unsigned)__builtin_amdgcn_readlane(my_page, 2 * bi + pp) * page_stride;
#pragma unroll
        for (int jj = 0; jj < IPP; ++jj) {
          const unsigned dst = dst0 + (pp * IPP + jj) * 1024;
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(dst),
                       "v"(isv ? voff_v[jj] : voff_k[jj]), "s"(pb)
                       : "memory");
        }
      }
      return;
    }
    // the last, partial block: rows past the end are redirected to the last row
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int row0 = 32 * bi + RPI * j;                   // first row of the instruction, relative to kv0
      const int pslot = min(row0, last_row) >> 4;           // uniform
      const int rip_lim = pslot == (last_row >> 4) ? (last_row & 15) : 15;
      const char *pb = pool + (size_t)(unsigned)__builtin_amdgcn_readlane(my_page, pslot) * page_stride;
      const int line = 4 * j + dq;                          // line inside the block
      const int cl = dslot ^ (isv ? Z::gv(line) : Z::gk(line));
      const int rip = (D == 128 ? line : 2 * line + (cl >> 3)) & 15;
      const int chunk16 = D == 128 ? cl : (cl & 7);
      const unsigned voff = (unsigned)(min(rip, rip_lim) * ROWB + chunk16 * 16);
      const unsigned dst = dst0 + j * 1024;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(dst), "v"(voff), "s"(pb)
                   : "memory");
    }
  };
  auto issue_block = [&](int bi) {  // ring forms: K and V of block bi into slot bi % NB
    const unsigned slot_base = (unsigned)((bi % NB) * SLOT);
    issue_mat(bi, false, slot_base);
    issue_mat(bi, true, slot_base + MBYTES);
  };

  // ---- LDS operand offsets of this lane inside a slot
  int kofs[G::kDSteps], vofs[G::kDBlocks];
#pragma unroll
  for (int s = 0; s < G::kDSteps; ++s) kofs[s] = Z::template offset<false>(col, 2 * s + half);
  {
    const int n = lane & 15, dg = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
      vofs[db] = Z::template offset<true>(4 * half + (n >> 2), 4 * db + 2 * dg + ((n & 3) >> 1)) + 8 * (n & 1);
  }
  f32x16 o[NT][G::kDBlocks];
  // MQ: a column may find every key of the wave's first blocks behind its causal limit; a
  // finite floor keeps exp2(m - m) defined for it (the partial is written as empty if l stays 0).
  float m[NT], l[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m[nt] = MQ ? -1e30f : -INFINITY;
    l[nt] = 0.f;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[nt][db][r] = 0.f;
  }

  if (VS) {  // requests are made in the order K0 V0 K1 | V1 K2 | V2 K3 | ... and retire in that order
    issue_mat(0, false, 0);
    issue_mat(0, true, 2 * MBYTES);
    if (nb > 1) issue_mat(1, false, MBYTES);
  } else {
#pragma unroll
    for (int bi = 0; bi < NB - 1; ++bi)
      if (bi < nb) issue_block(bi);
  }
  for (int i = 0; i < nb; ++i) {
    const lds_char *sbk, *sbv;  // K and V block of this iteration
    if (VS) {
      sbk = smem + (i & 1) * MBYTES;
      sbv = smem + 2 * MBYTES;
      // behind K(i) in the queue: V(i), and K(i+1) if there is one.  The last block waits for
      // everything (the fused append patches both of its matrices).
      if (i + 1 < nb) wait_vmcnt<2 * NI>();
      else if (APPEND) wait_vmcnt<0>();
      else wait_vmcnt<NI>();
    } else {
      // the slot of block i-1 is free again: keep NB-1 blocks in flight behind block i
      if (i + NB - 1 < nb) issue_block(i + NB - 1);
      const int behind = min(NB - 1, nb - 1 - i);  // blocks requested after block i
      if (behind >= 3 && NB > 3) wait_vmcnt<(NB > 3 ? 3 : 0) * LPB>();
      else if (behind == 2 && NB > 2) wait_vmcnt<(NB > 2 ? 2 : 0) * LPB>();
      else if (behind == 1 && NB > 1) wait_vmcnt<(NB > 1 ? 1 : 0) * LPB>();
      else wait_vmcnt<0>();
      sbk = smem + (i % NB) * SLOT;
      sbv = sbk + MBYTES;
    }
    const int base = kv0 + 32 * i;
    if (APPEND && MQ && base + 32 > ctx) {
      // Fused append of a short chunk: the rows of this block at positions >= ctx are not in the
      // cache yet (the loads brought stale bytes).  Every lane fetches its 16-byte pieces of the
      // new rows, patches the block in LDS and, for positions inside the wave's range, stores
      // them to their pages — one writer per (position, KV head).  Rows past the end of the
      // range take the chunk's last row: finite, and masked.  At most two blocks of a sequence
      // reach into its chunk, so the extra round trip is paid once or twice per sequence.
      const int tok0 = a.cu_q[seq];
      const int c = lane % CPR;
      const bool writer = head0 % a.group == 0;
#pragma unroll
      for (int j = 0; j < 32 * CPR / 64; ++j) {
        const int row = j * (64 / CPR) + lane / CPR;
        const int pos = base + row;
        // page of this position, from the lane that holds it: taken by all lanes, outside the
        // branch (a cross-lane read must not depend on which lanes the branch leaves active)
        const int pg = __shfl(my_page_raw, min((pos - kv0) >> 4, 63));
        if (pos >= ctx) {
          const int t = min(pos, L - 1) - ctx;
          const size_t noff = (((size_t)(tok0 + t) * a.Hkv + kvh) * CPR + c) * 16;
          const u32x4 kn = *reinterpret_cast<const u32x4 *>(a.k_new + noff);
          const u32x4 vn = *reinterpret_cast<const u32x4 *>(a.v_new + noff);
          *(lds_u32x4 *)(const_cast<lds_char *>(sbk) + Z::template offset<false>(row, c)) = kn;
          *(lds_u32x4 *)(const_cast<lds_char *>(sbv) + Z::template offset<true>(row, c)) = vn;
          if (writer && pos < kv1 && pg >= 0 && pg < a.num_pages) {
            const size_t dst = (size_t)(unsigned)pg * page_stride + (size_t)(pos & 15) * ROWB + c * 16;
            *reinterpret_cast<u32x4 *>(const_cast<char *>(kpool) + dst) = kn;
            *reinterpret_cast<u32x4 *>(const_cast<char *>(vpool) + dst) = vn;
          }
        }
      }
      wave_lds_fence();
    }
    if (APPEND && !MQ && kv1 == L && i == nb - 1) {
      // The block that holds position L-1 has landed (it is the last one: nothing behind it).
      // Its row for that position and the rows after it (redirected to it) are stale cache
      // bytes: overwrite them in LDS with the new row, and store the row to its page.
      const int r_new = last_row & 31;  // row of the new token inside this block
      const int c = lane % CPR;
#pragma unroll
      for (int j = 0; j < 32 * CPR / 64; ++j) {
        const int row = j * (64 / CPR) + lane / CPR;
        if (row >= r_new) {
          *(lds_u32x4 *)(const_cast<lds_char *>(sbk) + Z::template offset<false>(row, c)) = knew;
          *(lds_u32x4 *)(const_cast<lds_char *>(sbv) + Z::template offset<true>(row, c)) = vnew;
        }
      }
      const int pg = __builtin_amdgcn_readlane(my_page_raw, last_row >> 4);
      if (lane < CPR && head0 % a.group == 0 && pg >= 0 && pg < a.num_pages) {  // one writer per (sequence, KV head)
        const size_t dst = (size_t)(unsigned)pg * page_stride + (size_t)((kv0 + last_row) & 15) * ROWB + c * 16;
        *reinterpret_cast<u32x4 *>(const_cast<char *>(kpool) + dst) = knew;
        *reinterpret_cast<u32x4 *>(const_cast<char *>(vpool) + dst) = vnew;
      }
      wave_lds_fence();
    }

    f32x16 sacc[NT], sacc1[NT];  // two accumulators per tile halve the dependent MFMA chain a lone wave sits through
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[nt][r] = sacc1[nt][r] = 0.f;
#pragma unroll
    for (int s = 0; s < G::kDSteps; s += 2) {
      bf16x8 kop0 = *(const lds_bf16x8 *)(sbk + kofs[s]);
      bf16x8 kop1 = *(const lds_bf16x8 *)(sbk + kofs[s + 1]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        sacc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop0, qreg[nt][s], sacc[nt], 0, 0, 0);
        sacc1[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop1, qreg[nt][s + 1], sacc1[nt], 0, 0, 0);
      }
    }
    bf16x8 pop[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[nt][r] += sacc1[nt][r];
      if (MQ) {
        if (base + 32 > min(lim_min, kv1)) {  // the block reaches into the chunk: per-column causal limit
          const int lim = min(lim_col[nt], kv1);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int kv = base + 8 * (r >> 2) + 4 * half + (r & 3);
            if (kv >= lim) sacc[nt][r] = -INFINITY;
          }
        }
      } else if (base + 32 > kv1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int kv = base + 8 * (r >> 2) + 4 * half + (r & 3);
          if (kv >= kv1) sacc[nt][r] = -INFINITY;
        }
      }
      float mx = sacc[nt][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[nt][r]);
      mx = fmaxf(mx, other_half(mx));
      // The running max only moves when some column's block max exceeds it by more than 2^8 in
      // the exponent (tau); otherwise weights are taken against the stale max (bounded by 2^8,
      // harmless in fp32/bf16) and the O accumulators need no rescale.
      if (__builtin_amdgcn_ballot_w64(mx > m[nt] + a.tau) != 0) {  // wave-uniform, rare after the first block
        const float m_new = fmaxf(m[nt], mx);
        const float alpha = __builtin_amdgcn_exp2f((m[nt] - m_new) * a.sl2e);
        m[nt] = m_new;
        l[nt] *= alpha;
#pragma unroll
        for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[nt][db][r] *= alpha;
      }
      const float msc = m[nt] * a.sl2e;
      float lsum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[nt][r], a.sl2e, -msc));
        sacc[nt][r] = p;
        lsum += p;
      }
      l[nt] += lsum;
      pop[nt][0] = pack8(sacc[nt], 0);
      pop[nt][1] = pack8(sacc[nt], 8);
    }
    if (VS) {  // behind V(i) in the queue: K(i+1) if there is one
      if (i + 1 < nb) wait_vmcnt<NI>();
      else wait_vmcnt<0>();
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db) {
        bf16x8 vop = lds_read_vt(sbv + vofs[db] + 16 * ks * ROWB, ROWB);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          o[nt][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[nt][ks], o[nt][db], 0, 0, 0);
      }
    if (L <= 256) {  // short sequences: weights as hi + lo, so the bf16 rounding of P (which only averages out over many keys) stays out of the tolerance
      bf16x8 plo[NT][2];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        plo[nt][0] = pack8_residual(sacc[nt], 0, pop[nt][0]);
        plo[nt][1] = pack8_residual(sacc[nt], 8, pop[nt][1]);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < G::kDBlocks; ++db) {
          bf16x8 vop = lds_read_vt(sbv + vofs[db] + 16 * ks * ROWB, ROWB);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            o[nt][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, plo[nt][ks], o[nt][db], 0, 0, 0);
        }
    }
    if (VS) {
      // Every read of V(i) and of K(i) has been consumed by a multiply above (the scheduling
      // barrier keeps the requests below them): their bytes may be replaced.
      __builtin_amdgcn_sched_barrier(0);
      if (i + 1 < nb) issue_mat(i + 1, true, 2 * MBYTES);
      if (i + 2 < nb) issue_mat(i + 2, false, (i & 1) * MBYTES);
    }
  }

  // ---- the wave's partial: un-normalised o, m in log2 units, l
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float lt = l[nt] + other_half(l[nt]);
    if (col_valid[nt]) {
      const long pidx = prow_col[nt] * a.nsplit + split;
      float *po = a.part_o + pidx * D;
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *reinterpret_cast<f32x4 *>(po + 32 * db + 8 * r4 + 4 * half) =
              (f32x4){o[nt][db][4 * r4], o[nt][db][4 * r4 + 1], o[nt][db][4 * r4 + 2], o[nt][db][4 * r4 + 3]};
      if (half == 0)
        *reinterpret_cast<f32x2 *>(a.part_ml + pidx * 2) = (f32x2){MQ && lt == 0.f ? -INFINITY : m[nt] * a.sl2e, lt};
    }
  }
  if (FUSE) arrive_and_merge<D>(a, lane, seq, head0, ncols);
}

// Broadcast of lane k's float (k wave-uniform); the builtin is integer-typed, so bit-cast.
__device__ __forceinline__ float lane_bcast(float x, int k) {
  return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), k));
}
// Wave-wide max, returned wave-uniform: running max inside rows of 16 lanes by DPP shifts, then
// the two row broadcasts (gfx9 DPP), so that lane 63 holds the result.  Lanes without a source
// lane keep their own value.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_or_self(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(__float_as_uint(x), __float_as_uint(x), CTRL, ROWS, 0xF, false));
}
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_or_self<0x111, 0xF>(x));  // row_shr:1
  x = fmaxf(x, dpp_or_self<0x112, 0xF>(x));  // row_shr:2
  x = fmaxf(x, dpp_or_self<0x114, 0xF>(x));  // row_shr:4
  x = fmaxf(x, dpp_or_self<0x118, 0xF>(x));  // row_shr:8
  x = fmaxf(x, dpp_or_self<0x142, 0xA>(x));  // row_bcast:15 into rows 1 and 3
  x = fmaxf(x, dpp_or_self<0x143, 0xC>(x));  // row_bcast:31 into rows 2 and 3
  return lane_bcast(x, 63);
}

// One wave per 32-channel slice of an output row (a (sequence, head) of a decode batch, or a
// (token, head) of a key-split prefill).  The kernel is nothing but a chain of memory round trips,
// so it is built to be one trip long and to spread over many CUs: eight lanes x 16 bytes cover the
// slice of one split, a load instruction therefore covers eight splits, and NB of them (up to 256
// splits; NB is picked by the host from the split count) plus the matching (m, l) pairs are
// requested before any weight is known.  The loads are unconditional (indices past the end are
// clamped and their weights forced to 0): behind a branch each would wait for the one before.  Every split of
// the row holds a partial, real or empty (m = -inf; its o holds stale bytes that are only ever
// selected away, never multiplied by 0), so nothing depends on sequence lengths.  Lane group g
// accumulates the splits g, g + 8, g + 16, ... in that order and the eight groups are then added in
// a fixed butterfly, so the result does not depend on timing.  A row with no keys at all (every
// m = -inf) is written as zeros.
template <int D, int NB, int SPW>
__global__ __launch_bounds__(64) void combine_kernel(const float *__restrict__ part_o,
                                                     const float *__restrict__ part_ml,
                                                     char *__restrict__ out, int nsplit,
                                                     const int32_t *__restrict__ cu_q, int batch, int Hq, int route_cap) {
  // SPW = slices per wave: 1, or all D / 32 slices of the row when there are so many rows that
  // the launch would otherwise be tens of thousands of waves that each wait one round trip for
  // half a KiB (the weights are then computed once per row instead of once per slice).
  constexpr int SL = D / 32;  // slices per row
  static_assert(SPW == 1 || SPW == SL, "a wave takes one slice or the whole row");
  const long row = SPW == 1 ? blockIdx.x / SL : blockIdx.x;  // row of the partials
  const int sl0 = SPW == 1 ? (int)(blockIdx.x - row * SL) : 0;
  const int lane = threadIdx.x;
  const int g = lane >> 3, ch = sl0 * 32 + (lane & 7) * 4;
  // Rows of a varlen batch: only those of this call's sequences are written (a call on a
  // sub-range of a batch's sequences must leave the other rows of `out` alone).  Requested with
  // everything else, looked at only before the store.
  long row_lo = 0, row_hi = 0x7fffffffffffffffL, orow = row;
  if (route_cap > 0) {
    // Mixed batch: the partials are indexed [sequence][route_cap tokens][head]; the output row of
    // (sequence, token) follows from the sequence's first query token, and only sequences with at
    // most route_cap query tokens have partials at all.
    const int seq = (int)(row / ((long)route_cap * Hq));
    const int rem = (int)(row - (long)seq * route_cap * Hq);
    const int t = rem / Hq, head = rem - t * Hq;
    const int q0 = cu_q[seq], qn = cu_q[seq + 1] - q0;
    orow = (long)(q0 + t) * Hq + head;
    if (t >= qn || qn > route_cap) row_hi = -1;  // no such row: nothing is stored
  } else if (cu_q != nullptr) {
    row_lo = (long)cu_q[0] * Hq;
    row_hi = (long)cu_q[batch] * Hq;
  }
  char *dst = out + (orow * D + ch) * 2;  // slice p of the wave: + 64 p bytes
  if (part_o == nullptr) {  // every sequence of the batch is empty
#pragma unroll
    for (int p = 0; p < SPW; ++p)
      if (g == 0) *reinterpret_cast<bf16x4 *>(dst + 64 * p) = __builtin_convertvector((f32x4){0.f, 0.f, 0.f, 0.f}, bf16x4);
    return;
  }
  const f32x2 *ml = reinterpret_cast<const f32x2 *>(part_ml) + row * nsplit;
  const float *po = part_o + row * nsplit * D + ch;
  f32x4 acc[SPW];
#pragma unroll
  for (int p = 0; p < SPW; ++p) acc[p] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float den = 0.f, M = -INFINITY;
  for (int base = 0; base < nsplit; base += 8 * NB) {
    f32x2 w[NB];
    f32x4 v[SPW][NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int sc = min(base + 8 * u + g, nsplit - 1);  // past the end: the last split again, weight forced to 0
      w[u] = ml[sc];
#pragma unroll
      for (int p = 0; p < SPW; ++p) v[p][u] = *reinterpret_cast<const f32x4 *>(po + (long)sc * D + 32 * p);
    }
    // Everything above is in flight before anything below waits for it; the code below has no
    // branches either (given one, the compiler moves the row loads behind it, i.e. behind the wait
    // for the (m, l) pairs: a second round trip).
    __builtin_amdgcn_sched_barrier(0);
    float mb = -INFINITY;
#pragma unroll
    for (int u = 0; u < NB; ++u) mb = fmaxf(mb, base + 8 * u + g < nsplit ? w[u][0] : -INFINITY);
    const float Mn = fmaxf(M, wave_max(mb));                               // still -inf: only empty splits so far
    const float alpha = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M - Mn);  // rescale of what has been accumulated
#pragma unroll
    for (int p = 0; p < SPW; ++p) acc[p] *= alpha;
    den *= alpha;
    M = Mn;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const bool live = base + 8 * u + g < nsplit && w[u][0] != -INFINITY;  // not past the end, not an empty split
      const float f = live ? __builtin_amdgcn_exp2f(w[u][0] - M) : 0.f;
      den += live ? f * w[u][1] : 0.f;
#pragma unroll
      for (int p = 0; p < SPW; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[p][j] += live ? f * v[p][u][j] : 0.f;
    }
  }
  // the eight lane groups hold disjoint sets of splits of the same channels
#pragma unroll
  for (int o = 8; o <= 32; o <<= 1) {
    den += __shfl_xor(den, o);
#pragma unroll
    for (int p = 0; p < SPW; ++p)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[p][j] += __shfl_xor(acc[p][j], o);
  }
  if (g != 0 || orow < row_lo || orow >= row_hi) return;
  const float inv = M == -INFINITY ? 0.f : 1.0f / den;  // a row without keys: zeros
#pragma unroll
  for (int p = 0; p < SPW; ++p)
    *reinterpret_cast<bf16x4 *>(dst + 64 * p) =
        __builtin_convertvector(M == -INFINITY ? (f32x4){0.f, 0.f, 0.f, 0.f} : acc[p] * inv, bf16x4);
}

static thread_local int g_combine_rows_per_wave = 0;  // tuning hook: 0 heuristic, 1 one slice per wave, 2 whole rows
void set_combine_form(int form) { g_combine_rows_per_wave = form; }

int launch_combine(const float *part_o, const float *part_ml, void *out, long rows, int nsplit, int head_dim,
                   hipStream_t stream, const int32_t *cu_q, int batch, int num_q_heads, int route_cap) {
  if (rows <= 0) return SP_OK;
  const int nb = nsplit <= 32 ? 4 : nsplit <= 64 ? 8 : nsplit <= 128 ? 16 : 32;  // >= ceil(nsplit / 8) up to 256 splits
  const int sl = head_dim / 32;
  // whole rows per wave once one slice per wave would be more than 16 waves per CU (and the
  // loads of a whole row still fit the registers)
  const bool whole = nb <= 8 && (g_combine_rows_per_wave == 0 ? rows * sl > 4096 : g_combine_rows_per_wave == 2);
  const long blocks = whole ? rows : rows * sl;
  if (blocks > 0x7fffffffL) return fail(SP_ERR_BAD_SHAPE, "combine: %ld rows exceed the grid limit", rows);
  const dim3 grid((unsigned)blocks);
  char *o = (char *)out;
#define SP_COMBINE(D_, NB_, SPW_) \
  hipLaunchKernelGGL((combine_kernel<D_, NB_, SPW_>), grid, dim3(64), 0, stream, part_o, part_ml, o, nsplit, cu_q, batch, \
                     num_q_heads, route_cap)
  if (head_dim == 128) {
    if (whole && nb == 4) SP_COMBINE(128, 4, 4);
    else if (whole) SP_COMBINE(128, 8, 4);
    else if (nb == 4) SP_COMBINE(128, 4, 1);
    else if (nb == 8) SP_COMBINE(128, 8, 1);
    else if (nb == 16) SP_COMBINE(128, 16, 1);
    else SP_COMBINE(128, 32, 1);
  } else {
    if (whole && nb == 4) SP_COMBINE(64, 4, 2);
    else if (whole) SP_COMBINE(64, 8, 2);
    else if (nb == 4) SP_COMBINE(64, 4, 1);
    else if (nb == 8) SP_COMBINE(64, 8, 1);
    else if (nb == 16) SP_COMBINE(64, 16, 1);
    else SP_COMBINE(64, 32, 1);
  }
#undef SP_COMBINE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "combine launch: %s", hipGetErrorString(e));
  return SP_OK;
}

template <int D, int NB, bool APPEND, bool MQ = false, int NT = 1, bool FUSE = false>
static int launch_split(const DecodeArgs &a, int batch, hipStream_t stream) {
  static bool attr_set = false;  // benign if two threads race
  constexpr int smem = (NB == 1 ? 3 : 2 * NB) * 32 * D * 2;  // NB = 1: two K blocks and one V block
  auto fn = decode_split_kernel<D, NB, APPEND, MQ, NT, FUSE>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return fail(SP_ERR_HIP, "decode smem attribute: %s", hipGetErrorString(e));
    attr_set = true;
  }
  hipLaunchKernelGGL(fn, dim3(a.nsplit, (unsigned)(batch * a.n_hgroups)), dim3(64), smem, stream, a);
  return SP_OK;
}

// Arrival counters of the fused combine: a device array of the library (zero at load, left zero by
// every launch).  Each launch takes its own run of counters from a ring, so launches that overlap
// (other streams, other threads) do not share any; a launch recorded in a HIP graph keeps the run it
// was captured with.  As with every file-scope device variable, the array's name is only a
// host-side handle: its device address is looked up once per device.
constexpr int kArriveSlots = 1 << 18;
constexpr int kArriveRing = kArriveSlots - 65536;  // a launch needs at most 65535 counters
static __device__ int32_t g_arrive[kArriveSlots];
constexpr int kMaxDevices = 64;
static int32_t *g_arrive_ptr[kMaxDevices];
static std::mutex g_symbol_mu;
static std::atomic<unsigned> g_arrive_next{0};
static thread_local int g_fuse_mode = 0;  // tuning hook: 0 built-in choice (separate combine kernel), 1 the same, 2 fused where possible
void set_decode_fuse(int mode) { g_fuse_mode = mode; }

static int arrive_counters(int n, int32_t **ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(SP_ERR_UNSUPPORTED, "device ordinal %d (at most %d devices)", dev, kMaxDevices);
  {
    std::lock_guard<std::mutex> lock(g_symbol_mu);
    if (!g_arrive_ptr[dev]) {
      void *p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_arrive));
      if (e != hipSuccess || !p)
        return fail(SP_ERR_HIP, "hipGetSymbolAddress(arrival counters): %s", e != hipSuccess ? hipGetErrorString(e) : "null address");
      g_arrive_ptr[dev] = (int32_t *)p;
    }
  }
  *ptr = g_arrive_ptr[dev] + g_arrive_next.fetch_add((unsigned)n) % kArriveRing;
  return SP_OK;
}

template <int D>
static int launch_decode_d(DecodeArgs &a, char *out, int batch, hipStream_t stream) {
  long gy = (long)batch * a.n_hgroups;
  if (gy > 65535) return fail(SP_ERR_BAD_SHAPE, "sp_attn_decode: batch * head groups = %ld exceeds 65535", gy);
  const int ring = g_ring_override > 0 ? g_ring_override : 2;  // deeper rings and the 24 KiB form time the same or worse
  // One launch instead of two (combine by the last-arriving wave, up to 32 splits): only on request,
  // it measured three times slower than two launches (see arrive_and_merge).
  const bool fuse = a.nsplit <= 32 && ring == 2 && g_fuse_mode == 2;
  int rc;
  if (fuse) {
    if (int e = arrive_counters((int)gy, &a.arrive)) return e;
    a.out = out;
    rc = a.k_new ? launch_split<D, 2, true, false, 1, true>(a, batch, stream)
                 : launch_split<D, 2, false, false, 1, true>(a, batch, stream);
    if (rc != SP_OK) return rc;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SP_ERR_HIP, "decode launch: %s", hipGetErrorString(e));
    return SP_OK;
  }
  if (a.k_new) rc = launch_split<D, 2, true>(a, batch, stream);  // fused step: the measured-best ring only
  else rc = ring == 1 ? launch_split<D, 1, false>(a, batch, stream)
          : ring == 2 ? launch_split<D, 2, false>(a, batch, stream)
          : ring == 3 ? launch_split<D, 3, false>(a, batch, stream)
                      : launch_split<D, 4, false>(a, batch, stream);
  if (rc != SP_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "decode split launch: %s", hipGetErrorString(e));
  return launch_combine(a.part_o, a.part_ml, out, (long)batch * a.Hq, a.nsplit, D, stream);
}

// Head-group geometry shared by the single-token and the short-chunk launches.
static void set_head_groups(DecodeArgs &a, int num_q_heads, int num_kv_heads) {
  a.Hq = num_q_heads;
  a.Hkv = num_kv_heads;
  a.group = num_q_heads / num_kv_heads;
  a.geff = a.group < 32 ? a.group : 32;
  if (a.group % a.geff != 0) a.geff = 1;  // odd large groups: one head per tile
  a.n_hgroups = num_q_heads / a.geff;
  a.q_cap = 32 / a.geff;
}

// ---- short query chunks (sp_attn_prefill with a few tokens per sequence) on the split kernel
// A chunk qualifies when its tokens x the heads of a tile fit one 32-column tile of a wave, or
// two where that measured faster than the prefill kernel: with at most four heads per KV head
// (the prefill kernel then fills a quarter of its columns or less) and on small batches (which
// leave the prefill kernel's workgroups few and long).  Further tiles in further waves re-read
// the keys once per wave and measured slower than the prefill kernel.  Returns the number of
// tiles, 0 if the shape does not qualify.
static int multi_shape(int batch, int max_q_len, int num_q_heads, int num_kv_heads, DecodeArgs *a) {
  set_head_groups(*a, num_q_heads, num_kv_heads);
  if (max_q_len <= 0 || max_q_len > 2 * a->q_cap) return 0;
  if (max_q_len <= a->q_cap) return 1;
  return a->geff <= 4 || (long)batch * a->n_hgroups <= 32 ? 2 : 0;
}

size_t decode_multi_workspace_bytes(int batch, int total_q, int max_q_len, int max_kv_len, int num_q_heads,
                                    int num_kv_heads, int head_dim) {
  DecodeArgs a;
  if (max_kv_len <= 0 || total_q <= 0 || multi_shape(batch, max_q_len, num_q_heads, num_kv_heads, &a) == 0) return 0;
  if ((long)batch * a.n_hgroups > 65535) return 0;
  const int chunk = pick_chunk(batch, num_q_heads, max_kv_len, max_q_len);
  const size_t nsplit = (size_t)(max_kv_len + chunk - 1) / chunk;
  return (size_t)total_q * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

// Mixed batches (sequences with a few query tokens next to sequences with long chunks, the usual
// step of a continuous-batching scheduler): the short ones are served by the split kernel, which
// skips the others, with partials indexed [sequence][cap tokens][head].  cap = the tokens one
// column tile holds; 0 if the head configuration has no such form.
int decode_route_cap(int num_q_heads, int num_kv_heads) {
  DecodeArgs a;
  set_head_groups(a, num_q_heads, num_kv_heads);
  return a.q_cap;
}

size_t decode_routed_workspace_bytes(int batch, int max_kv_len, int num_q_heads, int num_kv_heads, int head_dim) {
  DecodeArgs a;
  set_head_groups(a, num_q_heads, num_kv_heads);
  if (max_kv_len <= 0 || batch <= 0 || (long)batch * a.n_hgroups > 65535) return 0;
  const int chunk = pick_chunk(batch, num_q_heads, max_kv_len, a.q_cap);
  const size_t nsplit = (size_t)(max_kv_len + chunk - 1) / chunk;
  return (size_t)batch * a.q_cap * num_q_heads * nsplit * (head_dim + 2) * sizeof(float);
}

// Returns SP_OK after launching, or 1 when the shape or the workspace does not qualify (the caller
// then runs the general prefill kernel).  routed: serve only the sequences with at most
// decode_route_cap query tokens (the caller's other kernel serves the rest).
int launch_decode_multi(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                        const int32_t *cu_q,
                        const int32_t *ctx_lens, const int32_t *block_table, int batch, int max_pages,
                        int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                        void *workspace, size_t workspace_bytes, hipStream_t stream, bool routed) {
  DecodeArgs a;
  int tiles;
  size_t need;
  long prows;
  if (routed) {
    need = decode_routed_workspace_bytes(batch, max_kv_len, num_q_heads, c.num_kv_heads, c.head_dim);
    set_head_groups(a, num_q_heads, c.num_kv_heads);
    tiles = 1;
    a.route_cap = a.q_cap;
    max_q_len = a.q_cap;
    prows = (long)batch * a.q_cap * num_q_heads;
  } else {
    need = decode_multi_workspace_bytes(batch, total_q, max_q_len, max_kv_len, num_q_heads, c.num_kv_heads, c.head_dim);
    tiles = multi_shape(batch, max_q_len, num_q_heads, c.num_kv_heads, &a);
    a.route_cap = 0;
    prows = (long)total_q * num_q_heads;
  }
  if (need == 0 || !workspace || workspace_bytes < need) return 1;
  a.k_pages = (const char *)c.k_pages;
  a.v_pages = (const char *)c.v_pages;
  a.k_new = (const char *)k_new;  // both NULL: the chunk's rows are in the cache already
  a.v_new = (const char *)v_new;
  a.q = (const char *)q;
  a.seq_lens = nullptr;
  a.arrive = nullptr;
  a.out = nullptr;
  a.cu_q = cu_q;
  a.ctx_lens = ctx_lens;
  a.block_table = block_table;
  a.max_pages = max_pages;
  a.num_pages = c.num_pages;
  a.sl2e = scale * 1.44269504088896340736f;
  a.tau = 8.0f / a.sl2e;
  a.chunk = pick_chunk(batch, num_q_heads, max_kv_len, max_q_len);
  a.nsplit = (max_kv_len + a.chunk - 1) / a.chunk;
  a.part_o = (float *)workspace;
  a.part_ml = a.part_o + (size_t)prows * a.nsplit * c.head_dim;
  int rc;
  if (k_new) {  // fused append of the chunk's rows
    if (tiles == 1)
      rc = c.head_dim == 128 ? launch_split<128, 2, true, true>(a, batch, stream)
                             : launch_split<64, 2, true, true>(a, batch, stream);
    else
      rc = c.head_dim == 128 ? launch_split<128, 2, true, true, 2>(a, batch, stream)
                             : launch_split<64, 2, true, true, 2>(a, batch, stream);
  } else if (tiles == 1) {
    rc = c.head_dim == 128 ? launch_split<128, 2, false, true>(a, batch, stream)
                           : launch_split<64, 2, false, true>(a, batch, stream);
  } else {
    rc = c.head_dim == 128 ? launch_split<128, 2, false, true, 2>(a, batch, stream)
                           : launch_split<64, 2, false, true, 2>(a, batch, stream);
  }
  if (rc != SP_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "short-chunk split launch: %s", hipGetErrorString(e));
  return launch_combine(a.part_o, a.part_ml, out, prows, a.nsplit, c.head_dim, stream, cu_q, batch, num_q_heads, a.route_cap);
}

int launch_decode(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                  const int32_t *seq_lens, const int32_t *block_table, int batch, int max_pages,
                  int max_seq_len, int num_q_heads, float scale, void *workspace, size_t workspace_bytes,
                  hipStream_t stream) {
  (void)workspace_bytes;
  DecodeArgs a;
  a.k_pages = (const char *)c.k_pages;
  a.v_pages = (const char *)c.v_pages;
  a.k_new = (const char *)k_new;  // both NULL: the rows are in the cache already
  a.v_new = (const char *)v_new;
  a.q = (const char *)q;
  a.seq_lens = seq_lens;
  a.arrive = nullptr;
  a.out = nullptr;
  a.route_cap = 0;
  a.cu_q = a.ctx_lens = nullptr;
  a.block_table = block_table;
  a.max_pages = max_pages;
  a.num_pages = c.num_pages;
  set_head_groups(a, num_q_heads, c.num_kv_heads);
  a.sl2e = scale * 1.44269504088896340736f;
  a.tau = 8.0f / a.sl2e;
  if (max_seq_len <= 0) {
    // every sequence is empty: the combine kernel alone writes the zero rows
    return launch_combine(nullptr, nullptr, out, (long)batch * num_q_heads, 1, c.head_dim, stream);
  }
  a.chunk = pick_chunk(batch, num_q_heads, max_seq_len);
  a.nsplit = (max_seq_len + a.chunk - 1) / a.chunk;
  a.part_o = (float *)workspace;
  a.part_ml = a.part_o + (size_t)batch * num_q_heads * a.nsplit * c.head_dim;
  if (c.head_dim == 128) return launch_decode_d<128>(a, (char *)out, batch, stream);
  return launch_decode_d<64>(a, (char *)out, batch, stream);
}

// ---- sp_attn_decode_static: the same decode for callers that cannot hand over a workspace
// (nor let anyone allocate one): the per-split partials go to a file-scope device array.  The
// array's name is only a host-side handle; its device address is asked for once per device, with
// that device current, and kept.  Nothing in it has to start at zero (every partial slot is
// written by the launch that reads it), so no clearing is needed between calls.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, 0 = not asked yet

static int static_scratch(void **ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SP_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(SP_ERR_UNSUPPORTED, "device ordinal %d (at most %d devices)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_symbol_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(SP_ERR_HIP, "hipGetSymbolAddress(scratch): %s", e != hipSuccess ? hipGetErrorString(e) : "null address");
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return SP_OK;
}

size_t decode_static_scratch_bytes() { return kStaticScratchBytes; }

int launch_decode_static(const sp_cache_desc &c, const void *q, void *out, const int32_t *seq_lens,
                         const int32_t *block_table, int batch, int max_pages, int max_seq_len, int num_q_heads,
                         float scale, hipStream_t stream) {
  const size_t need = decode_workspace_bytes(batch, max_seq_len, num_q_heads, c.head_dim);
  if (need > kStaticScratchBytes)
    return fail(SP_ERR_WORKSPACE, "sp_attn_decode_static: this shape needs %zu bytes of partials, the static scratch holds %zu",
                need, kStaticScratchBytes);
  void *ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  return launch_decode(c, nullptr, nullptr, q, out, seq_lens, block_table, batch, max_pages, max_seq_len, num_q_heads,
                       scale, ws, kStaticScratchBytes, stream);
}

}  // namespace sp
