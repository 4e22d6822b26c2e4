// Causal GQA flash attention over the paged KV cache for packed varlen query chunks
// (sp_attn_prefill): the attention each GPU runs on its head shard in the sequence-parallel
// mode after the sequence->head exchange, and for chunked prefill against a cached prefix.
// Per the paper's section "Introducing Shift Parallelism" this computation and its data
// mapping are the same in both parallel modes; only the query count per sequence differs.
//
// Decomposition.  One workgroup (8 waves) owns a tile of 256 query COLUMNS of one
// (sequence, KV head).  The G = Hq/Hkv query heads that share the KV head are stacked into the
// column dimension (column = token * G + head), so a K/V tile staged in LDS is reused by all
// G heads and all columns of a wave have nearly the same causal bound.  Each wave owns 32
// columns; the workgroup walks the visible keys in tiles of KVT tokens (KVT/16 pages, looked
// up in the block table), double-buffered in LDS.
//
// Bound: bf16 MFMA (4 * head_dim flops per visible (query, key) pair per head).  K/V HBM
// traffic is ~1/(8*columns) of that in bytes and is served mostly from L2.  Next to the matrix
// pipe the kernel keeps the VALU (softmax: 3.5 instructions per score, the exponential at half
// rate) and LDS (every MFMA takes one 1 KiB operand from it) busy at the same time.  Measured on
// a 32 k-token prefill, a tile max in every tile (a reduction plus a cross-lane step in front of
// every exponential) costs a quarter more cycles, and so do VALU instructions between the MFMAs
// of a matrix phase, while one plain instruction per score more or less in the softmax phase
// changes nothing at head_dim 128: so the softmax is a single pass without a tile max and the
// matrix phases carry no address arithmetic.  The matrix pipe is then busy in about 85 % of the
// cycles a CU is busy, and what limits the kernel beyond that is the clock the chip grants under
// this load (it is power-limited from the first tile on).
#include <type_traits>

#include "attn_tile.h"

namespace sp {

// Scheduling pattern of a software-pipelined MFMA sequence of N operands starting at fused
// index I0 (indices below NPV are V^T operands = 2 LDS reads, the rest K operands = 1 read):
// PFD operand reads up front, then "read operand i+PFD, MFMA i".  The group sizes must be
// compile-time constants, hence the recursion.
template <int I, int N, int I0, int NPV, int PFD>
__device__ __forceinline__ void sgb_prologue() {
  if constexpr (I < PFD && I < N) {
    if constexpr (I0 + I < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    sgb_prologue<I + 1, N, I0, NPV, PFD>();
  }
}
template <int I, int N, int I0, int NPV, int PFD, int VPM, int NE = N>
__device__ __forceinline__ void sgb_steady() {  // MFMAs [I, NE) of a sequence of N
  if constexpr (I < NE) {
    if constexpr (I + PFD < N) {
      if constexpr (I0 + I + PFD < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    // VPM plain VALU instructions ride behind every PV MFMA (the row sums of the weights it multiplies)
    if constexpr (VPM > 0 && I0 + I < NPV) __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
    sgb_steady<I + 1, N, I0, NPV, PFD, VPM, NE>();
  }
}

// Measurement switches (compile-time, all off in the product build; the profiles record what each
// costs): -DSP_PREFILL_ALWAYS_FULL computes the tile max in every tile (the full softmax pass
// everywhere); -DSP_PREFILL_SUM_DOT2 sums the bf16-rounded weight pairs with the dot-product
// instruction and -DSP_PREFILL_SUM_MFMA with 4x4x4 MFMAs against an all-ones operand, instead of
// adding the fp32 weights (both go through the matrix pipe, where they queue behind the other
// wave's 32-cycle MFMAs: a third more cycles for the whole kernel); -DSP_PREFILL_SUM_IN_MATRIX_PHASE
// moves the row sum out of the softmax phase, behind the PV MFMAs of the next matrix phase (unpack
// the rounded weights by shift / mask, add: four plain VALU instructions per MFMA, which a lone
// wave hides behind its MFMAs in an issue probe — in this kernel they cost 13 % more time);
// -DSP_PREFILL_PRIO raises the wave priority during the matrix phases; -DSP_PREFILL_QSCALED folds
// scale * log2(e) into the resident Q operand and anchors the running max at 0 where the first
// tile allows it, so that the common softmax pass is exp2, add and half a convert per score (2.5
// VALU instructions instead of 3.5) — no change in time at head_dim 128, 9 % faster at head_dim
// 64, at the price of a score error that grows with the score; -DSP_PREFILL_BARRIER_IN_SEQ puts the
// second group's barrier before the last four MFMAs of its matrix phase, so that the first
// group's operand reads after the barrier run behind them — no change in time either.
// -DSP_PREFILL_TRACE makes launches that do not use the workspace otherwise (no key-range pieces,
// no routed short sequences) write a timeline into it: per workgroup the 100 MHz wall clock at its
// start, after the prologue's barrier, at the end of either wave group's tile loop and at its end,
// its tile count and the CU it ran on, and for every eighth tile period of the first group the
// wall clock and the shader clock (paper_2507_11830_amd/trace_prefill.py reads it).
#ifdef SP_PREFILL_TRACE
constexpr int kTraceWgs = 8192, kTraceRec = 8, kTracePer = 64;  // workgroups covered, longs per record, period stamps
constexpr size_t kTraceBytes = (size_t)kTraceWgs * (kTraceRec + 2 * kTracePer) * sizeof(long);
#define SP_TRACE_STAMP(slot, tid)                                                  \
  do {                                                                             \
    if (trace_rec && threadIdx.x == (tid)) trace_rec[slot] = (long)wall_clock64(); \
  } while (0)
#else
#define SP_TRACE_STAMP(slot, tid)
#endif
#ifdef SP_PREFILL_PRIO
#define SP_MATRIX_PHASE_BEGIN() __builtin_amdgcn_s_setprio(3)
#define SP_MATRIX_PHASE_END() __builtin_amdgcn_s_setprio(0)
#else
#define SP_MATRIX_PHASE_BEGIN()
#define SP_MATRIX_PHASE_END()
#endif
#ifdef SP_PREFILL_ALWAYS_FULL
constexpr bool kAlwaysFullSoftmax = true;
#else
constexpr bool kAlwaysFullSoftmax = false;
#endif
#ifdef SP_PREFILL_BARRIER_IN_SEQ
constexpr bool kBarrierInSeq = true;
#else
constexpr bool kBarrierInSeq = false;
#endif
#ifdef SP_PREFILL_QSCALED
constexpr bool kScaledQSwitch = true;
#else
constexpr bool kScaledQSwitch = false;
#endif

struct PrefillArgs {
  const char *k_pages, *v_pages, *q;
  char *out;
  const int32_t *cu_q, *ctx_lens, *block_table;
  int max_pages, num_pages, Hq, Hkv, gshift, n_hgroups, ntiles_x;
  float sl2e;  // scale * log2(e)
  float tau;   // lazy-rescale threshold in raw score units (8 / sl2e)
  // PART kernels: blockIdx.z of kv_splits workgroups share a query tile's key range and write
  // un-normalised partials [row][kv_splits][D] and (max in log2 units, sum) [row][kv_splits][2]
  float *part_o, *part_ml;
  int kv_splits;
  int batch;
  int total_q;     // host count of query tokens (bounds the number of work items)
  int ranked;      // workgroups take their work items heaviest first (ranked_item below)
  int rank_shift;  // log2 of the weight unit in keys
  int route_cap;   // mixed batches: sequences with at most this many query tokens belong to the split kernel (0: none)
};

// Inclusive prefix sum over the 64 lanes (gfx9 DPP: shifts inside rows of 16, then the two row
// broadcasts); lane 63 ends up with the total.
__device__ __forceinline__ int wave_scan_incl(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false);  // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false);  // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false);  // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false);  // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
  return x;
}
__device__ __forceinline__ int wave_total(int x) { return __builtin_amdgcn_readlane(wave_scan_incl(x), 63); }
// Wave-wide max of non-negative values, wave-uniform (same DPP steps; a lane without a source lane
// contributes 0).
__device__ __forceinline__ int wave_max_i(int x) {
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false));
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false));
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false));
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false));
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));
  x = max(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));
  return __builtin_amdgcn_readlane(x, 63);
}

// Ranked dispatch.  The hardware starts workgroups in linear id order and a CU takes the next one
// when it has room, so the launch is a list schedule and its makespan depends on the list's
// order: longest items first is the classic 4/3 rule, and a chunked-prefill batch whose sequences
// sit on cached prefixes of very different lengths is far from it in (tile, sequence) order (the
// early query tiles of the sequence with the longest prefix are as heavy as anything in the batch
// but would start last).  Here the workgroup with linear id r finds the r-th heaviest (sequence,
// query tile) item by itself: the weight of an item is its number of visible keys in units of
// 2^rank_shift keys (the host picks the unit so that the heaviest item weighs at most 63: finer
// classes would not change the makespan, and every doubling costs a probe), the number of items at
// least as heavy as x is a sum over sequences of a closed form, so a binary search over x and one
// prefix sum over the ties select the item in a few hundred instructions, from the same two
// length arrays every workgroup reads anyway.  Ties are taken sequence by sequence, later tiles first.  One
// sequence per lane and slot: batches of up to 64 * kRankSlots sequences.  The search is a chain
// of dependent cross-lane operations in a single wave (about 0.2 us per probe), which is why the
// probes are few and DPP, not LDS permutes, carries them.
constexpr int kRankSlots = 4;

struct RankedItem {
  int seq, tile;
  int q0, q_len, ctx;  // the sequence's entries of the length arrays, so that nobody has to load them again
};

__device__ __forceinline__ bool ranked_item(const PrefillArgs &a, int tpt_shift, int r, int lane, RankedItem *out) {
  const int tpt = 1 << tpt_shift;
  int c[kRankSlots], q[kRankSlots], nt[kRankSlots], qs[kRankSlots];
  const int nslot = (a.batch + 63) >> 6;  // uniform
#pragma unroll
  for (int u = 0; u < kRankSlots; ++u) {
    const int s = u * 64 + lane;
    c[u] = q[u] = nt[u] = qs[u] = 0;
    if (u < nslot && s < a.batch) {
      const int q0 = a.cu_q[s];
      qs[u] = q0;
      q[u] = max(a.cu_q[s + 1] - q0, 0);
      if (q[u] <= a.route_cap) q[u] = 0;  // served by the split kernel (route_cap = 0: nothing is)
      c[u] = max(a.ctx_lens[s], 0);
      nt[u] = (q[u] + tpt - 1) >> tpt_shift;
    }
  }
  const int wsh = a.rank_shift;
  // first tile of slot u's sequence whose weight is >= x units (nt[u] if none)
  auto first_ge = [&](int u, int x) {
    const int xk = x << wsh;  // keys; x never exceeds the heaviest item's weight + 1
    if (nt[u] == 0 || c[u] + q[u] < xk) return nt[u];
    const int d = max(xk - c[u], 0);
    const int j0 = ((d + tpt - 1) >> tpt_shift) - 1;
    return min(max(j0, 0), nt[u] - 1);
  };
  auto total_ge = [&](int x) {
    int n = 0;
#pragma unroll
    for (int u = 0; u < kRankSlots; ++u)
      if (u < nslot) n += nt[u] - first_ge(u, x);
    return wave_total(n);
  };
  int n_items = 0, wmax = 0;
#pragma unroll
  for (int u = 0; u < kRankSlots; ++u) {
    n_items += nt[u];
    wmax = max(wmax, nt[u] ? (c[u] + q[u]) >> wsh : 0);
  }
  if (r >= wave_total(n_items)) return false;  // more workgroups than items
  wmax = wave_max_i(wmax);
  int lo = 0, hi = wmax + 1, n_hi = 0;  // total_ge(lo) > r >= total_ge(hi) = n_hi
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    const int n = total_ge(mid);
    if (n > r) {
      lo = mid;
    } else {
      hi = mid;
      n_hi = n;
    }
  }
  // the item weighs exactly lo units; it is number k among those, counted in sequence order
  int k = r - n_hi;
  bool found = false;
#pragma unroll
  for (int u = 0; u < kRankSlots; ++u) {
    if (u >= nslot || found) continue;
    const int j0 = first_ge(u, lo);
    const int ties = first_ge(u, lo + 1) - j0;  // this sequence's items of weight lo: tiles j0 .. j0 + ties - 1
    const int incl = wave_scan_incl(ties);
    const int tot = __builtin_amdgcn_readlane(incl, 63);
    if (k < tot) {
      const unsigned long long at = __builtin_amdgcn_ballot_w64(incl > k);
      const int ln = __builtin_ctzll(at);
      const int before = __builtin_amdgcn_readlane(incl - ties, ln);
      out->seq = u * 64 + ln;
      const int t_ln = __builtin_amdgcn_readlane(ties, ln);
      out->tile = __builtin_amdgcn_readlane(j0, ln) + (t_ln - 1 - (k - before));  // the sequence's later (heavier) tiles first
      out->q0 = __builtin_amdgcn_readlane(qs[u], ln);
      out->q_len = __builtin_amdgcn_readlane(q[u], ln);
      out->ctx = __builtin_amdgcn_readlane(c[u], ln);
      found = true;
    } else {
      k -= tot;
    }
  }
  return found;
}

// The waves form two groups of four, one wave of each group per SIMD (waves w and w+4 share a
// SIMD).  Inside every tile period the groups run the same two phases in opposite order: one
// multiplies (PV of the previous tile, then QK^T of the current one) while the other runs its
// softmax on the VALU, then they swap; one workgroup barrier per tile.  Barrier-synchronised
// waves that all do the same phase at the same time leave the matrix pipe idle during every
// softmax and the VALU idle during every MFMA burst.
//
// LDS: K[2] and V[2] tile buffers in the swizzled layout of SwzTile, filled by direct
// global -> LDS loads (no register staging, no LDS write instructions).  The loads for the
// next K tile and the current V tile are issued right after the barrier that frees their
// slots and are waited for right before the next barrier, so each has a full tile period to
// land.  The load instruction is written as inline assembly: issued through the compiler
// builtin, every later LDS read is preceded by a full vmcnt(0) wait, because the compiler
// cannot tell the slot being filled from the slot being read.  M0 (the LDS destination) is
// used by nothing else in this kernel.
//
// The running max is only moved when some column's tile max exceeds it by more than 2^8 in
// the exponent (tau); otherwise weights are taken against the stale max (bounded by 2^8,
// harmless in fp32/bf16) and the O accumulators need no rescale.
//
// SPLIT = false is the arrangement described above: the groups own neighbouring sets of 128
// columns and share every K/V tile (the first group issues all tile loads).  SPLIT = true
// is for small grids, where a few hundred workgroups with a triangular causal profile leave
// most CUs waiting for the one with the longest key range: both groups then own the SAME 128
// columns and take alternate key tiles (group g the tiles 2i + g, each with its own K and V
// stream in its own LDS region), so the critical path of the longest work item halves while
// the ping-pong stays intact; the two running states are merged through LDS at the end like
// the splits of the decode path.
//
// PART = true additionally cuts a query tile's key range into kv_splits contiguous pieces, one
// workgroup each (blockIdx.z), which write un-normalised partials for the combine pass: the way
// out when a batch has few query tokens on long cached prefixes (late chunks of a chunked
// prefill), where one workgroup per query tile would walk thousands of keys alone.  Only
// instantiated together with SPLIT (such launches are small grids).
template <int D, int KVT, int PFD, bool SPLIT, bool PART>
__global__ __launch_bounds__(512, 2) void prefill_kernel(PrefillArgs a) {
  using G = TileGeom<D>;
  using Z = SwzTile<D>;
  constexpr int COLS = SPLIT ? 128 : 256, KB = KVT / 32;
  constexpr int ROWB = D * 2;               // bytes of one K or V row
  constexpr int TBYTES = KVT * ROWB;        // one tile in LDS
  constexpr int REGION = 4 * TBYTES;        // K[2] at 0 and TBYTES, V[2] at 2 and 3 TBYTES
  constexpr int NIW = TBYTES / 1024 / 4;    // 1 KiB load instructions per wave and tile
  static_assert(KVT == 4 * kPage, "each of a group's four waves brings in one page of a tile");
  static_assert((TBYTES & (TBYTES - 1)) == 0, "slot toggling flips one address bit");
  extern __shared__ __align__(16) char smem_raw[];
  lds_char *smem = (lds_char *)smem_raw;
#ifdef SP_PREFILL_TRACE
  const unsigned trace_wg = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  long *trace_rec = !PART && a.part_o && trace_wg < (unsigned)kTraceWgs ? (long *)a.part_o + (size_t)trace_wg * kTraceRec : nullptr;
  long *trace_per = trace_rec ? (long *)a.part_o + (size_t)kTraceWgs * kTraceRec + (size_t)trace_wg * kTracePer : nullptr;
  SP_TRACE_STAMP(0, 0);
#endif

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps branches on it scalar
  const int col = lane & 31, half = lane >> 5;
  const int grp = w >> 2;  // wave-uniform; waves w and w+4 share a SIMD: one wave of each group per SIMD
  const int wq = w & 3;    // wave inside its group
  const int rb = SPLIT ? grp * REGION : 0;  // this group's tile buffers
  // Workgroups are dispatched in blockIdx.x-major order: the longest key ranges of ALL sequences
  // go first, the short ones fill in behind them.
  // Consecutive workgroup ids go round-robin over the 8 XCDs; with the (sequence, head group)
  // index rotated by the tile index, the workgroups of one sequence spread over all XCDs even
  // when the batch size is a multiple of 8 (unrotated, each sequence would sit on one XCD and a
  // batch of unequal lengths would leave most of the chip idle).
  int seq, hg, tile, piece, q0, q_len, ctx;
  const int tpt = COLS >> a.gshift;
  if (a.ranked) {
    // linear id -> (item rank, head group, piece): the pieces and head groups of an item are
    // neighbours in the dispatch order, i.e. they start together and spread over the XCDs
    const unsigned lid = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned per_item = (unsigned)(a.n_hgroups * a.kv_splits);
    const int r = (int)(lid / per_item);
    const int sub = (int)(lid - (unsigned)r * per_item);
    hg = sub / a.kv_splits;
    piece = sub - hg * a.kv_splits;
    RankedItem it;
    if (!ranked_item(a, (SPLIT ? 7 : 8) - a.gshift, r, lane, &it)) return;
    seq = __builtin_amdgcn_readfirstlane(it.seq);
    tile = __builtin_amdgcn_readfirstlane(it.tile);
    q0 = __builtin_amdgcn_readfirstlane(it.q0);
    q_len = __builtin_amdgcn_readfirstlane(it.q_len);
    ctx = __builtin_amdgcn_readfirstlane(it.ctx);
  } else {
    int sh, row;
    if ((gridDim.x & 7) == 0) {
      // A multiple of 8 (sequence, head group) streams: every XCD gets its own streams with ALL their
      // query tiles (workgroup ids go round-robin over the XCDs, so XCD x sees the ids = x mod 8),
      // heaviest tiles first.  The workgroups an XCD runs at any moment then belong to a few
      // streams and sit at neighbouring query tiles, so they walk the same K/V pages nearly in
      // step and the XCD's L2 serves most of their tile loads (rotating streams over the XCDs
      // instead puts about one workgroup per stream on an XCD, and every tile load misses L2).
      const unsigned lid = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
      const unsigned xcd = lid & 7, p = lid >> 3, spx = gridDim.x >> 3;
      row = (int)(p / spx);
      sh = (int)((p - (unsigned)row * spx) * 8 + xcd);
    } else {
      sh = (int)((blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x);
      row = (int)(blockIdx.y + gridDim.y * blockIdx.z);
    }
    seq = sh / a.n_hgroups;
    hg = sh - seq * a.n_hgroups;
    piece = row / (int)gridDim.y;
    tile = a.ntiles_x - 1 - (row - piece * (int)gridDim.y);
    q0 = a.cu_q[seq];
    q_len = a.cu_q[seq + 1] - q0;
    ctx = a.ctx_lens[seq];
    if (q_len <= a.route_cap) return;  // mixed batch: the split kernel serves this sequence
  }
  const int tok0 = tile * tpt;
  if (tok0 >= q_len) return;
  const int kv_end = ctx + min(q_len, tok0 + tpt);
  const int kvh = (hg << a.gshift) / (a.Hq / a.Hkv);
  const int32_t *bt_row = a.block_table + (long)seq * a.max_pages;
  const int gmask = (1 << a.gshift) - 1;

  // ---- this lane's column and the resident Q^T operands
  bf16x8 qreg[G::kDSteps];
  const int wc = SPLIT ? wq : w;  // wave's 32-column block inside the workgroup's columns
  const int C = wc * 32 + col;
  const int token = tok0 + (C >> a.gshift);
  const int head = (hg << a.gshift) | (C & gmask);
  const bool valid = token < q_len;
  const int lim = valid ? ctx + token + 1 : 1;
  const long out_off = ((long)(q0 + token) * a.Hq + head) * (D * 2);
#pragma unroll
  for (int s = 0; s < G::kDSteps; ++s) {
    if (valid) {
      qreg[s] = *reinterpret_cast<const bf16x8 *>(a.q + out_off + 32 * s + 16 * half);
    } else {
      u32x4 z = {0, 0, 0, 0};
      qreg[s] = *reinterpret_cast<bf16x8 *>(&z);
    }
  }
  // Rows with at most kPreciseKeys keys get hi + lo weights (see pv_residual below); the workgroups
  // that hold such rows run their own copy of the tile loop.
  constexpr int kPreciseKeys = 256;
  const bool precise_wg = ctx + tok0 < kPreciseKeys;  // group-uniform
  // The scaled-Q form (measurement switch): 2.5 instead of 3.5 VALU instructions per score.  At
  // head_dim 64, where halving the MFMAs per score leaves the softmax phase longer than the other
  // wave's matrix phase, it is 9 % faster; at head_dim 128 it changes nothing.  It is not the
  // product form at either: Q * scale * log2(e) is rounded to bf16 again, so the error of a score
  // grows with the score (relative 2^-9 per term), which is invisible on unit-variance inputs and
  // several per cent of a weight once scores reach the tens — the product keeps Q's products exact.
  constexpr bool kScaledQ = kScaledQSwitch && !SPLIT && !PART;
  if (kScaledQ && !precise_wg) {
    // Fold scale * log2(e) into the resident Q operand: the scores then leave the MFMAs in the
    // exponent's units and the softmax needs no multiply.  The product is rounded to bf16 again
    // (relative 2^-9 per component, a perturbation of each score far below the rounding of the
    // weights themselves).
#pragma unroll
    for (int s = 0; s < G::kDSteps; ++s) {
      union {
        bf16x8 v;
        uint32_t w[4];
        bf16x2 h[4];
      } u;
      u.v = qreg[s];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(u.w[i] << 16) * a.sl2e;
        const float hi = __uint_as_float(u.w[i] & 0xffff0000u) * a.sl2e;
        u.h[i] = __builtin_convertvector((f32x2){lo, hi}, bf16x2);
      }
      qreg[s] = u.v;
    }
  }
  const int wtok_first = tok0 + ((wc * 32) >> a.gshift);
  const int wtok_last = tok0 + (((wc + 1) * 32 - 1) >> a.gshift);
  const int wlim_min = wtok_last < q_len ? ctx + wtok_first + 1 : 1;

  f32x16 o[G::kDBlocks];
#pragma unroll
  for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  // A column of the second SPLIT group may see only masked keys in its first tiles, or none at
  // all: its running max starts at a large finite value so that "all masked" gives weights
  // exp2(-inf) = 0 instead of exp2(-inf + inf).  Tile 0 always holds a visible key otherwise.
  float m_used = (SPLIT || PART) ? -1e30f : -INFINITY, l = 0.f, l2 = 0.f;  // row sum in two chains
  bool m_zero = false;  // wave-uniform: every column's running max is the anchor 0 (scaled-Q form only)
  f32x16 sacc[KB];
  bf16x8 pop[KB][2];

  // key tiles [t_begin, T) of the query tile's range belong to this workgroup
  const int T_all = (kv_end + KVT - 1) / KVT;
  int t_begin = 0, T = T_all;
  if (PART) {
    const int per = (T_all + a.kv_splits - 1) / a.kv_splits;
    t_begin = piece * per;
    T = min(T_all, t_begin + per);
  }
  const long prow = ((long)(q0 + token) * a.Hq + head) * a.kv_splits + (PART ? piece : 0);  // partial slot
  if (PART && t_begin >= T) {  // nothing left for this piece: an empty partial
    if (valid && half == 0) *reinterpret_cast<f32x2 *>(a.part_ml + prow * 2) = (f32x2){-INFINITY, 0.f};
    return;
  }
  const int ntl = T - t_begin;
  const int Tl = SPLIT ? (ntl - grp + 1) / 2 : ntl;  // tiles this group computes on
  const int P = SPLIT ? (ntl + 1) / 2 : ntl;         // tile periods (= barriers) of the workgroup
  auto gtile = [&](int i) __attribute__((always_inline)) { return t_begin + (SPLIT ? 2 * i + grp : i); };  // local tile number -> key tile of the sequence

  // ---- tile loads, all issued by the first group during its MFMA phase (the one phase that
  // starts right after a barrier AND has issue slots to spare; the same instructions placed in
  // a softmax phase measurably lengthen it).  In SPLIT mode the first group therefore also
  // feeds the second group's private K/V stream.  Wave wq brings in page wq of every tile
  // (16 rows = NIW instructions of 1 KiB): lane l of instruction j fills chunk slot l % 16 of
  // line 4j + l / 16 of that page and fetches whichever global chunk the swizzle assigns to
  // that slot.  Rows past the end of the sequence are redirected to its last valid row (finite
  // data; their weights are masked to zero).  Page ids are wave-uniform and read from the block
  // table one period ahead.
  // Everything a load needs per lane is computed before the loop: the byte offset inside a
  // (page, kv head) block per instruction, for K and for V (their swizzles differ).  Only the
  // page that holds the sequence's last key needs other offsets (rows clamped); a stream reaches
  // it with its last loads and repeats it from then on, so the offsets are switched once, outside
  // the MFMA sequences, when that page comes up.  A VALU instruction in a matrix phase is not
  // free: measured with two waves on a SIMD, the second wave gets about five plain VALU
  // instructions in per 32-cycle MFMA of the first, and the softmax needs nearly all of them.
  constexpr int NSTREAM = SPLIT ? 2 : 1;  // K/V tile streams of the workgroup
  constexpr int NLD = NSTREAM * 2 * NIW;  // load instructions per wave and period
  const int last_kv = kv_end - 1, last_page = last_kv >> 4;
  const int dq = lane >> 4, dslot = lane & 15;
  auto stream_tile = [&](int g, int i) __attribute__((always_inline)) { return t_begin + (SPLIT ? 2 * i + g : i); };  // local tile i of stream g
  auto lane_off = [&](bool is_v, int j, int rip_lim) __attribute__((always_inline)) {  // instruction j of a page load: this lane's source offset
    const int lp = 4 * j + dq;  // line inside the page
    const int cl = dslot ^ (is_v ? Z::gv(lp) : Z::gk(lp));
    const int rip = D == 128 ? lp : 2 * lp + (cl >> 3);
    const int chunk = D == 128 ? cl : (cl & 7);
    return (unsigned)(min(rip, rip_lim) * ROWB + chunk * 16);
  };
  unsigned voff[NSTREAM][2][NIW];  // [stream][K, V][instruction]
#pragma unroll
  for (int g = 0; g < NSTREAM; ++g)
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int j = 0; j < NIW; ++j) voff[g][m][j] = lane_off(m != 0, j, 15);
  // The inline assembly below makes the compiler treat every later load as possibly clobbered,
  // so block-table reads are vector loads; the value stays in a VGPR until the load that needs
  // it is issued one period later, and only then moves to an SGPR.
  auto page_of = [&](int gt) __attribute__((always_inline)) {  // all lanes read the same entry
    return bt_row[min(min(gt, T - 1) * (KVT / kPage) + wq, last_page)];
  };
  struct TileLoad {   // wave-uniform description of one page-sized load (NIW instructions)
    const char *pb;   // start of the (page, kv head) block in the pool
    unsigned dst0;    // LDS byte address of this wave's part of the tile slot
  };
  auto dma_prep = [&](bool is_v, int g, int gt, int pg, int slot) __attribute__((always_inline)) {
    if (min(gt, T - 1) * (KVT / kPage) + wq >= last_page) {  // uniform: the page with the last key, from now on
#pragma unroll
      for (int j = 0; j < NIW; ++j) voff[g][is_v][j] = lane_off(is_v, j, last_kv & 15);
    }
    const unsigned page = (unsigned)min(max(__builtin_amdgcn_readfirstlane(pg), 0), a.num_pages - 1);  // no wild loads on bad metadata
    TileLoad tl;
    tl.pb = (is_v ? a.v_pages : a.k_pages) + ((size_t)page * a.Hkv + kvh) * (kPage * ROWB);
    tl.dst0 = (unsigned)(g * REGION + (is_v ? 2 : 0) * TBYTES + slot * TBYTES + wq * (NIW * 1024));
    return tl;
  };
  auto dma_emit = [&](const TileLoad &tl, unsigned off, int j) __attribute__((always_inline)) {  // instruction j of the load
    const unsigned dst = tl.dst0 + j * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off), "s"(tl.pb));
  };
  using std::false_type;
  using std::integral_constant;
  using std::true_type;
  // The loads of period i, prepared right after the barrier that opens it: for every stream, K
  // of local tile i+1 and V of local tile i go into the slots whose last readers finished
  // before that barrier (K(i+1) into slot (i+1) & 1, V(i) into slot i & 1).  Past a stream's
  // last tile the loads repeat the sequence's last tile into a slot nobody reads.  The NLD
  // instructions are then emitted one at a time, spread over the MFMA sequence: issued back to
  // back by four waves at once they queue up at the CU's one texture address unit, and since a
  // wave issues in order, everything behind them waits too.
  int pg_k[NSTREAM], pg_v[NSTREAM];  // page ids of the next K and V loads (kept in VGPRs)
  TileLoad ld[NSTREAM][2];
  auto issue_prep = [&](int i, auto parc) __attribute__((always_inline)) {  // parc: i & 1 as a compile-time constant
    constexpr int PAR = decltype(parc)::value;
#pragma unroll
    for (int g = 0; g < NSTREAM; ++g) {
      ld[g][0] = dma_prep(false, g, stream_tile(g, i + 1), pg_k[g], 1 - PAR);
      ld[g][1] = dma_prep(true, g, stream_tile(g, i), pg_v[g], PAR);
      pg_v[g] = pg_k[g];
      pg_k[g] = page_of(stream_tile(g, i + 2));
    }
  };
  auto issue_emit = [&](int n) __attribute__((always_inline)) {  // n-th instruction of the period, n < NLD: streams and matrices interleaved
    const int j = n / (2 * NSTREAM), g = (n / 2) % NSTREAM, m = n & 1;
    dma_emit(ld[g][m], voff[g][m][j], j);
  };
  auto wait_loads = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0x0F70); };  // vmcnt(0) only

  // ---- LDS operand addresses of this lane: absolute LDS byte addresses for slot 0 of the K and
  // of the V buffers.  Everything else an operand read adds — the slot (TBYTES), the 32-key block
  // and the 16-key step — is a compile-time constant that goes into the instruction's offset
  // field, so the matrix phases contain no address arithmetic at all; the tile loop is unrolled
  // by two for that, one copy per slot parity.
  const unsigned lds0 = (unsigned)(size_t)smem + (unsigned)rb;
  unsigned kadr[G::kDSteps], vadr[G::kDBlocks];
#pragma unroll
  for (int s = 0; s < G::kDSteps; ++s) kadr[s] = lds0 + Z::template offset<false>(col, 2 * s + half);
  {
    const int n = lane & 15, dg = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
      vadr[db] = lds0 + 2 * TBYTES + Z::template offset<true>(4 * half + (n >> 2), 4 * db + 2 * dg + ((n & 3) >> 1)) +
                 8 * (n & 1);
  }
  static_assert(TBYTES + (KVT - 8) * ROWB < 65536, "operand offsets must fit the 16-bit offset field");

  // ---- the phases of a tile, per wave.  The MFMA phases are written software-pipelined ("read
  // operand i+PFD, MFMA i") and pinned to that issue order with sched_group_barrier, so that LDS
  // reads run a fixed distance ahead of the MFMAs that consume them (left alone, the scheduler
  // places each read right before its use and the matrix pipe waits on LDS latency).
  constexpr int NPV = KB * 2 * G::kDBlocks, NQK = KB * G::kDSteps;
  // Operand i of the fused sequence "PV of one tile, then QK^T of the next": i < NPV is a V^T
  // operand (two transposing reads: key rows 32b + 16ks + 4*half + 0..3 and the same + 8, in the
  // row order the score accumulator dictates) from V slot VS, the rest are K operands (one
  // 16-byte read) from K slot KS.
  auto load_op = [&](int i, int KS, int VS) __attribute__((always_inline)) -> bf16x8 {
    if (i < NPV) {
      int db = i % G::kDBlocks, ks = (i / G::kDBlocks) & 1, b = i / (2 * G::kDBlocks);
      return lds_read_vt((const lds_char *)(size_t)(vadr[db] + (unsigned)(VS * TBYTES + (32 * b + 16 * ks) * ROWB)), ROWB);
    }
    int j = i - NPV;
    int s = j % G::kDSteps, b = j / G::kDSteps;
    return *(const lds_bf16x8 *)(size_t)(kadr[s] + (unsigned)(KS * TBYTES + 32 * b * ROWB));
  };
  // Measurement switch SP_PREFILL_SUM_IN_MATRIX_PHASE: the row sum behind the PV MFMAs (unpack the
  // bf16 weights of 16 / NPV packed registers of P by shift / mask, two chains of adds).
  constexpr int RPM = (KB * 2 * 4) / NPV;  // packed registers of P per PV MFMA
  auto do_mfma = [&](int i, bf16x8 op) __attribute__((always_inline)) {
    if (i < NPV) {
      int db = i % G::kDBlocks, ks = (i / G::kDBlocks) & 1, b = i / (2 * G::kDBlocks);
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op, pop[b][ks], o[db], 0, 0, 0);
#ifdef SP_PREFILL_SUM_IN_MATRIX_PHASE
#pragma unroll
      for (int e = 0; e < RPM; ++e) {
        const int pr = i * RPM + e;  // packed register pr of the tile's 16: pop[pr / 8][(pr / 4) & 1], word pr % 4
        union {
          bf16x8 v;
          uint32_t w[4];
        } u;
        u.v = pop[pr / 8][(pr / 4) & 1];
        l += __uint_as_float(u.w[pr % 4] << 16);
        l2 += __uint_as_float(u.w[pr % 4] & 0xffff0000u);
      }
#endif
    } else {
      int j = i - NPV;
      int s = j % G::kDSteps, b = j / G::kDSteps;
      if (s == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
      }
      sacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op, qreg[s], sacc[b], 0, 0, 0);
    }
  };
  // TAILB: the workgroup barrier sits inside the sequence, before its last PFD MFMAs.  All LDS
  // reads of the sequence are done by then (their operands wait in registers), so the waves on
  // the other side of the barrier may overwrite the slots, and their first operand reads run
  // behind these trailing MFMAs instead of leaving the matrix pipe idle.
  auto mfma_seq = [&](auto I0c, auto I1c, auto stagec, auto ksc, auto vsc, auto tailc) __attribute__((always_inline)) {
    constexpr bool TAILB = decltype(tailc)::value;
    constexpr int I0 = decltype(I0c)::value, I1 = decltype(I1c)::value, N = I1 - I0;
    constexpr int KS = decltype(ksc)::value, VS = decltype(vsc)::value;  // K and V slots read
    constexpr bool STAGE = decltype(stagec)::value;  // emit this period's tile loads along the way
    constexpr int GAP = N >= NLD ? N / NLD : 1, PER = N >= NLD ? 1 : NLD / N;  // loads per MFMA slot
    bf16x8 ops[N];
#pragma unroll
    for (int i = 0; i < PFD && i < N; ++i) ops[i] = load_op(I0 + i, KS, VS);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if (TAILB && i == N - PFD) {
        sgb_prologue<0, N, I0, NPV, PFD>();
        sgb_steady<0, N, I0, NPV, PFD, 0, N - PFD>();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      if (i + PFD < N) ops[i + PFD] = load_op(I0 + i + PFD, KS, VS);
      do_mfma(I0 + i, ops[i]);
      if (STAGE && i % GAP == 0 && i / GAP * PER < NLD) {
#pragma unroll
        for (int e = 0; e < PER; ++e) issue_emit(i / GAP * PER + e);
      }
    }
#ifdef SP_PREFILL_SUM_IN_MATRIX_PHASE
    // the row sums are only read at the very end of the kernel: without a use here the compiler
    // sinks their adds out of the matrix phase into the softmax that follows
    if (I0 < NPV) asm volatile("" : "+v"(l), "+v"(l2));
#endif
    if (!TAILB) {
      sgb_prologue<0, N, I0, NPV, PFD>();
#ifdef SP_PREFILL_SUM_IN_MATRIX_PHASE
      sgb_steady<0, N, I0, NPV, PFD, 4 * RPM>();
#else
      sgb_steady<0, N, I0, NPV, PFD, 0>();
#endif
    }
  };
  using slot0 = integral_constant<int, 0>;
  using slot1 = integral_constant<int, 1>;
  auto qk0 = [&]() __attribute__((always_inline)) {  // QK^T of a stream's first tile (K slot 0); its loads went out in the prologue
    mfma_seq(integral_constant<int, NPV>{}, integral_constant<int, NPV + NQK>{}, false_type{}, slot0{}, slot0{}, false_type{});
  };
  auto pv = [&](auto vsc) __attribute__((always_inline)) {  // PV of the tile in V slot vsc
    mfma_seq(integral_constant<int, 0>{}, integral_constant<int, NPV>{}, false_type{}, slot0{}, vsc, false_type{});
  };
  auto pv_qk = [&](auto stagec, auto parc, auto tailc) __attribute__((always_inline)) {  // period i of parity parc: PV of tile i-1 (V slot 1 - par), QK^T of tile i (K slot par)
    constexpr int PAR = decltype(parc)::value;
    mfma_seq(integral_constant<int, 0>{}, integral_constant<int, NPV + NQK>{}, stagec, parc, integral_constant<int, 1 - PAR>{}, tailc);
  };
  // Softmax of tile t.  The common case (FIRST = false, and the tile's scores stay within 2^8 of
  // the running max) is one pass of 3.5 VALU instructions per score: weight = exp2(score * c -
  // max * c), added to the row sum (two independent chains), rounded to bf16 in pairs.  No tile
  // max is computed: if a score had exceeded the running max by more than the threshold, its
  // weight and hence the lane's tile sum would exceed 2^8, and the wave falls back to the full
  // pass (tile max, lazy rescale of O and l, weights again from the raw scores, which the fast
  // pass leaves untouched).  The first tile always takes the full pass (the running max starts at
  // -inf), which also leaves the fp32 weights in sacc for the residual pass of short rows.
  // (Summing the rounded pairs with the bf16 dot-product instruction instead would be half the
  // additions, but measured it costs a third more cycles for the whole kernel: next to MFMAs that
  // instruction is far from full rate.)
  auto softmax = [&](int t, auto firstc, bool keep_fp32, auto qsc) __attribute__((always_inline)) {
    constexpr bool QS = decltype(qsc)::value;  // scores arrive in the exponent's units (Q was prescaled)
    constexpr bool FIRST = decltype(firstc)::value;  // keep_fp32 (wave-uniform): take the full pass, the residual pass follows
    const int base = gtile(t) * KVT;
    if (base + KVT > wlim_min) {
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int kv = base + 32 * b + 8 * (r >> 2) + 4 * half + (r & 3);
          if (kv >= lim) sacc[b][r] = -INFINITY;
        }
    }
    float lsum = 0.f;
    bool full = FIRST || keep_fp32 || kAlwaysFullSoftmax;
    const float sc = QS ? 1.0f : a.sl2e;
    if (!full) {
      const float msc = m_used * sc;
#ifdef SP_PREFILL_SUM_IN_MATRIX_PHASE
      uint32_t pmax = 0;  // weights are >= 0, so their bit patterns order like their values (and NaN sorts above all)
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          union {
            bf16x2 h[4];
            bf16x8 v;
          } u;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][8 * ks + 2 * i], a.sl2e, -msc));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][8 * ks + 2 * i + 1], a.sl2e, -msc));
            u.h[i] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
            pmax = max(pmax, max(__float_as_uint(p0), __float_as_uint(p1)));  // one v_max3_u32 per pair
          }
          pop[b][ks] = u.v;
        }
      // NaN (a masked score against a running max that is still -inf) must take the full pass too
      full = __builtin_amdgcn_ballot_w64(pmax > 0x43800000u) != 0;  // some weight above 2^8: wave-uniform, rare
#else
      float ls0 = 0.f, ls1 = 0.f;
#ifdef SP_PREFILL_SUM_MFMA
      f32x4 lacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#endif
      if (QS && m_zero) {
        // no running max to subtract: 2.5 VALU instructions per score
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            union {
              bf16x2 h[4];
              bf16x8 v;
            } u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float p0 = __builtin_amdgcn_exp2f(sacc[b][8 * ks + 2 * i]);
              const float p1 = __builtin_amdgcn_exp2f(sacc[b][8 * ks + 2 * i + 1]);
              u.h[i] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
              ls0 += p0;
              ls1 += p1;
            }
            pop[b][ks] = u.v;
          }
      } else
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          union {
            bf16x2 h[4];
            bf16x8 v;
          } u;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][8 * ks + 2 * i], sc, -msc));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][8 * ks + 2 * i + 1], sc, -msc));
            u.h[i] = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
#if defined(SP_PREFILL_SUM_DOT2)
            ls0 = __builtin_amdgcn_fdot2_f32_bf16(u.h[i], (bf16x2){(__bf16)1.0f, (__bf16)1.0f}, ls0, false);
#elif !defined(SP_PREFILL_SUM_MFMA)
            ls0 += p0;
            ls1 += p1;
#endif
          }
          pop[b][ks] = u.v;
#ifdef SP_PREFILL_SUM_MFMA
          {
            // row sums on the matrix pipe: a 4x4x4 MFMA (16 blocks) with an all-ones A operand adds up
            // the four bf16 values each lane holds in B; two of them cover this operand's eight
            union {
              bf16x8 v;
              s16x4 q[2];
            } w;
            w.v = u.v;
            const s16x4 ones4 = {0x3F80, 0x3F80, 0x3F80, 0x3F80};
            lacc[ks] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ones4, w.q[0], lacc[ks], 0, 0, 0);
            lacc[ks] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ones4, w.q[1], lacc[ks], 0, 0, 0);
          }
#endif
        }
#ifdef SP_PREFILL_SUM_MFMA
      lsum = lacc[0][0] + lacc[1][0];
#else
      lsum = ls0 + ls1;
#endif
      // NaN (a masked score against a running max that is still -inf) must take the full pass too
      full = __builtin_amdgcn_ballot_w64(!(lsum <= (QS ? 0x1p40f : 256.0f))) != 0;  // wave-uniform, rare
#endif
    }
    if (full) {
      float mx = sacc[0][0];
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[b][r]);
      mx = fmaxf(mx, other_half(mx));
      if (__builtin_amdgcn_ballot_w64(mx > m_used + (QS ? 8.0f : a.tau)) != 0) {  // wave-uniform
        float m_new = fmaxf(m_used, mx);
        // scaled-Q form: a first max within 2^+-32 anchors the column at 0, and while every column
        // of the wave sits there the fast pass skips the subtraction
        if (QS && FIRST && fabsf(mx) <= 32.0f) m_new = 0.f;
        const float alpha = __builtin_amdgcn_exp2f((m_used - m_new) * sc);
        m_used = m_new;
        if (QS) m_zero = __builtin_amdgcn_ballot_w64(m_used != 0.f) == 0;
        l *= alpha;
        l2 *= alpha;
#pragma unroll
        for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      }
      const float msc = m_used * sc;
      lsum = 0.f;
#pragma unroll
      for (int b = 0; b < KB; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sacc[b][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][r], sc, -msc));
#ifndef SP_PREFILL_SUM_IN_MATRIX_PHASE
          lsum += sacc[b][r];
#endif
        }
        pop[b][0] = pack8(sacc[b], 0);
        pop[b][1] = pack8(sacc[b], 8);
      }
    }
    l += lsum;
  };
  // Rows with at most kPreciseKeys keys take their weights as hi + lo: a second PV pass over the
  // tile with the bf16 residuals of P, so that the rounding of the weights (which only averages
  // out over many keys) stays out of the output tolerance there.  That concerns the first
  // kPreciseKeys / KVT key tiles of the workgroups whose first query sits below position
  // kPreciseKeys.  The pass needs the fp32 weights (the softmax's full pass leaves them in sacc)
  // and V of that tile in LDS: it runs at the start of the following period, before QK^T
  // overwrites sacc.
  auto precise = [&](int i) __attribute__((always_inline)) { return precise_wg && i >= 0 && gtile(i) * KVT < kPreciseKeys; };
  auto pv_residual = [&](auto vsc) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) pop[b][ks] = pack8_residual(sacc[b], 8 * ks, pop[b][ks]);
    pv(vsc);
#pragma unroll
    for (int b = 0; b < KB; ++b)  // back to the rounded weights (cheaper than keeping a copy live)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) pop[b][ks] = pack8(sacc[b], 8 * ks);
  };

  // prologue: K of every stream's first tile must be in LDS before anything is multiplied.  V of
  // that tile and K of the second one are requested in the same round trip (their slots are
  // free), so the first period has no load to wait for: a memory latency per workgroup that
  // small grids cannot hide behind other work.
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < NSTREAM; ++g) {
      const int gt0 = stream_tile(g, 0), gt1 = stream_tile(g, 1);
      const int pg0 = page_of(gt0), pg1 = page_of(gt1);
      TileLoad k0 = dma_prep(false, g, gt0, pg0, 0);
#pragma unroll
      for (int j = 0; j < NIW; ++j) dma_emit(k0, voff[g][0][j], j);
      TileLoad v0 = dma_prep(true, g, gt0, pg0, 0);
#pragma unroll
      for (int j = 0; j < NIW; ++j) dma_emit(v0, voff[g][1][j], j);
      TileLoad k1 = dma_prep(false, g, gt1, pg1, 1);
#pragma unroll
      for (int j = 0; j < NIW; ++j) dma_emit(k1, voff[g][0][j], j);
      pg_k[g] = page_of(stream_tile(g, 2));
      pg_v[g] = pg1;
    }
  }
  wait_loads();
  __syncthreads();
  SP_TRACE_STAMP(1, 0);

  // One barrier per key tile.  Inside a tile period the two groups run the same two phases in
  // OPPOSITE order: the first group multiplies (PV of tile t-1, QK^T of tile t) and then
  // exponentiates tile t; the second group first exponentiates tile t-1 and then multiplies.
  // One wave of each group sits on every SIMD, so the matrix pipe and the VALU are both busy
  // through the whole period, and since nothing forces the phase boundary to line up, a short
  // softmax simply lets the next MFMA phase start early.  Wave priorities are left alone: raising
  // the multiplying wave (or the other one) measured 5 % more cycles for the whole kernel.
  // Buffer hand-off: from period 1 on, K(t+1) and V(t) are requested in the first group's MFMA
  // phase of period t into the slots last read in period t-1, have landed before the barrier
  // that ends period t, and are first read in period t+1.  Periods alternate between two copies
  // of the loop body, one per slot parity.
  // The tile loop exists twice: the few workgroups that hold rows of at most kPreciseKeys keys
  // (at most eight key tiles long) take the copy with the residual passes, everything else the
  // copy without them, whose registers and schedule the rare case then cannot disturb.
  auto tile_loop = [&](auto precc) __attribute__((always_inline)) {
    constexpr bool PREC = decltype(precc)::value;
    if (grp == 0) {  // always has Tl == P >= 1
      qk0();  // the loads of period 0 went out in the prologue
      softmax(0, true_type{}, false, integral_constant<bool, kScaledQ && !PREC>{});
      __syncthreads();
      auto period = [&](int t, auto parc) __attribute__((always_inline)) {
        constexpr int PAR = decltype(parc)::value;
#ifdef SP_PREFILL_TRACE
        if (trace_per && threadIdx.x == 0 && (t & 7) == 0 && t < 8 * kTracePer) {
          trace_per[t >> 3] = (long)wall_clock64();
          trace_per[(size_t)kTraceWgs * kTracePer + (t >> 3)] = (long)clock64();
        }
#endif
        if (PREC && precise(t - 1)) pv_residual(integral_constant<int, 1 - PAR>{});  // V(t-1) became visible at the barrier
        issue_prep(t, parc);
        SP_MATRIX_PHASE_BEGIN();
        pv_qk(true_type{}, parc, false_type{});
        SP_MATRIX_PHASE_END();
        softmax(t, false_type{}, PREC && precise(t), integral_constant<bool, kScaledQ && !PREC>{});
        wait_loads();
        __syncthreads();
      };
      int t = 1;
      for (; t + 1 < Tl; t += 2) {  // single-exit loop over pairs of periods; an odd one out follows it
        period(t, slot1{});
        period(t + 1, slot0{});
      }
      if (t < Tl) {
        period(t, slot1{});
        if (PREC && precise(t)) pv_residual(slot1{});
        pv(slot1{});
      } else {
        if (PREC && precise(t - 1)) pv_residual(slot0{});
        pv(slot0{});
      }
    } else {  // SPLIT: may have one tile less than the first group, or none
      if (Tl > 0) qk0();
      __syncthreads();
      if (Tl > 0) {
        softmax(0, true_type{}, false, integral_constant<bool, kScaledQ && !PREC>{});
        auto period = [&](int t, auto parc) __attribute__((always_inline)) {
          constexpr int PAR = decltype(parc)::value;
          if (PREC && precise(t - 1)) pv_residual(integral_constant<int, 1 - PAR>{});
          SP_MATRIX_PHASE_BEGIN();
          pv_qk(false_type{}, parc, integral_constant<bool, kBarrierInSeq>{});  // the period's barrier is inside
          SP_MATRIX_PHASE_END();
          if (!kBarrierInSeq) __syncthreads();
          softmax(t, false_type{}, PREC && precise(t), integral_constant<bool, kScaledQ && !PREC>{});
        };
        int t = 1;
        for (; t + 1 < Tl; t += 2) {
          period(t, slot1{});
          period(t + 1, slot0{});
        }
        if (t < Tl) {
          period(t, slot1{});
          if (PREC && precise(t)) pv_residual(slot1{});
          pv(slot1{});
        } else {
          if (PREC && precise(t - 1)) pv_residual(slot0{});
          pv(slot0{});
        }
      }
      for (int t = max(Tl, 1); t < P; ++t) __syncthreads();  // keep the barrier count of the first group
    }
  };
  if (precise_wg) tile_loop(true_type{});
  else tile_loop(false_type{});
  SP_TRACE_STAMP(2, 0);
  SP_TRACE_STAMP(3, 256);

  if (SPLIT) {
    // ---- merge the second group's running state into the first group's (same columns, same
    // lane layout: wave w and wave w+4 hold the same (column, channel) positions).
    constexpr int NST = 16 * G::kDBlocks + 2;  // floats of state per lane
    static_assert(256 * NST * 4 <= 2 * REGION, "state must fit the tile buffers");
    lds_float *xch = (lds_float *)smem + wq * 64 + lane;  // [value][wave][lane]
    __syncthreads();  // every wave is done reading tiles
    if (grp == 1) {
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) xch[(16 * db + r) * 256] = o[db][r];
      xch[(NST - 2) * 256] = m_used;
      xch[(NST - 1) * 256] = l + l2;
    }
    __syncthreads();
    if (grp == 1) return;
    const float m_b = xch[(NST - 2) * 256], l_b = xch[(NST - 1) * 256];
    const float m_new = fmaxf(m_used, m_b);  // the first group always saw a key: finite
    const float fa = __builtin_amdgcn_exp2f((m_used - m_new) * a.sl2e);
    const float fb = __builtin_amdgcn_exp2f((m_b - m_new) * a.sl2e);  // 0 if the second group had no tile
    l = (l + l2) * fa + l_b * fb;
    l2 = 0.f;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = o[db][r] * fa + xch[(16 * db + r) * 256] * fb;
    m_used = m_new;  // what l and o now refer to (a partial carries it along)
  }

  l += l2;
  float lt = l + other_half(l);
  if (PART) {  // un-normalised partial for the combine pass
    if (valid) {
      float *po = a.part_o + prow * D;
#pragma unroll
      for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *reinterpret_cast<f32x4 *>(po + 32 * db + 8 * r4 + 4 * half) =
              (f32x4){o[db][4 * r4], o[db][4 * r4 + 1], o[db][4 * r4 + 2], o[db][4 * r4 + 3]};
      if (half == 0) *reinterpret_cast<f32x2 *>(a.part_ml + prow * 2) = (f32x2){m_used * a.sl2e, lt};
    }
    return;
  }
  // ---- normalise and store
  float inv = 1.0f / lt;
  if (valid) {
    char *dst = a.out + out_off;
#pragma unroll
    for (int db = 0; db < G::kDBlocks; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        store4_bf16(dst + (32 * db + 8 * r4 + 4 * half) * 2, o[db][4 * r4] * inv, o[db][4 * r4 + 1] * inv,
                    o[db][4 * r4 + 2] * inv, o[db][4 * r4 + 3] * inv);
  }
#ifdef SP_PREFILL_TRACE
  SP_TRACE_STAMP(4, 0);
  if (trace_rec && threadIdx.x == 0) {
    trace_rec[5] = T_all;
    // HW_ID (wave, SIMD, CU, shader array, shader engine) and XCC_ID of the wave
    trace_rec[6] = (long)__builtin_amdgcn_s_getreg((31 << 11) | 4) | ((long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32);
    trace_rec[7] = ((long)seq << 32) | (unsigned)tile;
  }
#endif
}

// Launch-shape overrides of the calling thread (sp_debug_set_tuning); 0 = built-in heuristic.
static thread_local int g_split_mode = 0;
static thread_local int g_kv_splits = 0;
static thread_local int g_short_chunk_mode = 0;
static thread_local int g_order_mode = 0;
void set_prefill_order(int mode) { g_order_mode = mode; }
void set_prefill_short_chunk(int mode) { g_short_chunk_mode = mode; }
void set_prefill_split(int mode) { g_split_mode = mode; }
void set_prefill_kv_splits(int n) { g_kv_splits = n; }

typedef void (*prefill_fn)(PrefillArgs);

constexpr int kMaxKvSplits = 16;
constexpr long kMaxPartialSlots = 1L << 17;  // (row, split) pairs the workspace is ever sized for

// Largest number of key-range pieces a batch of `rows` (token, head) rows may be cut into.
static int kv_split_cap(long rows) {
  if (rows <= 0) return 1;
  long cap = kMaxPartialSlots / rows;
  return (int)(cap < 1 ? 1 : cap > kMaxKvSplits ? kMaxKvSplits : cap);
}

// Mixed batch?  Decided from the host-side hints alone: chunks too long for the short-chunk path
// exist (max_q_len), and the tokens besides the longest chunk are so few that at least one other
// sequence must be short — those sequences are then routed to the split kernel (which reads a
// long cached prefix once, in pieces, at memory speed) and the rest to the prefill kernel, inside
// the one call.  Returns the token bound of "short" (one column tile of the split kernel), or 0.
static int mixed_route_cap(int batch, int total_q, int max_q_len, int num_q_heads, int num_kv_heads) {
  if (g_short_chunk_mode == 1 || batch < 2) return 0;
  const int cap = decode_route_cap(num_q_heads, num_kv_heads);
  if (cap <= 0 || max_q_len <= cap) return 0;  // no long chunk: the whole batch takes the short-chunk path
  const long rest = (long)total_q - max_q_len;
  if (rest <= 0 || rest >= (long)(batch - 1) * (cap + 1)) return 0;
  return cap;
}

size_t prefill_workspace_bytes(int batch, int total_q_tokens, int max_q_len, int max_kv_len, int num_q_heads,
                               int num_kv_heads, int head_dim) {
  const long rows = (long)total_q_tokens * num_q_heads;
  const int cap = kv_split_cap(rows);
  const size_t pieces = cap >= 2 ? (size_t)rows * cap * (head_dim + 2) * sizeof(float) : 0;
  size_t shortq = g_short_chunk_mode == 1 ? 0
                                          : decode_multi_workspace_bytes(batch, total_q_tokens, max_q_len, max_kv_len,
                                                                         num_q_heads, num_kv_heads, head_dim);
  if (mixed_route_cap(batch, total_q_tokens, max_q_len, num_q_heads, num_kv_heads) > 0)
    shortq = decode_routed_workspace_bytes(batch, max_kv_len, num_q_heads, num_kv_heads, head_dim);
  return pieces > shortq ? pieces : shortq;
}

// Launches one prefill kernel instantiation with `cols` query columns per workgroup.
static int launch_cfg(prefill_fn fn, bool *attr_set, size_t smem, int cols, const PrefillArgs &a0, int batch,
                      int max_q_len, hipStream_t stream) {
  PrefillArgs a = a0;
  int tpt = cols >> a.gshift;
  a.ntiles_x = (max_q_len + tpt - 1) / tpt;
  if (!*attr_set) {  // benign if two threads race
    hipError_t e = hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return fail(SP_ERR_HIP, "prefill smem attribute: %s", hipGetErrorString(e));
    *attr_set = true;
  }
  long gx = (long)batch * a.n_hgroups;
  if (gx > 0x7fffffffL || a.ntiles_x > 65535)
    return fail(SP_ERR_BAD_SHAPE, "sp_attn_prefill: grid %ld x %d exceeds the launch limits", gx, a.ntiles_x);
  dim3 grid((unsigned)gx, (unsigned)a.ntiles_x, (unsigned)a.kv_splits);
  if (a.ranked) {
    // Ranked workgroups take items by linear id, so the launch only needs as many workgroups as
    // there can be items: every sequence has at most q_len / tpt + 1 query tiles.  (The grid of
    // the static order is batch x tiles of the LONGEST chunk; in a ragged batch most of it is
    // empty, and an empty workgroup still holds a CU for a microsecond.)
    const long items = (long)a.total_q / tpt + batch;
    const long wgs = items * a.n_hgroups * a.kv_splits;
    if (wgs > 0x7fffffffL) a.ranked = 0;  // workgroups are numbered in 32 bits
    else grid = dim3((unsigned)wgs, 1, 1);
  }
  hipLaunchKernelGGL(fn, grid, dim3(512), smem, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SP_ERR_HIP, "prefill launch: %s", hipGetErrorString(e));
  return SP_OK;
}

template <int D>
static int launch_prefill_d(const PrefillArgs &a, bool split, int batch, int max_q_len, hipStream_t stream) {
  constexpr int KVT = 64, PFD = 4;
  constexpr size_t smem = 4 * (size_t)KVT * D * 2;  // K[2] V[2], unpadded
  static bool set[3] = {false, false, false};
  // Key ranges are only cut into pieces on small grids, which take the 128-column form anyway;
  // the 256-column form with partial outputs is not instantiated (it would not fit the register
  // budget of two workgroups per CU).
  if (a.kv_splits > 1) return launch_cfg(prefill_kernel<D, KVT, PFD, true, true>, &set[0], 2 * smem, 128, a, batch, max_q_len, stream);
  if (split) return launch_cfg(prefill_kernel<D, KVT, PFD, true, false>, &set[1], 2 * smem, 128, a, batch, max_q_len, stream);
  return launch_cfg(prefill_kernel<D, KVT, PFD, false, false>, &set[2], smem, 256, a, batch, max_q_len, stream);
}

int launch_chunk_step(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                      const int32_t *cu_q, const int32_t *ctx_lens, const int32_t *block_table, int batch,
                      int max_pages, int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                      void *workspace, size_t workspace_bytes, hipStream_t stream) {
  if (g_short_chunk_mode != 1) {
    // short chunks: the decode kernels append the rows themselves
    int rc = launch_decode_multi(c, k_new, v_new, q, out, cu_q, ctx_lens, block_table, batch, max_pages, total_q,
                                 max_q_len, max_kv_len, num_q_heads, scale, workspace, workspace_bytes, stream);
    if (rc != 1) return rc;
  }
  int rc = launch_kv_append(c, k_new, v_new, cu_q, ctx_lens, block_table, batch, max_pages, total_q, stream);
  if (rc != SP_OK) return rc;
  return launch_prefill(c, q, out, cu_q, ctx_lens, block_table, batch, max_pages, total_q, max_q_len, max_kv_len,
                        num_q_heads, scale, workspace, workspace_bytes, stream);
}

int launch_prefill(const sp_cache_desc &c, const void *q, void *out, const int32_t *cu_q,
                   const int32_t *ctx_lens, const int32_t *block_table, int batch, int max_pages,
                   int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                   void *workspace, size_t workspace_bytes, hipStream_t stream) {
  if (g_short_chunk_mode != 1) {
    // Every chunk is a few tokens long: the bandwidth-bound split kernel of the decode path reads
    // each sequence's keys once for all of its query tokens.
    int rc = launch_decode_multi(c, nullptr, nullptr, q, out, cu_q, ctx_lens, block_table, batch, max_pages, total_q, max_q_len,
                                 max_kv_len, num_q_heads, scale, workspace, workspace_bytes, stream);
    if (rc != 1) return rc;
  }
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
  a.tau = 8.0f / a.sl2e;

  // ---- shape of the launch, from host-side counts only.  wg128 estimates the 128-column
  // workgroups that find work (rows / 128 plus half a partial tile per sequence and head group).
  const long rows = (long)total_q * num_q_heads;
  const long wg128 = rows / 128 + ((long)batch * a.n_hgroups + 1) / 2;
  // Up to about one 256-column workgroup per CU: let the two wave groups split the key range of
  // 128 columns instead (halves the critical path of the longest work item; measured faster up
  // to that grid size, slower beyond it because every K/V tile is then staged for half the
  // columns).
  const bool small_grid = g_split_mode == 0 ? wg128 <= 576 : g_split_mode == 2;
  // How many pieces the key range of a query tile is cut into (1 = none): only when even the
  // 128-column workgroups leave most CUs idle and the key ranges are long, and bounded by what
  // the caller's workspace holds.  A piece's partial costs about as much HBM time as 500 keys
  // cost matrix time, so pieces stay around 1500 keys or longer.
  const size_t slot_bytes = (size_t)(c.head_dim + 2) * sizeof(float);
  int kvs = 1;
  if (workspace && rows > 0) {
    if (g_kv_splits > 0) {
      kvs = g_kv_splits;
    } else if (small_grid) {
      const long by_grid = 256 / (wg128 > 0 ? wg128 : 1);
      const long by_len = (long)max_kv_len / 1536;
      kvs = (int)(by_grid < by_len ? by_grid : by_len);
    }
    const int cap = kv_split_cap(rows);
    if (kvs > cap) kvs = cap;
    const size_t fit = workspace_bytes / ((size_t)rows * slot_bytes);
    if ((size_t)kvs > fit) kvs = (int)fit;
    if (kvs < 1) kvs = 1;
  }
  // Mixed batch: short sequences go to the split kernel (launched last, below) when the workspace
  // holds their partials; the prefill kernel then skips them, and its key ranges stay uncut (the
  // longest key range of the batch, which sizes the pieces, belongs to a short sequence as a rule).
  a.route_cap = 0;
  {
    const int cap = mixed_route_cap(batch, total_q, max_q_len, num_q_heads, c.num_kv_heads);
    const size_t need = cap > 0 ? decode_routed_workspace_bytes(batch, max_kv_len, num_q_heads, c.num_kv_heads, c.head_dim) : 0;
    if (need > 0 && workspace && workspace_bytes >= need) {
      a.route_cap = cap;
      if (g_kv_splits == 0) kvs = 1;
    }
  }
  a.kv_splits = kvs;
  // Heaviest-first dispatch when the static (tile, sequence) order is not already that: several
  // sequences with cached prefixes (without prefixes the last query tiles of all sequences are
  // the heaviest items, and they are first in the static order too).
  a.batch = batch;
  a.total_q = total_q;
  const bool can_rank = batch <= 64 * kRankSlots;
  a.ranked = can_rank && (g_order_mode == 0 ? batch >= 2 && max_kv_len > max_q_len : g_order_mode == 2);
  a.rank_shift = 6;
  while (a.rank_shift < 24 && (max_kv_len >> a.rank_shift) > 63) ++a.rank_shift;
  a.part_o = (float *)workspace;
  a.part_ml = a.part_o + (size_t)rows * kvs * c.head_dim;
#ifdef SP_PREFILL_TRACE
  if (kvs == 1 && (a.route_cap > 0 || workspace_bytes < kTraceBytes)) a.part_o = nullptr;  // no room for the timeline
#endif

  const bool split = small_grid || kvs > 1;
  int rc = c.head_dim == 128 ? launch_prefill_d<128>(a, split, batch, max_q_len, stream)
                             : launch_prefill_d<64>(a, split, batch, max_q_len, stream);
  if (rc != SP_OK) return rc;
  if (kvs > 1) {
    rc = launch_combine(a.part_o, a.part_ml, out, rows, kvs, c.head_dim, stream, cu_q, batch, num_q_heads);
    if (rc != SP_OK) return rc;
  }
  if (a.route_cap > 0) {
    // ... and the short sequences of a mixed batch on the split kernel, in the same stream: it runs
    // after the launches above, so it may reuse the workspace, and its rows are its own.
    rc = launch_decode_multi(c, nullptr, nullptr, q, out, cu_q, ctx_lens, block_table, batch, max_pages, total_q, max_q_len,
                             max_kv_len, num_q_heads, scale, workspace, workspace_bytes, stream, true);
    if (rc == 1) return fail(SP_ERR_WORKSPACE, "sp_attn_prefill: workspace too small for the routed short sequences");
  }
  return rc;
}

}  // namespace sp
