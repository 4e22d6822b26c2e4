/*
 * fp64 CPU oracle for causal grouped-query attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared
 * against; the product path never calls it.  It shares no code, header, table or
 * helper with the HIP kernels.
 *
 * What it computes is the plain definition of scaled-dot-product attention for the
 * per-GPU head shard that Shift Parallelism assigns to one device in both of its
 * modes (paper section "Introducing Shift Parallelism", the paragraph on the
 * invariant KV-cache layout and the identical attention computation under TP and SP,
 * and Figure 2).  The paper writes no formula; the reading taken is the standard
 * Llama-3 attention:
 *
 *     s_j = scale * <q, k_j>            j = 0 .. p   (p = absolute query position)
 *     w_j = exp(s_j - max_j s) / sum_j exp(s_j - max_j s)
 *     o   = sum_j w_j v_j,              lse = max_j s + log(sum_j exp(s_j - max))
 *
 * with query head h reading KV head g = h / (Hq / Hkv), and token j of sequence s
 * living in cache slot  block_table[s][j / 16] * 16 + j % 16.
 *
 * All inputs are bf16 bit patterns (uint16); widening bf16 -> fp64 is exact, and every
 * operation after that is fp64.  No blocking, no online softmax, no splitting: two
 * passes over the visible keys, exactly as the definition reads.
 *
 * Pins (tests/test_oracle_pins.py): dense numpy brute force, torch fp64 SDPA, weights
 * summing to one, causal invariance, closed forms (row 0, zero query -> running mean),
 * chunked == monolithic, decode == prefill row, paged == contiguous, GQA map, split
 * log-sum-exp identity, shift invariance, dominating key.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PAGE 16

static double widen(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* Element index of (token slot, kv head g, channel c) in a [num_pages][Hkv][16][d] pool. */
static size_t pool_index(int32_t page, int off, int g, int c, int Hkv, int d) {
  return (((size_t)page * Hkv + g) * PAGE + off) * d + c;
}

/*
 * Cache image builder: writes the new tokens of every sequence into the page pools.
 * Token i of sequence s lands at absolute position ctx_lens[s] + i.  Slots that are not
 * written keep whatever the caller put there (tests use a canary fill).
 * Returns 0, or -1 if a block-table entry is outside [0, num_pages).
 */
int oracle_kv_append(uint16_t *k_pages, uint16_t *v_pages, int num_pages, int Hkv, int d,
                     const uint16_t *k_new, const uint16_t *v_new, const int32_t *cu_new,
                     const int32_t *ctx_lens, const int32_t *block_table, int batch,
                     int max_pages) {
  for (int s = 0; s < batch; ++s) {
    int n_new = cu_new[s + 1] - cu_new[s];
    for (int i = 0; i < n_new; ++i) {
      int pos = ctx_lens[s] + i;
      int logical = pos / PAGE;
      if (logical >= max_pages) return -1;
      int32_t page = block_table[(size_t)s * max_pages + logical];
      if (page < 0 || page >= num_pages) return -1;
      int off = pos % PAGE;
      size_t tok = (size_t)cu_new[s] + i;
      for (int g = 0; g < Hkv; ++g)
        for (int c = 0; c < d; ++c) {
          k_pages[pool_index(page, off, g, c, Hkv, d)] = k_new[(tok * Hkv + g) * d + c];
          v_pages[pool_index(page, off, g, c, Hkv, d)] = v_new[(tok * Hkv + g) * d + c];
        }
    }
  }
  return 0;
}

/*
 * One output row through the block table.  bt_row = block_table + s * max_pages.
 * q_row: d bf16 values of query head h at absolute position p.  g: its KV head.
 * out: d doubles.  lse: one double (may be NULL).  weights: p+1 doubles (may be NULL).
 */
void oracle_attn_row_paged(const uint16_t *k_pages, const uint16_t *v_pages, int Hkv, int d,
                           const int32_t *bt_row, int p, const uint16_t *q_row, int g,
                           double scale, double *out, double *lse, double *weights) {
  int n = p + 1;
  double *sc = (double *)malloc((size_t)n * sizeof(double));
  double m = -INFINITY;
  for (int j = 0; j < n; ++j) {
    int32_t page = bt_row[j / PAGE];
    int off = j % PAGE;
    double dot = 0.0;
    for (int c = 0; c < d; ++c)
      dot += widen(q_row[c]) * widen(k_pages[pool_index(page, off, g, c, Hkv, d)]);
    sc[j] = scale * dot;
    if (sc[j] > m) m = sc[j];
  }
  double Z = 0.0;
  for (int j = 0; j < n; ++j) {
    sc[j] = exp(sc[j] - m);
    Z += sc[j];
  }
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (int j = 0; j < n; ++j) {
    double w = sc[j] / Z;
    if (weights) weights[j] = w;
    int32_t page = bt_row[j / PAGE];
    int off = j % PAGE;
    for (int c = 0; c < d; ++c) out[c] += w * widen(v_pages[pool_index(page, off, g, c, Hkv, d)]);
  }
  if (lse) *lse = m + log(Z);
  free(sc);
}

/*
 * Same row, but K and V given contiguously as [L][Hkv][d] for one sequence (no paging).
 * Same operations in the same order as the paged routine.
 */
void oracle_attn_row_contig(const uint16_t *k, const uint16_t *v, int Hkv, int d, int p,
                            const uint16_t *q_row, int g, double scale, double *out,
                            double *lse, double *weights) {
  int n = p + 1;
  double *sc = (double *)malloc((size_t)n * sizeof(double));
  double m = -INFINITY;
  for (int j = 0; j < n; ++j) {
    double dot = 0.0;
    for (int c = 0; c < d; ++c) dot += widen(q_row[c]) * widen(k[((size_t)j * Hkv + g) * d + c]);
    sc[j] = scale * dot;
    if (sc[j] > m) m = sc[j];
  }
  double Z = 0.0;
  for (int j = 0; j < n; ++j) {
    sc[j] = exp(sc[j] - m);
    Z += sc[j];
  }
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (int j = 0; j < n; ++j) {
    double w = sc[j] / Z;
    if (weights) weights[j] = w;
    for (int c = 0; c < d; ++c) out[c] += w * widen(v[((size_t)j * Hkv + g) * d + c]);
  }
  if (lse) *lse = m + log(Z);
  free(sc);
}

/*
 * Restricted row: attends only to the keys j whose mask[j] != 0 (mask has p+1 entries).
 * Used by the split/combine identity pin; at least one key must be selected.
 */
void oracle_attn_row_subset(const uint16_t *k_pages, const uint16_t *v_pages, int Hkv, int d,
                            const int32_t *bt_row, int p, const uint8_t *mask,
                            const uint16_t *q_row, int g, double scale, double *out,
                            double *lse) {
  int n = p + 1;
  double *sc = (double *)malloc((size_t)n * sizeof(double));
  double m = -INFINITY;
  for (int j = 0; j < n; ++j) {
    if (!mask[j]) continue;
    int32_t page = bt_row[j / PAGE];
    int off = j % PAGE;
    double dot = 0.0;
    for (int c = 0; c < d; ++c)
      dot += widen(q_row[c]) * widen(k_pages[pool_index(page, off, g, c, Hkv, d)]);
    sc[j] = scale * dot;
    if (sc[j] > m) m = sc[j];
  }
  double Z = 0.0;
  for (int j = 0; j < n; ++j) {
    if (!mask[j]) continue;
    sc[j] = exp(sc[j] - m);
    Z += sc[j];
  }
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (int j = 0; j < n; ++j) {
    if (!mask[j]) continue;
    double w = sc[j] / Z;
    int32_t page = bt_row[j / PAGE];
    int off = j % PAGE;
    for (int c = 0; c < d; ++c) out[c] += w * widen(v_pages[pool_index(page, off, g, c, Hkv, d)]);
  }
  *lse = m + log(Z);
  free(sc);
}

/*
 * Prefill driver: packed varlen queries q[total_q][Hq][d]; sequence s owns query tokens
 * cu_q[s] .. cu_q[s+1]-1 at absolute positions ctx_lens[s] + i.  The chunk's own K/V must
 * already be in the cache.  out: [total_q][Hq][d] doubles, lse: [total_q][Hq] (may be NULL).
 */
void oracle_attn_prefill(const uint16_t *k_pages, const uint16_t *v_pages, int Hkv, int d,
                         const uint16_t *q, const int32_t *cu_q, const int32_t *ctx_lens,
                         const int32_t *block_table, int batch, int max_pages, int Hq,
                         double scale, double *out, double *lse) {
  int group = Hq / Hkv;
  for (int s = 0; s < batch; ++s) {
    int nq = cu_q[s + 1] - cu_q[s];
    long rows = (long)nq * Hq;
#pragma omp parallel for schedule(dynamic, 8)
    for (long r = 0; r < rows; ++r) {
      int i = (int)(r / Hq), h = (int)(r % Hq);
      size_t tok = (size_t)cu_q[s] + i;
      oracle_attn_row_paged(k_pages, v_pages, Hkv, d, block_table + (size_t)s * max_pages,
                            ctx_lens[s] + i, q + (tok * Hq + h) * d, h / group, scale,
                            out + (tok * Hq + h) * d, lse ? lse + tok * Hq + h : NULL, NULL);
    }
  }
}

/*
 * Decode driver: one query token per sequence, q[batch][Hq][d], at absolute position
 * seq_lens[s] - 1 (seq_lens counts the current token, whose K/V is already cached).
 * Sequences with seq_lens[s] == 0 produce zeros.
 */
void oracle_attn_decode(const uint16_t *k_pages, const uint16_t *v_pages, int Hkv, int d,
                        const uint16_t *q, const int32_t *seq_lens, const int32_t *block_table,
                        int batch, int max_pages, int Hq, double scale, double *out,
                        double *lse) {
  int group = Hq / Hkv;
  long rows = (long)batch * Hq;
#pragma omp parallel for schedule(dynamic, 1)
  for (long r = 0; r < rows; ++r) {
    int s = (int)(r / Hq), h = (int)(r % Hq);
    double *o = out + ((size_t)s * Hq + h) * d;
    if (seq_lens[s] <= 0) {
      for (int c = 0; c < d; ++c) o[c] = 0.0;
      if (lse) lse[(size_t)s * Hq + h] = -INFINITY;
      continue;
    }
    oracle_attn_row_paged(k_pages, v_pages, Hkv, d, block_table + (size_t)s * max_pages,
                          seq_lens[s] - 1, q + ((size_t)s * Hq + h) * d, h / group, scale, o,
                          lse ? lse + (size_t)s * Hq + h : NULL, NULL);
  }
}

/*
 * Sampled rows: for the n_rows triples (seq[r], pos_in_chunk[r], head[r]) compute that one
 * output row of the prefill problem above.  Lets a test check a full-size GPU result on a
 * sample without paying for every row.  out: [n_rows][d].
 */
void oracle_attn_prefill_rows(const uint16_t *k_pages, const uint16_t *v_pages, int Hkv, int d,
                              const uint16_t *q, const int32_t *cu_q, const int32_t *ctx_lens,
                              const int32_t *block_table, int max_pages, int Hq, double scale,
                              const int32_t *row_seq, const int32_t *row_tok,
                              const int32_t *row_head, int n_rows, double *out) {
  int group = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n_rows; ++r) {
    int s = row_seq[r], i = row_tok[r], h = row_head[r];
    size_t tok = (size_t)cu_q[s] + i;
    oracle_attn_row_paged(k_pages, v_pages, Hkv, d, block_table + (size_t)s * max_pages,
                          ctx_lens[s] + i, q + (tok * Hq + h) * d, h / group, scale,
                          out + (size_t)r * d, NULL, NULL);
  }
}

/*
 * The local halves of the sequence-parallel head exchange (paper section on Arctic Sequence
 * Parallelism: the sequence is split across the P GPUs, and Figure 2: in the SP mode every GPU
 * attends with its own subset of the heads over all tokens).  Before attention a GPU holds its
 * T_loc tokens with ALL H heads and must hand head slice j to GPU j; after attention it gets
 * its tokens' outputs back one head slice per peer.  With tokens distributed in contiguous
 * slices in rank order, the exchange itself is a plain all-to-all of equal blocks and only
 * these two permutations remain local (bit copies, written out index by index):
 *
 *   pack:    send[j][t][h'][c] = x[t][j * (H/P) + h'][c]          x: [T_loc][H][d]
 *   unpack:  y[t][j * (H/P) + h'][c] = recv[j][t][h'][c]          recv: [P][T_loc][H/P][d]
 */
void oracle_ulysses_pack(const uint16_t *x, uint16_t *send, int T_loc, int H, int d, int P) {
  int hp = H / P;
  for (int j = 0; j < P; ++j)
    for (int t = 0; t < T_loc; ++t)
      for (int h = 0; h < hp; ++h)
        for (int c = 0; c < d; ++c)
          send[(((size_t)j * T_loc + t) * hp + h) * d + c] = x[((size_t)t * H + (size_t)j * hp + h) * d + c];
}

void oracle_ulysses_unpack(const uint16_t *recv, uint16_t *y, int T_loc, int H, int d, int P) {
  int hp = H / P;
  for (int j = 0; j < P; ++j)
    for (int t = 0; t < T_loc; ++t)
      for (int h = 0; h < hp; ++h)
        for (int c = 0; c < d; ++c)
          y[((size_t)t * H + (size_t)j * hp + h) * d + c] = recv[(((size_t)j * T_loc + t) * hp + h) * d + c];
}
