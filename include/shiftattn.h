/*
 * shiftattn — C ABI of the Shift Parallelism attention hot path on one MI355X (gfx950).
 *
 * The operation is causal grouped-query attention over ONE GPU's head shard, reading a
 * paged KV cache.  Source: the paper's section "Introducing Shift Parallelism" and Figure 2.
 * Two facts stated there shape this interface: switching between the sequence-parallel
 * (Ulysses) mode and the tensor-parallel mode leaves the KV cache where it is whenever the
 * two degrees multiply to the size of the GPU group, and under either mode a GPU attends
 * with the same subset of heads over every token.  Both are structural here: sp_kv_append,
 * sp_attn_prefill and sp_attn_decode take the same sp_cache_desc and block table, and the
 * ABI has no re-layout entry point.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HBM) unless the name starts with host_.
 *     The sp_cache_desc struct itself is read on the HOST at call time.
 *   - bf16 tensors are raw 16-bit patterns; index arrays are int32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: no allocation, no synchronisation, no host<->device copies.
 *   - The caller owns every buffer; the library keeps no device state between calls.  Host
 *     state: the calling thread's last error text and its sp_debug_set_tuning overrides, both
 *     thread-local.
 *   - Return value: SP_OK (0) or a negative sp_status.  On any error nothing is launched.
 *     No exception crosses the ABI.  Device-side metadata (lengths, block-table entries)
 *     is NOT validated by the hot calls; sp_debug_validate_metadata and
 *     sp_debug_validate_hints do that, synchronously, for tests.  With bad metadata the hot
 *     calls stay inside the pools (page ids are clamped for loads; stores to pages outside the
 *     pool or past the block-table row are skipped) and return unspecified finite-or-not values.
 *   - Page indexing (exact int32 arithmetic): token j of sequence s lives in physical page
 *     block_table[s * max_pages_per_seq + j / 16], row j % 16.
 *   - GQA map: query head h reads KV head h / (num_q_heads / num_kv_heads).
 *   - Causal convention with a cached prefix: the query at absolute position p sees keys
 *     0..p inclusive.
 */
#ifndef SHIFTATTN_H
#define SHIFTATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sp_status {
  SP_OK = 0,
  SP_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  SP_ERR_BAD_SHAPE = -2,   /* negative count, num_q_heads % num_kv_heads != 0, ...          */
  SP_ERR_UNSUPPORTED = -3, /* page_size != 16, head_dim not in {64,128}, causal != 1, ...   */
  SP_ERR_WORKSPACE = -4,   /* workspace missing or too small                                */
  SP_ERR_HIP = -5          /* HIP runtime error at launch; text in sp_last_error()          */
} sp_status;

/* The paged KV cache of one GPU's head shard.  Caller-owned device memory; the library
 * never allocates, frees or re-lays it out.  Both pools have the layout
 *     bf16 [num_pages][num_kv_heads][page_size = 16][head_dim]
 * so every (page, kv head) is one contiguous 16 x head_dim block (4 KiB at head_dim 128). */
typedef struct sp_cache_desc {
  void *k_pages;        /* device, bf16                                                   */
  void *v_pages;        /* device, bf16, same shape                                       */
  int32_t num_pages;    /* physical pages in the pool                                     */
  int32_t page_size;    /* must be 16                                                     */
  int32_t num_kv_heads; /* KV heads of THIS shard (1 for Llama-3.3-70B at P = 8)          */
  int32_t head_dim;     /* 64 or 128                                                      */
} sp_cache_desc;

/*
 * sp_kv_append — write the new tokens' K and V into their pages (the step in front of both
 * attention calls).  Paper, section "Introducing Shift Parallelism", the paragraph on the
 * invariant KV-cache layout: one cache image serves both modes, so there is one append.
 *   k_new, v_new    bf16 [total_new_tokens][num_kv_heads][head_dim], packed by sequence
 *   cu_seqlens_new  int32 [batch + 1] prefix sums of new tokens per sequence
 *   ctx_lens        int32 [batch] tokens already cached per sequence; new token i of
 *                   sequence s goes to absolute position ctx_lens[s] + i
 *   block_table     int32 [batch][max_pages_per_seq]
 * Sequences with zero new tokens are no-ops.  batch == 0 or total_new_tokens == 0 returns
 * SP_OK without launching.  Slots not named by the inputs are left untouched; rows whose page
 * id lies outside the pool or past the block-table row are skipped.
 * Sub-ranges: as for sp_attn_prefill (keep k_new, v_new and total_new_tokens, advance the three
 * index arrays); tokens outside [cu_seqlens_new[0], cu_seqlens_new[batch]) are not touched.
 */
int sp_kv_append(const sp_cache_desc *cache, const void *k_new, const void *v_new,
                 const int32_t *cu_seqlens_new, const int32_t *ctx_lens,
                 const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                 int32_t total_new_tokens, void *stream);

/*
 * sp_attn_prefill — causal GQA attention for a packed varlen batch of query chunks (the SP
 * mode after the sequence->head all-to-all, and chunked prefill against a cached prefix).
 * Paper, section "Introducing Shift Parallelism" and Figure 2: in the sequence-parallel mode a
 * GPU attends with its own heads over all tokens of the request, reading the shared cache.
 *   q, out          bf16 [total_q_tokens][num_q_heads][head_dim]; out is written with one
 *                   round-to-nearest-even from fp32
 *   cu_seqlens_q    int32 [batch + 1]
 *   ctx_lens        int32 [batch] tokens cached BEFORE this chunk; the chunk's own K/V must
 *                   already have been appended (query i of sequence s is at ctx_lens[s] + i)
 *   max_q_len       host hint: >= the longest chunk in the batch (sizes the grid)
 *   max_kv_len      host hint: >= the largest ctx_lens[s] + chunk length (sizes launches and
 *                   the workspace)
 *                   A hint that is too SMALL is not detected by the call: query rows beyond
 *                   max_q_len are then not computed (their `out` rows keep their old bytes)
 *                   and keys beyond max_kv_len may be ignored.  sp_debug_validate_hints checks
 *                   both hints and total_q_tokens against the device arrays.
 *   scale           softmax scale, normally 1/sqrt(head_dim)
 *   causal          must be 1
 *   workspace       optional device scratch (contents need no initialisation).  With at least
 *                   sp_attn_prefill_workspace_size(...) bytes the library may cut long key
 *                   ranges into pieces computed by separate workgroups and merged by a
 *                   log-sum-exp combine pass, which it does for batches of few query tokens on
 *                   long cached prefixes; with NULL / 0 (or less than that) it uses fewer
 *                   pieces or none.  The result is the same up to fp32 summation order.
 *                   Batches whose chunks are all a few tokens long (max_q_len times the query
 *                   heads per KV head <= 32, for some shapes <= 64: the verification step of
 *                   speculative decoding) are served, when the workspace allows, by the decode
 *                   kernels: bandwidth-bound, all of a sequence's query tokens share one read
 *                   of its keys.
 * Sub-ranges.  The call touches only the rows of `out` that belong to its sequences, so a batch
 * may be attended in several calls on sub-ranges of its sequences: keep q, out and
 * total_q_tokens, advance cu_seqlens_q, ctx_lens and block_table to the first sequence of the
 * range and pass the range's batch size and hints (cu_seqlens_q keeps its absolute token
 * offsets).
 * Mixed batches — sequences with a few query tokens (single-token decodes, verification chunks)
 * next to sequences with long prefill chunks in one step — are served by one call: given the
 * workspace, the library routes the short sequences (at most 32 / (query heads per KV head)
 * tokens) to the decode kernels and the others to the prefill kernel, by the lengths it finds
 * on the device.  It takes a batch for mixed when the hints say so: max_q_len beyond that token
 * count, and total_q_tokens - max_q_len smaller than (batch - 1) times that count plus one.
 * Arithmetic: bf16 MFMA with fp32 accumulation, fp32 online softmax.  The error bound of
 * 1e-2 absolute against the exact result holds for inputs distributed like N(0,1) q, k, v with
 * scale 1/sqrt(head_dim); it scales with |out| (bf16 output: half an ulp is 2^-9 |out|) and,
 * for nearly one-hot softmax rows, with the bf16 rounding of the dominant weight (2^-8 |out|).
 */
int sp_attn_prefill(const sp_cache_desc *cache, const void *q, void *out,
                    const int32_t *cu_seqlens_q, const int32_t *ctx_lens,
                    const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                    int32_t total_q_tokens, int32_t max_q_len, int32_t max_kv_len,
                    int32_t num_q_heads, float scale, int32_t causal, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * sp_attn_decode — one query token per sequence (the TP mode), split over the key range
 * with a log-sum-exp combine pass.  Paper, section "Introducing Shift Parallelism" and
 * Figure 2: in the tensor-parallel mode the same GPU attends with the same heads, reading the
 * same cache the prefill mode filled.
 *   q, out          bf16 [batch][num_q_heads][head_dim]
 *   seq_lens        int32 [batch] INCLUDING the current token, whose K/V is already cached;
 *                   a sequence with seq_lens[s] == 0 gets an all-zero output row
 *   max_seq_len     host hint: >= max seq_lens[s] (sizes the split grid and the workspace)
 *   workspace       device scratch of at least sp_attn_decode_workspace_size(...) bytes for
 *                   the per-split partial results; contents need no initialisation
 */
int sp_attn_decode(const sp_cache_desc *cache, const void *q, void *out,
                   const int32_t *seq_lens, const int32_t *block_table, int32_t batch,
                   int32_t max_pages_per_seq, int32_t max_seq_len, int32_t num_q_heads,
                   float scale, void *workspace, size_t workspace_bytes, void *stream);

/*
 * sp_attn_decode_static — sp_attn_decode for callers that cannot allocate or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and same result, bit for bit, as sp_attn_decode, but the per-split
 * partials live in a static device array inside the library (16 MiB, held on every GPU the
 * library has run this call on until the process ends), and the call makes no allocation of
 * any kind.
 *   - Shapes whose partials exceed 16 MiB (sp_attn_decode_workspace_size(...) > 16 MiB) are
 *     refused with SP_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two
 *     streams, two threads) race and must be serialised by the caller.  The array needs no
 *     clearing between calls (every slot is written by the launch that reads it).
 *   - The first call on a device looks up the array's device address (and sets kernel
 *     attributes); make that call outside any stream capture.
 */
int sp_attn_decode_static(const sp_cache_desc *cache, const void *q, void *out,
                          const int32_t *seq_lens, const int32_t *block_table, int32_t batch,
                          int32_t max_pages_per_seq, int32_t max_seq_len, int32_t num_q_heads,
                          float scale, void *stream);

/*
 * sp_chunk_step — one chunk step in one call: sp_kv_append of every sequence's new tokens
 * followed by sp_attn_prefill over them (chunked prefill, or the verification step of
 * speculative decoding: the last accepted token plus the draft tokens).
 *   k_new, v_new    bf16 [total_q_tokens][num_kv_heads][head_dim]: K/V of the chunks' tokens,
 *                   packed like q (cu_seqlens_q serves both)
 *   everything else as in sp_attn_prefill (ctx_lens = tokens cached before the chunk),
 *   same workspace size.
 * Where sp_attn_prefill would take its short-chunk path, the append happens inside the attention
 * kernel (the waves whose key range holds the new positions fetch the rows, use them and store
 * them to their pages): one launch less in a launch-bound step.  Otherwise the call is
 * sp_kv_append + sp_attn_prefill.  Either way the cache afterwards holds the new rows exactly
 * as sp_kv_append would have written them and `out` equals sp_attn_prefill's on that cache.
 */
int sp_chunk_step(const sp_cache_desc *cache, const void *k_new, const void *v_new,
                  const void *q, void *out, const int32_t *cu_seqlens_q,
                  const int32_t *ctx_lens, const int32_t *block_table, int32_t batch,
                  int32_t max_pages_per_seq, int32_t total_q_tokens, int32_t max_q_len,
                  int32_t max_kv_len, int32_t num_q_heads, float scale, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * sp_decode_step — one decode step in one call: sp_kv_append of one new token per sequence
 * followed by sp_attn_decode, with the append done inside the attention kernel (the step in
 * front of the TP-mode attention fused into it; a decode step is launch-bound, and this removes
 * one of its launches).
 *   k_new, v_new    bf16 [batch][num_kv_heads][head_dim]: the new token's K/V of every sequence
 *   seq_lens        int32 [batch] INCLUDING the new token, which goes to position
 *                   seq_lens[s] - 1 (its page must be present in the block table); a sequence
 *                   with seq_lens[s] == 0 appends nothing and gets an all-zero output row
 *   everything else as in sp_attn_decode, same workspace size.
 * Afterwards the cache holds the new rows exactly as sp_kv_append would have written them and
 * `out` equals what sp_attn_decode would return on that cache.
 */
int sp_decode_step(const sp_cache_desc *cache, const void *k_new, const void *v_new,
                   const void *q, void *out, const int32_t *seq_lens,
                   const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                   int32_t max_seq_len, int32_t num_q_heads, float scale, void *workspace,
                   size_t workspace_bytes, void *stream);

/* Bytes of workspace for the given host-side shape: what sp_attn_decode requires, and what lets
 * sp_attn_prefill split key ranges or take its short-chunk path (0 when neither would be used:
 * too many query rows for it to pay).  max_q_len / max_kv_len are the hints later passed to
 * sp_attn_prefill; the sizes are not monotone in the length hints (the split length follows the
 * shape), so ask again when the hints change: a call checks its workspace against the size for
 * the hints it is given. */
size_t sp_attn_prefill_workspace_size(int32_t batch, int32_t total_q_tokens, int32_t max_q_len,
                                      int32_t max_kv_len, int32_t num_q_heads,
                                      int32_t num_kv_heads, int32_t head_dim);
size_t sp_attn_decode_workspace_size(int32_t batch, int32_t max_seq_len, int32_t num_q_heads,
                                     int32_t head_dim);

/*
 * sp_ulysses_pack / sp_ulysses_unpack — the local halves of the sequence-parallel head exchange
 * (the steps either side of the attention path in SP mode; the all-to-all itself is not part of
 * this library).  A rank holds `tokens` tokens with all `num_heads` heads; `world` ranks.
 *   pack    x     bf16 [tokens][num_heads][head_dim]
 *           send  bf16 [world][tokens][num_heads / world][head_dim]; block j holds head slice j,
 *                 contiguous, ready to be sent to rank j
 *   unpack  recv  bf16 [world][tokens][num_heads / world][head_dim]; block j came from rank j
 *           y     bf16 [tokens][num_heads][head_dim]
 * Pure bit copies (unpack inverts pack).  num_heads % world != 0 -> SP_ERR_BAD_SHAPE; head_dim
 * must be a multiple of 8; in-place use is refused; tokens == 0 is a no-op.
 */
int sp_ulysses_pack(const void *x, void *send, int32_t tokens, int32_t num_heads,
                    int32_t head_dim, int32_t world, void *stream);
int sp_ulysses_unpack(const void *recv, void *y, int32_t tokens, int32_t num_heads,
                      int32_t head_dim, int32_t world, void *stream);

/*
 * sp_debug_validate_metadata — SYNCHRONOUS test helper: copies the int32 arrays to the host
 * and checks 0 <= page < num_pages for every page a sequence uses and
 * ceil(seq_lens[s] / 16) <= max_pages_per_seq.  Returns SP_OK or SP_ERR_BAD_SHAPE.
 */
int sp_debug_validate_metadata(const sp_cache_desc *cache, const int32_t *seq_lens,
                               const int32_t *block_table, int32_t batch,
                               int32_t max_pages_per_seq);

/*
 * sp_debug_validate_hints — SYNCHRONOUS test helper: copies the length arrays to the host and
 * checks the host-side hints of an attention call against them.
 *   cu_seqlens      int32 [batch + 1] (device) of sp_kv_append / sp_attn_prefill / sp_chunk_step,
 *                   or NULL for sp_attn_decode / sp_decode_step
 *   lens            int32 [batch] (device): ctx_lens when cu_seqlens is given, else seq_lens
 *   total_tokens    the call's total_q_tokens / total_new_tokens (ignored without cu_seqlens)
 *   max_q_len       the call's max_q_len (ignored without cu_seqlens)
 *   max_len         the call's max_kv_len, or max_seq_len for the decode calls
 * Checks: lengths non-negative; cu_seqlens non-decreasing with 0 <= cu_seqlens[0] and
 * cu_seqlens[batch] <= total_tokens; every chunk <= max_q_len; every lens[s] + chunk (or
 * seq_lens[s]) <= max_len.  Returns SP_OK or SP_ERR_BAD_SHAPE with the first violation in
 * sp_last_error().
 */
int sp_debug_validate_hints(const int32_t *cu_seqlens, const int32_t *lens, int32_t batch,
                            int32_t total_tokens, int32_t max_q_len, int32_t max_len);

/*
 * sp_debug_set_tuning — override of an internal launch parameter for the CALLING THREAD (the
 * workspace-size helpers and the attention calls made by that thread see it; other threads keep
 * their own values), for tuning sweeps and tests.  Keys:
 *   "decode_chunk"  keys per decode split: 0 (built-in heuristic) or a multiple of 32 in
 *                   [128, 1024].  Changes what sp_attn_decode_workspace_size returns.
 *   "decode_ring"   32-key blocks a decode wave keeps in its LDS ring (one computed on, the
 *                   rest in flight): 0 (built-in choice), 2..4, or 1 for two K blocks and a
 *                   single V block (less LDS per wave, one more resident wave per CU).
 *   "decode_fuse"   where the log-sum-exp combine of sp_attn_decode / sp_decode_step runs: 0 (built-in
 *                   choice: a kernel of its own), 1 (the same), 2 (inside the split kernel, by the
 *                   wave of a (sequence, head group) that finishes last; only taken up to 32
 *                   splits; slower on this chip, kept for measurement).
 *   "combine_form"  work of a wave of the log-sum-exp combine kernel: 0 (built-in choice on the row
 *                   count), 1 (one 32-channel slice of a row), 2 (a whole row; only taken up to
 *                   64 splits per row).
 *   "prefill_kv_splits" pieces the key range of a prefill query tile is cut into when a
 *                   workspace is given: 0 (built-in heuristic) or 1..16 (still bounded by the
 *                   workspace size).
 *   "prefill_split" how a prefill workgroup's two wave groups divide the work: 0 (built-in
 *                   heuristic on the grid size), 1 (neighbouring query columns, shared key
 *                   tiles), 2 (same query columns, alternate key tiles, merged at the end).
 *                   Both give the same result up to fp32 summation order.  Launches that cut
 *                   key ranges into pieces always take form 2.
 *   "prefill_order" which work item (sequence, query tile) a prefill workgroup takes: 0 (built-in
 *                   choice), 1 (by launch index: last query tiles of all sequences first), 2 (the
 *                   workgroup with the r-th launch index takes the r-th heaviest item; batches of
 *                   up to 256 sequences).  Same result bit for bit.
 *   "prefill_short_chunk" 0 (built-in choice: batches of short chunks go to the decode
 *                   kernels when the workspace allows) or 1 (never; always the prefill kernel).
 *                   Changes what sp_attn_prefill_workspace_size returns.
 * Returns SP_OK, SP_ERR_NULL or SP_ERR_UNSUPPORTED (unknown key / value out of range).
 */
int sp_debug_set_tuning(const char *key, int32_t value);

const char *sp_status_string(int status); /* static string                              */
const char *sp_last_error(void);          /* thread-local detail of the last failure    */
int sp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SHIFTATTN_H */
