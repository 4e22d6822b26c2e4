// C-ABI entry points: argument validation, error reporting, dispatch to the kernel launchers.
// The operation and its conventions are documented in include/shiftattn.h.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "sp_common.h"

namespace sp {

static thread_local char g_err[512] = "";

int fail(int status, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}

static int check_cache(const sp_cache_desc *c) {
  if (!c) return fail(SP_ERR_NULL, "cache descriptor is NULL");
  if (!c->k_pages || !c->v_pages) return fail(SP_ERR_NULL, "cache pools are NULL");
  if (c->num_pages <= 0 || c->num_kv_heads <= 0)
    return fail(SP_ERR_BAD_SHAPE, "num_pages=%d num_kv_heads=%d must be positive", c->num_pages,
                c->num_kv_heads);
  if (c->page_size != kPage) return fail(SP_ERR_UNSUPPORTED, "page_size=%d (only 16)", c->page_size);
  if (c->head_dim != 64 && c->head_dim != 128)
    return fail(SP_ERR_UNSUPPORTED, "head_dim=%d (only 64 or 128)", c->head_dim);
  return SP_OK;
}

static int check_heads(const sp_cache_desc *c, int num_q_heads) {
  if (num_q_heads <= 0 || num_q_heads % c->num_kv_heads != 0)
    return fail(SP_ERR_BAD_SHAPE, "num_q_heads=%d is not a positive multiple of num_kv_heads=%d",
                num_q_heads, c->num_kv_heads);
  return SP_OK;
}

static int check_scale(float scale) {
  if (!(scale > 0.0f) || !std::isfinite(scale))
    return fail(SP_ERR_UNSUPPORTED, "scale=%g must be positive and finite", (double)scale);
  return SP_OK;
}

}  // namespace sp

using namespace sp;

extern "C" {

int sp_kv_append(const sp_cache_desc *cache, const void *k_new, const void *v_new,
                 const int32_t *cu_seqlens_new, const int32_t *ctx_lens,
                 const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                 int32_t total_new_tokens, void *stream) {
  if (int rc = check_cache(cache)) return rc;
  if (batch < 0 || total_new_tokens < 0 || max_pages_per_seq < 0)
    return fail(SP_ERR_BAD_SHAPE, "negative count (batch=%d total_new_tokens=%d max_pages=%d)", batch,
                total_new_tokens, max_pages_per_seq);
  if (batch == 0 || total_new_tokens == 0) return SP_OK;
  if (!k_new || !v_new || !cu_seqlens_new || !ctx_lens || !block_table)
    return fail(SP_ERR_NULL, "sp_kv_append: NULL argument");
  if (max_pages_per_seq == 0) return fail(SP_ERR_BAD_SHAPE, "max_pages_per_seq=0 with tokens to append");
  return launch_kv_append(*cache, k_new, v_new, cu_seqlens_new, ctx_lens, block_table, batch,
                          max_pages_per_seq, total_new_tokens, (hipStream_t)stream);
}

int sp_attn_prefill(const sp_cache_desc *cache, const void *q, void *out,
                    const int32_t *cu_seqlens_q, const int32_t *ctx_lens,
                    const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                    int32_t total_q_tokens, int32_t max_q_len, int32_t max_kv_len,
                    int32_t num_q_heads, float scale, int32_t causal, void *workspace,
                    size_t workspace_bytes, void *stream) {
  if (int rc = check_cache(cache)) return rc;
  if (int rc = check_heads(cache, num_q_heads)) return rc;
  if (causal != 1) return fail(SP_ERR_UNSUPPORTED, "causal=%d (only causal attention)", causal);
  if (int rc = check_scale(scale)) return rc;
  if (batch < 0 || total_q_tokens < 0 || max_pages_per_seq < 0 || max_q_len < 0 || max_kv_len < 0)
    return fail(SP_ERR_BAD_SHAPE, "negative count in sp_attn_prefill");
  if (batch == 0 || total_q_tokens == 0 || max_q_len == 0) return SP_OK;
  if (!q || !out || !cu_seqlens_q || !ctx_lens || !block_table)
    return fail(SP_ERR_NULL, "sp_attn_prefill: NULL argument");
  if (max_pages_per_seq == 0) return fail(SP_ERR_BAD_SHAPE, "max_pages_per_seq=0 with queries");
  return launch_prefill(*cache, q, out, cu_seqlens_q, ctx_lens, block_table, batch, max_pages_per_seq,
                        total_q_tokens, max_q_len, max_kv_len, num_q_heads, scale,
                        workspace_bytes ? workspace : nullptr, workspace_bytes, (hipStream_t)stream);
}

int sp_chunk_step(const sp_cache_desc *cache, const void *k_new, const void *v_new, const void *q, void *out,
                  const int32_t *cu_seqlens_q, const int32_t *ctx_lens, const int32_t *block_table,
                  int32_t batch, int32_t max_pages_per_seq, int32_t total_q_tokens, int32_t max_q_len,
                  int32_t max_kv_len, int32_t num_q_heads, float scale, void *workspace, size_t workspace_bytes,
                  void *stream) {
  if (int rc = check_cache(cache)) return rc;
  if (int rc = check_heads(cache, num_q_heads)) return rc;
  if (int rc = check_scale(scale)) return rc;
  if (batch < 0 || total_q_tokens < 0 || max_pages_per_seq < 0 || max_q_len < 0 || max_kv_len < 0)
    return fail(SP_ERR_BAD_SHAPE, "negative count in sp_chunk_step");
  if (batch == 0 || total_q_tokens == 0 || max_q_len == 0) return SP_OK;
  if (!k_new || !v_new || !q || !out || !cu_seqlens_q || !ctx_lens || !block_table)
    return fail(SP_ERR_NULL, "sp_chunk_step: NULL argument");
  if (max_pages_per_seq == 0) return fail(SP_ERR_BAD_SHAPE, "max_pages_per_seq=0 with tokens to append");
  return launch_chunk_step(*cache, k_new, v_new, q, out, cu_seqlens_q, ctx_lens, block_table, batch,
                           max_pages_per_seq, total_q_tokens, max_q_len, max_kv_len, num_q_heads, scale,
                           workspace_bytes ? workspace : nullptr, workspace_bytes, (hipStream_t)stream);
}

static int decode_common(const char *name, const sp_cache_desc *cache, const void *k_new, const void *v_new,
                         const void *q, void *out, const int32_t *seq_lens, const int32_t *block_table,
                         int32_t batch, int32_t max_pages_per_seq, int32_t max_seq_len, int32_t num_q_heads,
                         float scale, void *workspace, size_t workspace_bytes, void *stream) {
  if (int rc = check_cache(cache)) return rc;
  if (int rc = check_heads(cache, num_q_heads)) return rc;
  if (int rc = check_scale(scale)) return rc;
  if (batch < 0 || max_pages_per_seq < 0 || max_seq_len < 0)
    return fail(SP_ERR_BAD_SHAPE, "negative count in %s", name);
  if (batch == 0) return SP_OK;
  if (!q || !out || !seq_lens || !block_table) return fail(SP_ERR_NULL, "%s: NULL argument", name);
  if (max_pages_per_seq == 0 && max_seq_len > 0)
    return fail(SP_ERR_BAD_SHAPE, "max_pages_per_seq=0 with max_seq_len=%d", max_seq_len);
  size_t need = decode_workspace_bytes(batch, max_seq_len, num_q_heads, cache->head_dim);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(SP_ERR_WORKSPACE, "decode workspace: need %zu bytes, got %zu", need,
                workspace ? workspace_bytes : (size_t)0);
  return launch_decode(*cache, k_new, v_new, q, out, seq_lens, block_table, batch, max_pages_per_seq,
                       max_seq_len, num_q_heads, scale, workspace, workspace_bytes, (hipStream_t)stream);
}

int sp_attn_decode(const sp_cache_desc *cache, const void *q, void *out, const int32_t *seq_lens,
                   const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq,
                   int32_t max_seq_len, int32_t num_q_heads, float scale, void *workspace,
                   size_t workspace_bytes, void *stream) {
  return decode_common("sp_attn_decode", cache, nullptr, nullptr, q, out, seq_lens, block_table, batch,
                       max_pages_per_seq, max_seq_len, num_q_heads, scale, workspace, workspace_bytes, stream);
}

int sp_attn_decode_static(const sp_cache_desc *cache, const void *q, void *out, const int32_t *seq_lens,
                          const int32_t *block_table, int32_t batch, int32_t max_pages_per_seq, int32_t max_seq_len,
                          int32_t num_q_heads, float scale, void *stream) {
  if (int rc = check_cache(cache)) return rc;
  if (int rc = check_heads(cache, num_q_heads)) return rc;
  if (int rc = check_scale(scale)) return rc;
  if (batch < 0 || max_pages_per_seq < 0 || max_seq_len < 0)
    return fail(SP_ERR_BAD_SHAPE, "negative count in sp_attn_decode_static");
  if (batch == 0) return SP_OK;
  if (!q || !out || !seq_lens || !block_table) return fail(SP_ERR_NULL, "sp_attn_decode_static: NULL argument");
  if (max_pages_per_seq == 0 && max_seq_len > 0)
    return fail(SP_ERR_BAD_SHAPE, "max_pages_per_seq=0 with max_seq_len=%d", max_seq_len);
  return launch_decode_static(*cache, q, out, seq_lens, block_table, batch, max_pages_per_seq, max_seq_len,
                              num_q_heads, scale, (hipStream_t)stream);
}

int sp_decode_step(const sp_cache_desc *cache, const void *k_new, const void *v_new, const void *q, void *out,
                   const int32_t *seq_lens, const int32_t *block_table, int32_t batch,
                   int32_t max_pages_per_seq, int32_t max_seq_len, int32_t num_q_heads, float scale,
                   void *workspace, size_t workspace_bytes, void *stream) {
  if (batch > 0 && (!k_new || !v_new)) return fail(SP_ERR_NULL, "sp_decode_step: NULL k_new / v_new");
  return decode_common("sp_decode_step", cache, k_new, v_new, q, out, seq_lens, block_table, batch,
                       max_pages_per_seq, max_seq_len, num_q_heads, scale, workspace, workspace_bytes, stream);
}

static int ulysses_common(bool pack, const void *src, void *dst, int32_t tokens, int32_t num_heads,
                          int32_t head_dim, int32_t world, void *stream) {
  if (tokens < 0 || num_heads <= 0 || world <= 0)
    return fail(SP_ERR_BAD_SHAPE, "tokens=%d num_heads=%d world=%d", tokens, num_heads, world);
  if (num_heads % world != 0)
    return fail(SP_ERR_BAD_SHAPE, "num_heads=%d is not a multiple of world=%d", num_heads, world);
  if (head_dim <= 0 || head_dim % 8 != 0)
    return fail(SP_ERR_UNSUPPORTED, "head_dim=%d must be a positive multiple of 8", head_dim);
  if (tokens == 0) return SP_OK;
  if (!src || !dst) return fail(SP_ERR_NULL, "ulysses permute: NULL buffer");
  if (src == dst) return fail(SP_ERR_UNSUPPORTED, "ulysses permute: in-place use is not supported");
  return launch_ulysses(pack, src, dst, tokens, num_heads, head_dim, world, (hipStream_t)stream);
}

int sp_ulysses_pack(const void *x, void *send, int32_t tokens, int32_t num_heads, int32_t head_dim,
                    int32_t world, void *stream) {
  return ulysses_common(true, x, send, tokens, num_heads, head_dim, world, stream);
}

int sp_ulysses_unpack(const void *recv, void *y, int32_t tokens, int32_t num_heads, int32_t head_dim,
                      int32_t world, void *stream) {
  return ulysses_common(false, recv, y, tokens, num_heads, head_dim, world, stream);
}

size_t sp_attn_prefill_workspace_size(int32_t batch, int32_t total_q_tokens, int32_t max_q_len,
                                      int32_t max_kv_len, int32_t num_q_heads, int32_t num_kv_heads,
                                      int32_t head_dim) {
  if (batch <= 0 || total_q_tokens <= 0 || num_q_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 ||
      num_q_heads % num_kv_heads != 0)
    return 0;
  return prefill_workspace_bytes(batch, total_q_tokens, max_q_len, max_kv_len, num_q_heads, num_kv_heads,
                                 head_dim);
}

size_t sp_attn_decode_workspace_size(int32_t batch, int32_t max_seq_len, int32_t num_q_heads,
                                     int32_t head_dim) {
  if (batch <= 0 || max_seq_len < 0 || num_q_heads <= 0 || head_dim <= 0) return 0;
  return decode_workspace_bytes(batch, max_seq_len, num_q_heads, head_dim);
}

int sp_debug_validate_metadata(const sp_cache_desc *cache, const int32_t *seq_lens,
                               const int32_t *block_table, int32_t batch,
                               int32_t max_pages_per_seq) {
  if (int rc = check_cache(cache)) return rc;
  if (batch < 0 || max_pages_per_seq < 0) return fail(SP_ERR_BAD_SHAPE, "negative count");
  if (batch == 0) return SP_OK;
  if (!seq_lens || !block_table) return fail(SP_ERR_NULL, "NULL metadata");
  std::vector<int32_t> lens(batch), bt((size_t)batch * max_pages_per_seq);
  hipError_t e = hipMemcpy(lens.data(), seq_lens, lens.size() * 4, hipMemcpyDeviceToHost);
  if (e == hipSuccess && !bt.empty())
    e = hipMemcpy(bt.data(), block_table, bt.size() * 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail(SP_ERR_HIP, "hipMemcpy: %s", hipGetErrorString(e));
  for (int s = 0; s < batch; ++s) {
    if (lens[s] < 0) return fail(SP_ERR_BAD_SHAPE, "seq_lens[%d]=%d is negative", s, lens[s]);
    int pages = (lens[s] + kPage - 1) / kPage;
    if (pages > max_pages_per_seq)
      return fail(SP_ERR_BAD_SHAPE, "sequence %d needs %d pages > max_pages_per_seq=%d", s, pages,
                  max_pages_per_seq);
    for (int p = 0; p < pages; ++p) {
      int32_t pg = bt[(size_t)s * max_pages_per_seq + p];
      if (pg < 0 || pg >= cache->num_pages)
        return fail(SP_ERR_BAD_SHAPE, "block_table[%d][%d]=%d outside [0,%d)", s, p, pg, cache->num_pages);
    }
  }
  return SP_OK;
}

int sp_debug_validate_hints(const int32_t *cu_seqlens, const int32_t *lens, int32_t batch, int32_t total_tokens,
                            int32_t max_q_len, int32_t max_len) {
  if (batch < 0) return fail(SP_ERR_BAD_SHAPE, "negative batch");
  if (batch == 0) return SP_OK;
  if (!lens) return fail(SP_ERR_NULL, "NULL length array");
  std::vector<int32_t> ln(batch), cu(cu_seqlens ? batch + 1 : 0);
  hipError_t e = hipMemcpy(ln.data(), lens, ln.size() * 4, hipMemcpyDeviceToHost);
  if (e == hipSuccess && cu_seqlens) e = hipMemcpy(cu.data(), cu_seqlens, cu.size() * 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail(SP_ERR_HIP, "hipMemcpy: %s", hipGetErrorString(e));
  if (cu_seqlens) {
    if (cu[0] < 0) return fail(SP_ERR_BAD_SHAPE, "cu_seqlens[0]=%d is negative", cu[0]);
    if (cu[batch] > total_tokens)
      return fail(SP_ERR_BAD_SHAPE, "cu_seqlens[%d]=%d exceeds total_tokens=%d", batch, cu[batch], total_tokens);
  }
  for (int s = 0; s < batch; ++s) {
    if (ln[s] < 0) return fail(SP_ERR_BAD_SHAPE, "lens[%d]=%d is negative", s, ln[s]);
    long reach = ln[s];
    if (cu_seqlens) {
      const long n = (long)cu[s + 1] - cu[s];
      if (n < 0) return fail(SP_ERR_BAD_SHAPE, "cu_seqlens decreases at sequence %d (%d -> %d)", s, cu[s], cu[s + 1]);
      if (n > max_q_len) return fail(SP_ERR_BAD_SHAPE, "sequence %d has %ld tokens > max_q_len=%d", s, n, max_q_len);
      reach += n;
    }
    if (reach > max_len)
      return fail(SP_ERR_BAD_SHAPE, "sequence %d reaches %ld keys > the length hint %d", s, reach, max_len);
  }
  return SP_OK;
}

int sp_debug_set_tuning(const char *key, int32_t value) {
  if (!key) return fail(SP_ERR_NULL, "tuning key is NULL");
  if (!strcmp(key, "decode_chunk")) {
    if (value != 0 && (value < 128 || value > 1024 || value % 32 != 0))
      return fail(SP_ERR_UNSUPPORTED, "decode_chunk=%d (0, or a multiple of 32 in [128, 1024])", value);
    set_decode_chunk(value);
    return SP_OK;
  }
  if (!strcmp(key, "decode_ring")) {
    if (value < 0 || value > 4) return fail(SP_ERR_UNSUPPORTED, "decode_ring=%d (0..4)", value);
    set_decode_ring(value);
    return SP_OK;
  }
  if (!strcmp(key, "decode_fuse")) {
    if (value < 0 || value > 2) return fail(SP_ERR_UNSUPPORTED, "decode_fuse=%d (0, 1 or 2)", value);
    set_decode_fuse(value);
    return SP_OK;
  }
  if (!strcmp(key, "prefill_kv_splits")) {
    if (value < 0 || value > 16) return fail(SP_ERR_UNSUPPORTED, "prefill_kv_splits=%d (0..16)", value);
    set_prefill_kv_splits(value);
    return SP_OK;
  }
  if (!strcmp(key, "prefill_split")) {
    if (value < 0 || value > 2) return fail(SP_ERR_UNSUPPORTED, "prefill_split=%d (0, 1 or 2)", value);
    set_prefill_split(value);
    return SP_OK;
  }
  if (!strcmp(key, "combine_form")) {
    if (value < 0 || value > 2) return fail(SP_ERR_UNSUPPORTED, "combine_form=%d (0, 1 or 2)", value);
    set_combine_form(value);
    return SP_OK;
  }
  if (!strcmp(key, "prefill_order")) {
    if (value < 0 || value > 2) return fail(SP_ERR_UNSUPPORTED, "prefill_order=%d (0, 1 or 2)", value);
    set_prefill_order(value);
    return SP_OK;
  }
  if (!strcmp(key, "prefill_short_chunk")) {
    if (value < 0 || value > 1) return fail(SP_ERR_UNSUPPORTED, "prefill_short_chunk=%d (0 or 1)", value);
    set_prefill_short_chunk(value);
    return SP_OK;
  }
  return fail(SP_ERR_UNSUPPORTED, "unknown tuning key '%s'", key);
}

const char *sp_status_string(int status) {
  switch (status) {
    case SP_OK: return "SP_OK";
    case SP_ERR_NULL: return "SP_ERR_NULL";
    case SP_ERR_BAD_SHAPE: return "SP_ERR_BAD_SHAPE";
    case SP_ERR_UNSUPPORTED: return "SP_ERR_UNSUPPORTED";
    case SP_ERR_WORKSPACE: return "SP_ERR_WORKSPACE";
    case SP_ERR_HIP: return "SP_ERR_HIP";
    default: return "SP_ERR_UNKNOWN";
  }
}

const char *sp_last_error(void) { return g_err; }

int sp_version(void) { return 100; }

}  // extern "C"
