// Shared declarations for the gfx950 kernels of the Shift Parallelism attention hot path
// (per-GPU head shard, paged KV cache with a mode-invariant layout; paper section
// "Introducing Shift Parallelism").  Internal to the library: nothing here is part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "shiftattn.h"

namespace sp {

constexpr int kPage = 16;  // tokens per KV page (fixed by the cache layout)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// Records a failure text for sp_last_error() and passes the status through.
int fail(int status, const char *fmt, ...);

// Kernel launchers (each validates nothing: the entry points in api.hip did that).
int launch_kv_append(const sp_cache_desc &c, const void *k_new, const void *v_new,
                     const int32_t *cu_new, const int32_t *ctx_lens, const int32_t *block_table,
                     int batch, int max_pages, int total_new, hipStream_t stream);

int launch_prefill(const sp_cache_desc &c, const void *q, void *out, const int32_t *cu_q,
                   const int32_t *ctx_lens, const int32_t *block_table, int batch, int max_pages,
                   int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                   void *workspace, size_t workspace_bytes, hipStream_t stream);
// Append the chunks' K/V rows, then attend (sp_chunk_step): one fused launch where the short-chunk
// path applies, else launch_kv_append + launch_prefill.
int launch_chunk_step(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                      const int32_t *cu_q, const int32_t *ctx_lens, const int32_t *block_table, int batch,
                      int max_pages, int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                      void *workspace, size_t workspace_bytes, hipStream_t stream);
size_t prefill_workspace_bytes(int batch, int total_q_tokens, int max_q_len, int max_kv_len, int num_q_heads,
                               int num_kv_heads, int head_dim);

// [T_loc][H][d] <-> [P][T_loc][H/P][d] (pack = to the blocked side), bf16 elements.
int launch_ulysses(bool pack, const void *src, void *dst, int T_loc, int H, int d, int P, hipStream_t stream);

// Tuning hooks behind sp_debug_set_tuning (0 restores the built-in heuristic).
void set_decode_chunk(int chunk);
void set_combine_form(int form);  // combine kernel: 0 heuristic, 1 one 32-channel slice per wave, 2 a whole row per wave
void set_decode_fuse(int mode);    // combine pass of the single-token decode: 0 heuristic, 1 separate kernel, 2 inside the split kernel (up to 32 splits)
void set_decode_ring(int slots);   // LDS ring depth of the decode split kernel: 0 heuristic, 2..4, 1 = two K blocks + one V block
void set_prefill_kv_splits(int n);  // pieces a query tile's key range is cut into: 0 heuristic, 1..16
void set_prefill_short_chunk(int mode);  // 0 heuristic, 1 short query chunks stay on the prefill kernel
void set_prefill_split(int mode);
void set_prefill_order(int mode);  // 0 heuristic, 1 workgroups in (tile, sequence) order, 2 heaviest work item first  // 0 heuristic, 1 never split the key range over the wave groups, 2 always

// Log-sum-exp merge of per-split partials: part_o [rows][nsplit][head_dim] fp32 un-normalised,
// part_ml [rows][nsplit][2] fp32 (max in log2 units, sum); out [rows][head_dim] bf16.
// part_o == nullptr writes zero rows.
// cu_q non-NULL (varlen batches): only the rows [cu_q[0], cu_q[batch]) x num_q_heads are written.
// route_cap > 0 (mixed batches): the partials' rows are [sequence][route_cap tokens][head] (see launch_decode_multi).
int launch_combine(const float *part_o, const float *part_ml, void *out, long rows, int nsplit, int head_dim,
                   hipStream_t stream, const int32_t *cu_q = nullptr, int batch = 0, int num_q_heads = 0,
                   int route_cap = 0);

size_t decode_workspace_bytes(int batch, int max_seq_len, int num_q_heads, int head_dim);
// k_new / v_new non-NULL: fused decode step (the new token's rows are appended by the kernel).
int launch_decode(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                  const int32_t *seq_lens, const int32_t *block_table, int batch, int max_pages,
                  int max_seq_len, int num_q_heads, float scale, void *workspace, size_t workspace_bytes,
                  hipStream_t stream);

// sp_attn_decode_static: partials in the library's own static device array instead of a workspace.
size_t decode_static_scratch_bytes();
int launch_decode_static(const sp_cache_desc &c, const void *q, void *out, const int32_t *seq_lens,
                         const int32_t *block_table, int batch, int max_pages, int max_seq_len, int num_q_heads,
                         float scale, hipStream_t stream);

// Short query chunks (a few tokens per sequence on long prefixes) on the decode split kernel:
// same arguments as launch_prefill.  Returns 1 without launching anything when the shape or the
// workspace does not qualify; decode_multi_workspace_bytes is 0 for shapes that never qualify.
// k_new / v_new non-NULL: the chunks' K/V rows ([total_q][Hkv][d]) are not in the cache yet and are
// appended by the kernel (fused chunk step).
size_t decode_multi_workspace_bytes(int batch, int total_q, int max_q_len, int max_kv_len, int num_q_heads,
                                    int num_kv_heads, int head_dim);
int launch_decode_multi(const sp_cache_desc &c, const void *k_new, const void *v_new, const void *q, void *out,
                        const int32_t *cu_q,
                        const int32_t *ctx_lens, const int32_t *block_table, int batch, int max_pages,
                        int total_q, int max_q_len, int max_kv_len, int num_q_heads, float scale,
                        void *workspace, size_t workspace_bytes, hipStream_t stream, bool routed = false);
// Mixed batches: routed = true serves only the sequences with at most decode_route_cap query tokens
// (partials indexed [sequence][cap][head]; workspace size from decode_routed_workspace_bytes).
int decode_route_cap(int num_q_heads, int num_kv_heads);
size_t decode_routed_workspace_bytes(int batch, int max_kv_len, int num_q_heads, int num_kv_heads, int head_dim);

}  // namespace sp
