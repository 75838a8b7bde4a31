/*
 * fusionrag.h -- C ABI of the MI355X (gfx950) selective-prefill library.
 *
 * One transformer layer of FusionRAG's online reprocessing stage (arXiv 2601.12904):
 *
 *   fr_rope_shift           stitch the cached chunks: move each chunk's keys from the positions
 *                           they were cached at to their positions in the assembled prompt
 *   fr_score_select         Query-Guided Selection: critical score per context token, top-k,
 *                           and the Q index (critical tokens, then question tokens)
 *   fr_sparse_prefill_attn  causal attention of the Q-index rows only, over the whole K/V
 *   fr_kv_scatter           place the recomputed K/V rows in the cache
 *
 * Conventions shared by every entry point
 *   - Tensors are token-major [tokens, heads, head_dim], head_dim contiguous, no padding, element
 *     type fr_layer_desc.dtype.  "dev" pointers are device (HBM) addresses, 16-byte aligned;
 *     "host" pointers are ordinary host memory read before the call returns.
 *   - The caller owns every tensor.  The library owns only the workspace allocated by fr_create.
 *   - Every call enqueues its kernels on the given HIP stream (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns without synchronising it.  Calls that share a
 *     context share its workspace and must be stream-ordered with respect to each other.
 *     After fr_create no call allocates, frees or synchronises anything, and scratch memory is cleared by
 *     kernels, so a sequence of calls can be captured into a HIP graph and replayed (run each call once
 *     eagerly first: a kernel's shared-memory limit is raised at its first launch, outside any capture;
 *     FR_OPT_ATTN_KERNEL_TIMER records events and is for eager runs).
 *   - Positions and token indices are 0-based (the paper counts from 1).
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).  Logits are scaled by
 *     1/sqrt(head_dim).
 *   - Arguments are validated on the host before anything is launched; on an invalid argument
 *     nothing is enqueued and FR_ERR_INVALID_ARG / FR_ERR_UNSUPPORTED is returned.  The contents
 *     of device buffers (for example that q_index is ascending) are preconditions and are not
 *     checked.  No call throws or aborts.
 */
#ifndef FUSIONRAG_H
#define FUSIONRAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fr_ctx fr_ctx; /* opaque: layer description + device workspace */

typedef enum {
    FR_OK = 0,
    FR_ERR_INVALID_ARG = 1, /* null / misaligned pointer, bad size, offsets not ascending, ...   */
    FR_ERR_UNSUPPORTED = 2, /* a shape or mode this build has no kernel for                      */
    FR_ERR_WORKSPACE = 3,   /* the call needs more workspace than fr_create was sized for        */
    FR_ERR_DEVICE = 4       /* no GPU, or a HIP call failed (message in fr_last_error)           */
} fr_status;

typedef enum { FR_F32 = 0, FR_BF16 = 1 } fr_dtype;

/* How the two members of a rotary pair are laid out in the head dimension.
 * INTERLEAVED: pairs (0,1), (2,3), ... -- the paper's definition (Appendix A:
 * rotate(k) = [-k2, k1, -k4, k3, ...], theta repeated pairwise).  HALF: pairs (p, p + d/2). */
typedef enum { FR_ROPE_INTERLEAVED = 0, FR_ROPE_HALF = 1 } fr_rope_layout;

/* What "attention weight" means when the critical scores are summed (Sec. 3.2).
 * PER_CHUNK: softmax over the keys of the token's own chunk (the matrix is built per chunk).
 * GLOBAL:    one softmax over all context keys.
 * RAW:       no softmax, the scaled logits themselves.                                         */
typedef enum { FR_NORM_PER_CHUNK = 0, FR_NORM_GLOBAL = 1, FR_NORM_RAW = 2 } fr_score_norm;

typedef struct {
    int32_t n_q_heads;       /* Hq                                                               */
    int32_t n_kv_heads;      /* Hkv, divides Hq                                                  */
    int32_t head_dim;        /* d: 64 or 128                                                     */
    int32_t dtype;           /* fr_dtype: storage type of Q, K, V and O                          */
    double rope_base;        /* theta_p = rope_base^(-2 (p + rope_index_base) / d)               */
    int32_t rope_layout;     /* fr_rope_layout                                                   */
    int32_t rope_index_base; /* 0: p = 0..d/2-1 (usual); 1: the appendix's printed i = 1..d/2    */
} fr_layer_desc;

#define FR_MAX_CHUNKS 256 /* chunk tables travel as kernel arguments                           */

/* Create a context for one layer shape.  max_tokens bounds L (context + question tokens),
 * max_chunks (<= FR_MAX_CHUNKS) the number of chunks, max_question_tokens bounds nq.  Allocates
 * the device workspace on the current device; with no GPU present the context is still created
 * (argument validation works) and every launching call returns FR_ERR_DEVICE.
 * *out is set to NULL on failure. */
fr_status fr_create(const fr_layer_desc* desc, int64_t max_tokens, int32_t max_chunks,
                    int32_t max_question_tokens, fr_ctx** out);

/* Free the workspace.  The caller must have synchronised every stream the context was used on. */
void fr_destroy(fr_ctx* ctx);

/* Message of the last failing call on this context (valid until the next call on it). */
const char* fr_last_error(const fr_ctx* ctx);

/* Bytes of device workspace the context holds (0 without a GPU). */
int64_t fr_workspace_bytes(const fr_ctx* ctx);

/* Tuning / test switches.  FR_OPT_ATTN_SOFTMAX chooses how the tiled bf16 attention kernel keeps exp() in
 * range: AUTO (default) fixes each row's exponent reference at the maximum over its first 32 visible keys
 * and recomputes, with a running maximum, only the workgroups whose sums overflowed; RUNNING_MAX uses the
 * running maximum everywhere.  Both give the same softmax; the option exists so that tests reach both.
 * FR_OPT_ATTN_SPLIT: AUTO (default) deals the key range of every (row tile, KV head) to two or more workgroups when
 * there are too few of those to fill the chip (few recomputed rows, e.g. question-only prefill or the offline stage of
 * eq. 10); OFF: never; ON: two workgroups each whenever the partial results fit the workspace.  Same results up to the
 * summation order and the partial sums' storage format (half precision after a per-column power-of-two scale: 11
 * significant bits of a column's largest partial value, finer than the bf16 output).
 * FR_OPT_DECODE_KERNEL: AUTO (default) lets fr_decode_attn form the logits on the matrix cores where it can (bf16,
 * head_dim 128); GENERIC forces the all-vector-ALU kernel that every other shape uses (so that tests reach both).
 * FR_OPT_GEMM_TILE: output features per workgroup of the projection kernels, 0 (default: 256 where the feature count
 * is a multiple of 256, else 128), 128 or 256; for tests and tuning.
 * FR_OPT_GEMM_TAIL_SPLIT: 1 (default): when the output tiles of a projection do not fill the last round of
 * workgroups (one per CU), the tiles of that round are split along K over several workgroups each and a second small
 * kernel adds the parts; 0: never.  Same results up to fp32 summation order; for tests and tuning.  (Like every
 * option these two belong to the context they are set on.)
 * FR_OPT_ATTN_KERNEL_TIMER: value n in [0, 256]: the tiled attention launch attaches an event pair to the dispatch of
 * its dominant kernel (the key-tile loop) on the call's stream, start and end of that kernel's execution, and keeps
 * the last n pairs; 0 (default) switches the timer off.  Read with fr_attn_kernel_times.  For benchmarks: the events
 * see one kernel, not the whole call. */
typedef enum { FR_OPT_ATTN_SOFTMAX = 1, FR_OPT_ATTN_SPLIT = 2, FR_OPT_DECODE_KERNEL = 3, FR_OPT_GEMM_TILE = 4,
               FR_OPT_ATTN_KERNEL_TIMER = 5, FR_OPT_GEMM_TAIL_SPLIT = 6 } fr_option;
typedef enum { FR_DECODE_KERNEL_AUTO = 0, FR_DECODE_KERNEL_GENERIC = 1 } fr_decode_kernel;
typedef enum { FR_ATTN_SOFTMAX_AUTO = 0, FR_ATTN_SOFTMAX_RUNNING_MAX = 1 } fr_attn_softmax;
typedef enum { FR_ATTN_SPLIT_AUTO = 0, FR_ATTN_SPLIT_OFF = 1, FR_ATTN_SPLIT_ON = 2 } fr_attn_split;
fr_status fr_set_option(fr_ctx* ctx, int32_t option, int64_t value);

/* Durations (ms) of the dominant attention kernel of the most recent launches recorded under
 * FR_OPT_ATTN_KERNEL_TIMER, oldest first: at most `capacity` values into the host array ms_out, their number into
 * *n_out.  Waits for the recorded launches to finish. */
fr_status fr_attn_kernel_times(fr_ctx* ctx, float* ms_out, int32_t capacity, int32_t* n_out);

/* Number of context tokens a recompute ratio selects: floor(ratio * L_ctx + 0.5) clamped to
 * [0, L_ctx].  The ratio counts context tokens; question tokens are always computed (Sec. 4.3).
 * Pure host function. */
int64_t fr_topk_count(int64_t L_ctx, double ratio);

/* Position recovery while stitching chunk caches (Sec. 2.2.1 footnote, Appendix A).
 * For chunk c (rows chunk_offsets[c] .. chunk_offsets[c+1]-1) every key is rotated by
 * Delta_c = dst_pos0[c] - src_pos0[c] positions: pair (a, b) of rotary index p becomes
 * (a cos(Delta_c theta_p) - b sin(..), b cos(..) + a sin(..)).  RoPE is additive, so a key cached
 * at position s lands at position s + Delta_c.  Values are not touched.
 *   k_src, k_dst   dev [n_batch][L_ctx, Hkv, d]; batch b starts at b * batch_stride elements
 *                  (n_batch > 1 is the all-layers case: the same chunk table for every layer);
 *                  k_dst may equal k_src (in place), otherwise the two must not overlap
 *   chunk_offsets  host [n_chunks + 1], [0] = 0, non-decreasing, [n_chunks] = L_ctx
 *   chunk_src_pos0 host [n_chunks]: position the chunk's first token was cached at
 *   chunk_dst_pos0 host [n_chunks], or NULL: chunk c lands at chunk_offsets[c] + dst_base
 * Arithmetic: fp32 on cos/sin rounded from fp64; output rounded to dtype (nearest-even). */
fr_status fr_rope_shift(fr_ctx* ctx, const void* k_src, void* k_dst, const int32_t* chunk_offsets,
                        const int32_t* chunk_src_pos0, const int32_t* chunk_dst_pos0,
                        int32_t dst_base, int32_t n_chunks, int32_t n_batch,
                        int64_t src_batch_stride, int64_t dst_batch_stride, void* stream);

/* Query-Guided Selection (Sec. 3.2) and the Q index (Sec. 4.3).
 * score[j] = sum over query heads h and question tokens i of w[h, i, j], where w is the attention
 * weight of question query (i, h) on context key j under `norm`; then the k highest scores are
 * chosen (equal scores: lower index first) and
 *   q_index_out = ascending(chosen) ++ [L_ctx, L_ctx + 1, ..., L_ctx + nq - 1].
 *   q_question  dev [nq, Hq, d]: the question's queries, already rotated at positions L_ctx..
 *   k_ctx       dev [L_ctx, Hkv, d]: context keys at their global positions (fr_rope_shift output)
 *   chunk_offsets host [n_chunks + 1] as above (used by FR_NORM_PER_CHUNK; L_ctx = last entry)
 *   k           number of context tokens to choose, 0 <= k <= L_ctx
 *   scores_out  dev [L_ctx] fp32, or NULL
 *   q_index_out dev [k + nq] int32
 * No causal mask is involved: every context key precedes every question token. */
fr_status fr_score_select(fr_ctx* ctx, const void* q_question, int32_t nq, const void* k_ctx,
                          const int32_t* chunk_offsets, int32_t n_chunks, int64_t k, int32_t norm,
                          float* scores_out, int32_t* q_index_out, void* stream);

/* Query-Guided Selection over a chunk store that is shared between queries and never written (Sec. 4.3): the
 * same scores and Q index as fr_rope_shift followed by fr_score_select, without the per-query copy of the keys.
 * Chunk c of the prompt (positions chunk_offsets[c] .. chunk_offsets[c+1] - 1) is read from store rows
 * chunk_store_row0[c] .., and its keys are moved from the positions they were cached at (chunk_src_pos0[c] ..) to
 * their prompt positions on the way into the kernels (Appendix A; same arithmetic as fr_rope_shift).
 *   k_store  dev [n_store_rows, Hkv, d], read only
 *   chunk_offsets, chunk_store_row0, chunk_src_pos0  host, as in fr_sparse_prefill_attn_shared
 *   norm     FR_NORM_PER_CHUNK or FR_NORM_GLOBAL
 * Everything else as in fr_score_select.  Contexts the tiled kernels do not take (fp32, head_dim 64, group sizes
 * other than 1, 2, 4, 8) gather the shifted keys into the context's workspace and run the generic kernel. */
fr_status fr_score_select_shared(fr_ctx* ctx, const void* q_question, int32_t nq, const void* k_store,
                                 int64_t n_store_rows, const int32_t* chunk_offsets, const int32_t* chunk_store_row0,
                                 const int32_t* chunk_src_pos0, int32_t n_chunks, int64_t k, int32_t norm,
                                 float* scores_out, int32_t* q_index_out, void* stream);

/* Only the selection half of the call above, over scores the caller already has (any selector:
 * for example the KV deviation of eq. 7-8).  scores dev [n] fp32 (finite), q_index_out dev [k + nq]. */
fr_status fr_select_topk(fr_ctx* ctx, const float* scores, int64_t n, int64_t k, int32_t nq,
                         int32_t* q_index_out, void* stream);

/* fr_select_topk for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It needs no context and calls no allocating routine: the scratch of the
 * multi-workgroup selection (about 4.2 MB: state, histograms, per-tile status words, candidate list) is a static
 * device array inside the library, one copy per GPU, held until the process ends.  Same kernels and same result as
 * fr_select_topk.
 *   ctx     NULL, or a context that only receives the error message of a failing call (fr_last_error)
 *   scores, n, k, nq, q_index_out, stream: as in fr_select_topk; the tensors live on the current device, which is
 *           also the stream's
 * n > FR_SELECT_STATIC_MAX_SCORES is refused with FR_ERR_WORKSPACE before anything is launched.  The array's address
 * is resolved at the first call on a device (or by fr_create on that device), so make one of the two eagerly before
 * capturing a graph.  All calls on one GPU share that GPU's array: calls that overlap in time (different streams)
 * race; calls on one stream are ordered and each clears what it needs. */
#define FR_SELECT_STATIC_MAX_SCORES (1 << 24)
fr_status fr_select_topk_static(fr_ctx* ctx, const float* scores, int64_t n, int64_t k, int32_t nq,
                                int32_t* q_index_out, void* stream);

/* KV deviation of one layer (eq. 7): deviation_out[t] = sum over the n_kv_heads * head_dim components c of
 * (kv_a[t, c] - kv_b[t, c])^2, accumulated in fp32.  Followed by fr_select_topk it is the CacheBlend selector
 * (eq. 8), which the paper compares Query-Guided Selection against.  The paper takes the key half of layer 2.
 *   kv_a, kv_b     dev [n_tokens, Hkv, d] in the context's dtype, 16-byte aligned (e.g. the keys of full
 *                  attention and the cached keys of the same tokens); read only
 *   deviation_out  dev [n_tokens] fp32
 * n_tokens = 0 is a no-op.  Errors: FR_ERR_INVALID_ARG (NULL or misaligned pointer, n_tokens < 0 or > 2^31 - 1). */
fr_status fr_kv_deviation(fr_ctx* ctx, const void* kv_a, const void* kv_b, int64_t n_tokens, float* deviation_out,
                          void* stream);

/* Sparse prefill attention (eq. 9, Sec. 4.3).  Row r holds the query of the token at position
 * q_index[r]; it attends to every key at a position <= q_index[r].  The key/value at a position
 * listed in q_index is the recomputed one (k_new/v_new row of that token), every other position
 * reads the cache: the stale cache entries of recomputed tokens are never read.
 *   q_rows   dev [R, Hq, d]
 *   q_index  dev [R] int32, strictly ascending, every entry < L
 *   k_cache, v_cache dev [L, Hkv, d] (read only)
 *   k_new, v_new     dev [R, Hkv, d], or both NULL: the cache already holds the fresh rows
 *   out      dev [R, Hq, d]
 *   lse_out  dev [R, Hq] fp32 natural-log-sum-exp of the scaled logits, or NULL
 * Arithmetic: products of dtype inputs accumulated in fp32, softmax in fp32, out rounded to dtype. */
fr_status fr_sparse_prefill_attn(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                 const void* k_cache, const void* v_cache, int64_t L,
                                 const void* k_new, const void* v_new, void* out, float* lse_out,
                                 void* stream);

/* fr_sparse_prefill_attn followed by fr_kv_scatter in one call (the write-back fused into the attention's tile
 * packing pass): same output, and afterwards k_cache[q_index[r]] = k_new[r], v_cache[q_index[r]] = v_new[r].
 * k_new / v_new are required; k_cache / v_cache are read and written. */
fr_status fr_sparse_prefill_attn_writeback(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                           void* k_cache, void* v_cache, int64_t L, const void* k_new,
                                           const void* v_new, void* out, float* lse_out, void* stream);

/* Sparse prefill attention over a shared chunk store (Sec. 4.3: the chunk caches are shared by the queries and never
 * modified; the recomputed K/V of a query live in its own page).  Same result as fr_rope_shift into a per-query
 * cache followed by fr_sparse_prefill_attn and fr_kv_scatter, without the per-query copy and without the scatter:
 * prompt position j of chunk c (chunk_offsets[c] <= j < chunk_offsets[c+1]) reads store row
 * chunk_store_row0[c] + j - chunk_offsets[c], its key moved from the position it was cached at
 * (chunk_src_pos0[c] + j - chunk_offsets[c]) to j while the tile is loaded; positions listed in q_index read
 * k_new / v_new (the page) instead, and the store's entries of those tokens are never read.
 *   k_store, v_store   dev [n_store_rows, Hkv, d], read only
 *   chunk_offsets      host [n_chunks + 1], prompt positions as in fr_rope_shift; L_ctx = last entry <= L
 *   chunk_store_row0, chunk_src_pos0   host [n_chunks]
 *   L                  prompt length; every position in [L_ctx, L) must be listed in q_index
 *   q_rows, q_index, R, k_new, v_new (both required), out, lse_out: as in fr_sparse_prefill_attn
 * Errors as fr_sparse_prefill_attn, plus FR_ERR_INVALID_ARG for chunk rows outside the store.  Contexts the tiled
 * kernels do not take (fp32, head_dim 64, group sizes other than 1, 2, 4, 8) gather the query's shifted keys and its
 * values into the context's workspace (2 x max_tokens rows, part of fr_workspace_bytes) and run the generic kernel. */
fr_status fr_sparse_prefill_attn_shared(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                        const void* k_store, const void* v_store, int64_t n_store_rows,
                                        const int32_t* chunk_offsets, const int32_t* chunk_store_row0,
                                        const int32_t* chunk_src_pos0, int32_t n_chunks, int64_t L, const void* k_new,
                                        const void* v_new, void* out, float* lse_out, void* stream);

/* The same for several queries in one call (Sec. 4.3: queries that retrieve chunks of one store are served
 * together; each has its own chunk list, Q index, page of fresh rows and output).  All queries of the call share one
 * attention launch (groups of 16), which fills the chip where a single sparse query cannot; results equal those of
 * fr_sparse_prefill_attn_shared query by query.
 *   queries    host [n_queries]: the per-query arguments of fr_sparse_prefill_attn_shared (host and device pointers
 *              as there); a query with R = 0 is skipped
 *   workspace  dev, 256-byte aligned, at least fr_shared_batch_workspace_bytes(ctx, n_queries, max over queries of L)
 *              bytes: tile images, index maps and rotation tables of the queries in flight (78 MB per 17k-token
 *              query); owned by the caller, contents undefined afterwards, must stay untouched until the call's
 *              work on the stream has finished
 * Every query is validated before the first launch.  Errors as fr_sparse_prefill_attn_shared (the message names
 * the query), plus FR_ERR_WORKSPACE when workspace_bytes is too small.  Contexts served by the generic kernel run
 * the queries one after the other from the context's own workspace: fr_shared_batch_workspace_bytes is 0 for them
 * and workspace may be NULL. */
typedef struct {
    const void* q_rows;                /* dev [R, Hq, d] */
    const int32_t* q_index;            /* dev [R] */
    int32_t R;
    const int32_t* chunk_offsets;      /* host [n_chunks + 1] */
    const int32_t* chunk_store_row0;   /* host [n_chunks] */
    const int32_t* chunk_src_pos0;     /* host [n_chunks] */
    int32_t n_chunks;
    int64_t L;
    const void* k_new;                 /* dev [R, Hkv, d] */
    const void* v_new;                 /* dev [R, Hkv, d] */
    void* out;                         /* dev [R, Hq, d] */
    float* lse_out;                    /* dev [R, Hq] or NULL */
} fr_shared_query;
int64_t fr_shared_batch_workspace_bytes(const fr_ctx* ctx, int32_t n_queries, int64_t max_L);
fr_status fr_sparse_prefill_attn_shared_batch(fr_ctx* ctx, const fr_shared_query* queries, int32_t n_queries,
                                              const void* k_store, const void* v_store, int64_t n_store_rows,
                                              void* workspace, int64_t workspace_bytes, void* stream);

/* Batch decoding attention over shared chunk caches and per-query exclusive pages (Sec. 4.3; decoding step of
 * Sec. 2.1).  The chunk store (k_shared, v_shared) is shared by all queries of the batch and is never written.
 * Query b's prompt consists of the store segments seg_*[seg_offsets[b] .. seg_offsets[b+1]): rows
 * [seg_row0, seg_row0 + seg_len) of the store, whose keys were cached seg_delta positions before the place they
 * take in this prompt (Appendix A: they are used as if rotated by seg_delta; the kernel rotates the query by
 * -seg_delta instead, so no copy of the keys is made).  Store rows whose bit is set in query b's mask are skipped:
 * they are the query's recomputed tokens, whose fresh K/V sit in its exclusive page together with the K/V of its
 * question and of its generated tokens (all page keys rotated at their positions in the prompt; the decoding
 * token's own entry included).  out[b, h] = softmax over all those keys of (q[b, h] . key / sqrt(d)) applied to
 * the values.
 *   q            dev [n_queries, Hq, d]: the decoding tokens' queries, rotated at their positions
 *   k_shared, v_shared  dev [n_shared_rows, Hkv, d]
 *   seg_offsets  dev [n_queries + 1] int32, ascending, seg_offsets[0] = 0, last = n_segments
 *   seg_row0, seg_len, seg_delta  dev [n_segments] int32
 *   stale_bits   dev [n_queries][stale_words] uint32, bit (r & 31) of word r >> 5 = store row r is stale for the
 *                query; NULL = no row is stale (see fr_mark_stale_rows)
 *   k_pages, v_pages  dev [n_queries][page_stride_rows][Hkv][d]; page_len dev [n_queries] int32 rows in use
 *   out          dev [n_queries, Hq, d];  lse_out dev [n_queries, Hq] fp32 natural-log normalisers, or NULL
 * All tensors 16-byte aligned, in the context's dtype.  The descriptor arrays live on the device, so the host does
 * not check their contents: the kernels clamp every row range to its tensor (rows outside are not read and do not
 * count).  Errors: FR_ERR_INVALID_ARG (NULL / misaligned pointers, negative sizes), FR_ERR_WORKSPACE
 * (n_segments + n_queries > 4096). */
fr_status fr_decode_attn(fr_ctx* ctx, const void* q, int32_t n_queries, const void* k_shared, const void* v_shared,
                         int64_t n_shared_rows, const int32_t* seg_offsets, const int32_t* seg_row0,
                         const int32_t* seg_len, const int32_t* seg_delta, int32_t n_segments,
                         const uint32_t* stale_bits, int64_t stale_words, const void* k_pages, const void* v_pages,
                         int64_t page_stride_rows, const int32_t* page_len, void* out, float* lse_out, void* stream);

/* Sets, in one query's mask of fr_decode_attn, the bits of the listed store rows (its recomputed tokens).
 *   stale_bits dev [n_words] uint32 (one query's words); rows dev [n_rows] int32; clear != 0 zeroes the words first.
 * Rows outside [0, 32 * n_words) are ignored. */
fr_status fr_mark_stale_rows(fr_ctx* ctx, uint32_t* stale_bits, int64_t n_words, const int32_t* rows, int32_t n_rows,
                             int32_t clear, void* stream);

/* Write-back (Sec. 4.3): k_cache[q_index[r]] = k_new[r], v_cache[q_index[r]] = v_new[r],
 * bit-exact copies; other rows are not touched.  Shapes as above. */
fr_status fr_kv_scatter(fr_ctx* ctx, const void* k_new, const void* v_new, const int32_t* q_index,
                        int32_t R, void* k_cache, void* v_cache, int64_t L, void* stream);

/* ---- The model steps around the path, for the recomputed rows only (eq. 9: the sparse prefill feeds the
 * rows cat(X[C_idx], Q) through every layer).  bf16 contexts only.  All matrices are row-major with the
 * contraction dimension contiguous; M = number of rows (any), N and F multiples of 128, K a multiple of 64.
 * Products accumulate in fp32 and are rounded once to bf16 after the fused epilogue. ---------------------- */

/* out[r, :] = x[r, :] * rsqrt(mean(x[r, :]^2) + eps) * gain.   x, out dev [R, hidden]; gain dev [hidden];
 * hidden a multiple of 8. */
fr_status fr_rmsnorm(fr_ctx* ctx, const void* x, const void* gain, int32_t R, int32_t hidden, float eps, void* out,
                     void* stream);

/* out = a . w^T (+ residual).   a dev [M, K]; w dev [N, K]; residual dev [M, N] or NULL; out dev [M, N]
 * (out may equal residual). */
fr_status fr_linear(fr_ctx* ctx, const void* a, const void* w, int32_t M, int32_t N, int32_t K, const void* residual,
                    void* out, void* stream);

/* out[:, j] = silu(a . w_gate_up[2j]) * (a . w_gate_up[2j + 1]): gate and up projections with their rows
 * interleaved in one weight matrix.   a dev [M, K]; w_gate_up dev [2 F, K]; out dev [M, F]. */
fr_status fr_linear_swiglu(fr_ctx* ctx, const void* a, const void* w_gate_up, int32_t M, int32_t F, int32_t K,
                           void* out, void* stream);

/* Q/K/V projection of the recomputed rows with the rotary embedding of each row's own position (the position
 * list of eq. 9, i.e. the Q index) applied to q and k; rope parameters from the context's layer description.
 *   a dev [M, K]; w_qkv dev [(Hq + 2 Hkv) d, K]: query heads, then key heads, then value heads;
 *   positions dev [M] int32;  q_out dev [M, Hq, d];  k_out, v_out dev [M, Hkv, d]. */
fr_status fr_qkv_rope(fr_ctx* ctx, const void* a, const void* w_qkv, int32_t M, int32_t K, const int32_t* positions,
                      void* q_out, void* k_out, void* v_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FUSIONRAG_H */
