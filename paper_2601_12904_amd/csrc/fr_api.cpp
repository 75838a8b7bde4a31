// C ABI of libfusionrag: argument validation, workspace, dispatch.  No kernels here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <new>

#include "fr_internal.hpp"

#include <string>
#include <vector>

using namespace fr;

namespace {

fr_status fail(fr_ctx* ctx, fr_status st, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return st;
}

fr_status hip_fail(fr_ctx* ctx, const char* what, hipError_t e) {
    return fail(ctx, FR_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Validates a host chunk table and copies it into the by-value form.
fr_status read_chunks(fr_ctx* ctx, const int32_t* offs, int32_t n_chunks, int64_t max_ctx, ChunkTable* ct,
                      int* max_len) {
    if (!offs) return fail(ctx, FR_ERR_INVALID_ARG, "chunk_offsets is NULL");
    if (n_chunks < 0) return fail(ctx, FR_ERR_INVALID_ARG, "n_chunks = %d is negative", n_chunks);
    if (n_chunks > ctx->max_chunks)
        return fail(ctx, FR_ERR_WORKSPACE, "n_chunks = %d exceeds the context's max_chunks = %d", n_chunks,
                    ctx->max_chunks);
    if (offs[0] != 0) return fail(ctx, FR_ERR_INVALID_ARG, "chunk_offsets[0] = %d, must be 0", offs[0]);
    int ml = 0;
    ct->n = n_chunks;
    ct->off[0] = 0;
    for (int c = 0; c < n_chunks; ++c) {
        if (offs[c + 1] < offs[c])
            return fail(ctx, FR_ERR_INVALID_ARG, "chunk_offsets not ascending at %d: %d then %d", c, offs[c],
                        offs[c + 1]);
        ct->off[c + 1] = offs[c + 1];
        if (offs[c + 1] - offs[c] > ml) ml = offs[c + 1] - offs[c];
    }
    if ((int64_t)offs[n_chunks] > max_ctx)
        return fail(ctx, FR_ERR_WORKSPACE, "L_ctx = %d exceeds the context's max_tokens = %lld", offs[n_chunks],
                    (long long)max_ctx);
    if (max_len) *max_len = ml;
    return FR_OK;
}

fr_status need_device(fr_ctx* ctx) {
    if (!ctx->has_device) return fail(ctx, FR_ERR_DEVICE, "no HIP device: this context can only validate arguments");
    return FR_OK;
}

}  // namespace

extern "C" {

int64_t fr_topk_count(int64_t L_ctx, double ratio) {
    if (L_ctx <= 0 || !(ratio > 0.0)) return 0;
    const double v = floor(ratio * (double)L_ctx + 0.5);
    if (v >= (double)L_ctx) return L_ctx;
    return (int64_t)v;
}

fr_status fr_create(const fr_layer_desc* desc, int64_t max_tokens, int32_t max_chunks, int32_t max_question_tokens,
                    fr_ctx** out) {
    if (!out) return FR_ERR_INVALID_ARG;
    *out = nullptr;
    if (!desc) return FR_ERR_INVALID_ARG;
    if (desc->n_q_heads <= 0 || desc->n_kv_heads <= 0 || desc->n_q_heads % desc->n_kv_heads != 0)
        return FR_ERR_INVALID_ARG;
    if (desc->dtype != FR_F32 && desc->dtype != FR_BF16) return FR_ERR_INVALID_ARG;
    if (desc->rope_layout != FR_ROPE_INTERLEAVED && desc->rope_layout != FR_ROPE_HALF) return FR_ERR_INVALID_ARG;
    if (desc->rope_index_base != 0 && desc->rope_index_base != 1) return FR_ERR_INVALID_ARG;
    if (!(desc->rope_base > 1.0) || !isfinite(desc->rope_base)) return FR_ERR_INVALID_ARG;
    if (max_tokens <= 0 || max_tokens > (int64_t)1 << 30) return FR_ERR_INVALID_ARG;
    if (max_chunks <= 0 || max_question_tokens < 0 || max_question_tokens > max_tokens) return FR_ERR_INVALID_ARG;
    if (desc->head_dim != 64 && desc->head_dim != 128) return FR_ERR_UNSUPPORTED;
    if (max_chunks > FR_MAX_CHUNKS) return FR_ERR_UNSUPPORTED;
    if (desc->n_q_heads > 1024) return FR_ERR_UNSUPPORTED;

    fr_ctx* ctx = new (std::nothrow) fr_ctx();
    if (!ctx) return FR_ERR_WORKSPACE;
    Shape& s = ctx->shape;
    s.Hq = desc->n_q_heads;
    s.Hkv = desc->n_kv_heads;
    s.d = desc->head_dim;
    s.G = s.Hq / s.Hkv;
    s.dtype = desc->dtype;
    s.esize = desc->dtype == FR_BF16 ? 2 : 4;
    s.rope_base = desc->rope_base;
    s.rope_layout = desc->rope_layout;
    s.rope_index_base = desc->rope_index_base;
    ctx->max_tokens = max_tokens;
    ctx->max_chunks = max_chunks;
    ctx->max_q = max_question_tokens;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        ctx->has_device = false;
        *out = ctx;
        return FR_OK;
    }
    if (hipGetDevice(&ctx->device) != hipSuccess) {
        delete ctx;
        return FR_ERR_DEVICE;
    }

    // carve the workspace
    Workspace& w = ctx->ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += round_up(bytes, 256);
        return o;
    };
    const size_t o_table = take((size_t)max_chunks * (s.d / 2) * sizeof(float2));
    // normalisers per (head, chunk or whole context, question token); the tiled kernels pad every row of
    // G x question tokens to a multiple of 64
    const size_t o_lse = take((size_t)s.Hkv * (max_chunks + 1) * ((size_t)s.G * (max_question_tokens > 0 ? max_question_tokens : 1) + 63) * 4);
    const size_t o_col = take((size_t)s.Hkv * max_tokens * 4);
    const size_t o_scores = take((size_t)max_tokens * 4);
    const size_t o_inv = take((size_t)max_tokens * 4);
    const size_t o_srow = take((size_t)max_tokens * 4);
    const size_t o_cid = take((size_t)max_tokens * 4);
    const size_t o_sel = take(select_workspace_bytes());
    const size_t o_qsum = take(score_raw_workspace_bytes(s));
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) {
        delete ctx;
        return FR_ERR_DEVICE;
    }
    w.n_cu = prop.multiProcessorCount;
    w.attn_flags_elems = (size_t)(max_tokens / 32 + 1) * s.Hkv;   // one per (row tile of >= 32 rows, KV head)
    const size_t o_flags = take(w.attn_flags_elems * 4);
    w.kv_images_bytes = (s.dtype == FR_BF16 && s.d == 128) ? (size_t)((max_tokens + 63) / 64) * s.Hkv * 36864 : 0;
    const size_t o_img = take(w.kv_images_bytes);
    w.attn_partials_bytes = (s.dtype == FR_BF16 && s.d == 128) ? attn_mfma_partials_bytes(s, max_tokens) : 0;
    const size_t o_part = take(w.attn_partials_bytes);
    const size_t o_dpart = take(decode_partials_bytes(s));
    const size_t o_drot = take(decode_rot_table_bytes(s));
    const size_t o_rr = take((size_t)max_tokens * (s.d / 2) * sizeof(float2));
    w.gemm_partials_bytes = (s.dtype == FR_BF16) ? gemm_partials_bytes() : 0;
    const size_t o_gp = take(w.gemm_partials_bytes);
    // shapes without a tiled path serve the shared chunk store through a gathered copy of the query's keys and values
    const size_t store_copy_bytes =
        (attn_mfma_supported(s) && score_mfma_supported(s)) ? 0 : (size_t)max_tokens * s.Hkv * s.d * s.esize;
    const size_t o_sk = take(store_copy_bytes);
    const size_t o_sv = take(store_copy_bytes);
    w.bytes = off;
    hipError_t e = hipMalloc((void**)&w.base, w.bytes);
    if (e != hipSuccess) {
        delete ctx;
        return FR_ERR_WORKSPACE;
    }
    w.rope_table = (float2*)(w.base + o_table);
    w.lse = (float*)(w.base + o_lse);
    w.col_partial = (float*)(w.base + o_col);
    w.scores = (float*)(w.base + o_scores);
    w.inv_index = (int32_t*)(w.base + o_inv);
    w.store_row_map = (int32_t*)(w.base + o_srow);
    w.chunk_id_map = (int32_t*)(w.base + o_cid);
    w.select_tmp = (uint32_t*)(w.base + o_sel);
    if (hipMemset(w.select_tmp, 0, select_zeroed_bytes()) != hipSuccess) {   // the selection expects (and leaves) it zero
        (void)hipFree(w.base);
        w.base = nullptr;
        delete ctx;
        return FR_ERR_DEVICE;
    }
    w.qsum = (float*)(w.base + o_qsum);
    w.attn_flags = (int32_t*)(w.base + o_flags);
    w.kv_images = (unsigned char*)(w.base + o_img);
    w.attn_partials = (float*)(w.base + o_part);
    w.decode_partials = (float*)(w.base + o_dpart);
    w.decode_rot = (float2*)(w.base + o_drot);
    w.rope_rows = (float2*)(w.base + o_rr);
    w.gemm_partials = w.gemm_partials_bytes ? (float*)(w.base + o_gp) : nullptr;
    w.store_k = store_copy_bytes ? (void*)(w.base + o_sk) : nullptr;
    w.store_v = store_copy_bytes ? (void*)(w.base + o_sv) : nullptr;
    ctx->has_device = true;
    (void)select_static_prepare();   // this device's static scratch of fr_select_topk_static (no allocation; failure is reported there)
    *out = ctx;
    return FR_OK;
}

void fr_destroy(fr_ctx* ctx) {
    if (!ctx) return;
    for (int i = 0; i < KernelTimer::MAX_SLOTS; ++i) {
        if (ctx->attn_timer.start[i]) (void)hipEventDestroy(ctx->attn_timer.start[i]);
        if (ctx->attn_timer.stop[i]) (void)hipEventDestroy(ctx->attn_timer.stop[i]);
    }
    if (ctx->ws.base) (void)hipFree(ctx->ws.base);
    delete ctx;
}

const char* fr_last_error(const fr_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int64_t fr_workspace_bytes(const fr_ctx* ctx) { return ctx ? (int64_t)ctx->ws.bytes : 0; }

fr_status fr_set_option(fr_ctx* ctx, int32_t option, int64_t value) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    switch (option) {
        case FR_OPT_ATTN_SOFTMAX:
            if (value != FR_ATTN_SOFTMAX_AUTO && value != FR_ATTN_SOFTMAX_RUNNING_MAX)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_ATTN_SOFTMAX: unknown value %lld", (long long)value);
            ctx->attn_softmax_mode = (int)value;
            return FR_OK;
        case FR_OPT_DECODE_KERNEL:
            if (value != FR_DECODE_KERNEL_AUTO && value != FR_DECODE_KERNEL_GENERIC)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_DECODE_KERNEL: unknown value %lld", (long long)value);
            ctx->decode_generic = (value == FR_DECODE_KERNEL_GENERIC) ? 1 : 0;
            return FR_OK;
        case FR_OPT_ATTN_KERNEL_TIMER: {
            if (value < 0 || value > KernelTimer::MAX_SLOTS)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_ATTN_KERNEL_TIMER: %lld slots outside [0, %d]", (long long)value,
                            KernelTimer::MAX_SLOTS);
            fr_status st = need_device(ctx);
            if (st != FR_OK) return st;
            KernelTimer& t = ctx->attn_timer;
            for (int i = 0; i < (int)value; ++i) {   // events are created once and kept until fr_destroy
                if (!t.start[i] && (hipEventCreate(&t.start[i]) != hipSuccess || hipEventCreate(&t.stop[i]) != hipSuccess))
                    return hip_fail(ctx, "event creation", hipGetLastError());
            }
            t.n_slots = (int)value;
            t.n_recorded = 0;
            return FR_OK;
        }
        case FR_OPT_GEMM_TILE:
            if (value != 0 && value != 128 && value != 256)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_GEMM_TILE: %lld is not 0, 128 or 256", (long long)value);
            ctx->gemm_tuning.tile = (int)value;
            return FR_OK;
        case FR_OPT_GEMM_TAIL_SPLIT:
            if (value != 0 && value != 1)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_GEMM_TAIL_SPLIT: %lld is not 0 or 1", (long long)value);
            ctx->gemm_tuning.tail_split = (int)value;
            return FR_OK;
        case FR_OPT_ATTN_SPLIT:
            if (value != FR_ATTN_SPLIT_AUTO && value != FR_ATTN_SPLIT_OFF && value != FR_ATTN_SPLIT_ON)
                return fail(ctx, FR_ERR_INVALID_ARG, "FR_OPT_ATTN_SPLIT: unknown value %lld", (long long)value);
            ctx->attn_split_mode = (int)value;
            return FR_OK;
        default:
            return fail(ctx, FR_ERR_INVALID_ARG, "unknown option %d", option);
    }
}

fr_status fr_attn_kernel_times(fr_ctx* ctx, float* ms_out, int32_t capacity, int32_t* n_out) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (!ms_out || !n_out || capacity < 0) return fail(ctx, FR_ERR_INVALID_ARG, "ms_out / n_out is NULL or capacity < 0");
    KernelTimer& t = ctx->attn_timer;
    const int64_t have = t.n_recorded < t.n_slots ? t.n_recorded : t.n_slots;
    const int n = (int)(have < capacity ? have : capacity);
    for (int i = 0; i < n; ++i) {   // oldest of the kept launches first
        const int slot = (int)((t.n_recorded - have + i) % t.n_slots);
        if (hipEventSynchronize(t.stop[slot]) != hipSuccess ||
            hipEventElapsedTime(&ms_out[i], t.start[slot], t.stop[slot]) != hipSuccess)
            return hip_fail(ctx, "reading kernel timer events", hipGetLastError());
    }
    *n_out = n;
    return FR_OK;
}

fr_status fr_rope_shift(fr_ctx* ctx, const void* k_src, void* k_dst, const int32_t* chunk_offsets,
                        const int32_t* chunk_src_pos0, const int32_t* chunk_dst_pos0, int32_t dst_base,
                        int32_t n_chunks, int32_t n_batch, int64_t src_batch_stride, int64_t dst_batch_stride,
                        void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    ChunkTable ct;
    int max_len = 0;
    fr_status st = read_chunks(ctx, chunk_offsets, n_chunks, ctx->max_tokens, &ct, &max_len);
    if (st != FR_OK) return st;
    if (!chunk_src_pos0) return fail(ctx, FR_ERR_INVALID_ARG, "chunk_src_pos0 is NULL");
    if (n_batch < 0 || n_batch > 65535) return fail(ctx, FR_ERR_INVALID_ARG, "n_batch = %d out of range", n_batch);
    const int64_t L_ctx = ct.off[ct.n];
    const int64_t layer_elems = L_ctx * s.Hkv * s.d;
    if (n_batch > 1 && (src_batch_stride < layer_elems || dst_batch_stride < layer_elems))
        return fail(ctx, FR_ERR_INVALID_ARG, "batch stride smaller than one layer (%lld elements)",
                    (long long)layer_elems);
    if (n_batch > 1 && ((src_batch_stride * s.esize) % 16 != 0 || (dst_batch_stride * s.esize) % 16 != 0))
        return fail(ctx, FR_ERR_INVALID_ARG, "batch strides must keep 16-byte alignment");
    if (L_ctx > 0 && n_batch > 0) {
        if (!k_src || !k_dst) return fail(ctx, FR_ERR_INVALID_ARG, "k_src / k_dst is NULL");
        if (!aligned16(k_src) || !aligned16(k_dst))
            return fail(ctx, FR_ERR_INVALID_ARG, "k_src / k_dst must be 16-byte aligned");
        if (k_src != k_dst) {
            const char* a = (const char*)k_src;
            const char* b = (const char*)k_dst;
            const int64_t span_a = ((int64_t)(n_batch - 1) * src_batch_stride + layer_elems) * s.esize;
            const int64_t span_b = ((int64_t)(n_batch - 1) * dst_batch_stride + layer_elems) * s.esize;
            if (a < b + span_b && b < a + span_a)
                return fail(ctx, FR_ERR_INVALID_ARG, "k_src and k_dst overlap without being equal");
        }
    }
    ChunkDeltas dl;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t dst = chunk_dst_pos0 ? (int64_t)chunk_dst_pos0[c] : (int64_t)ct.off[c] + dst_base;
        const int64_t delta = dst - (int64_t)chunk_src_pos0[c];
        if (delta > INT32_MAX || delta < INT32_MIN) return fail(ctx, FR_ERR_INVALID_ARG, "position delta overflows");
        dl.delta[c] = (int32_t)delta;
    }
    if (L_ctx == 0 || n_batch == 0) return FR_OK;
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    hipError_t e = launch_rope_table(s, dl, n_chunks, ctx->ws.rope_table, hs);
    if (e != hipSuccess) return hip_fail(ctx, "rope table launch", e);
    e = launch_rope_shift(s, k_src, k_dst, ct, max_len, ctx->ws.rope_table, n_batch, src_batch_stride,
                          dst_batch_stride, nullptr, hs);
    if (e != hipSuccess) return hip_fail(ctx, "rope shift launch", e);
    return FR_OK;
}

fr_status fr_select_topk(fr_ctx* ctx, const float* scores, int64_t n, int64_t k, int32_t nq, int32_t* q_index_out,
                         void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (n < 0 || n > INT32_MAX - (int64_t)(nq > 0 ? nq : 0))
        return fail(ctx, FR_ERR_INVALID_ARG, "n = %lld out of range", (long long)n);
    if (nq < 0) return fail(ctx, FR_ERR_INVALID_ARG, "nq = %d is negative", nq);
    if (k < 0 || k > n) return fail(ctx, FR_ERR_INVALID_ARG, "k = %lld outside [0, n = %lld]", (long long)k, (long long)n);
    if (k + nq == 0) return FR_OK;
    if (!q_index_out) return fail(ctx, FR_ERR_INVALID_ARG, "q_index_out is NULL");
    if (n > 0 && k > 0 && !scores) return fail(ctx, FR_ERR_INVALID_ARG, "scores is NULL");
    if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(q_index_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "scores / q_index_out must be 4-byte aligned");
    fr_status st = need_device(ctx);
    if (st != FR_OK) return st;
    hipError_t e = launch_select(scores, n, k, nq, q_index_out, ctx->ws.select_tmp, select_workspace_bytes(), (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "select launch", e);
    return FR_OK;
}

fr_status fr_kv_deviation(fr_ctx* ctx, const void* kv_a, const void* kv_b, int64_t n_tokens, float* deviation_out,
                          void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (n_tokens < 0 || n_tokens > INT32_MAX)
        return fail(ctx, FR_ERR_INVALID_ARG, "n_tokens = %lld out of range", (long long)n_tokens);
    if (n_tokens == 0) return FR_OK;
    if (!kv_a || !kv_b || ((reinterpret_cast<uintptr_t>(kv_a) | reinterpret_cast<uintptr_t>(kv_b)) & 15u))
        return fail(ctx, FR_ERR_INVALID_ARG, "kv_a / kv_b is NULL or not 16-byte aligned");
    if (!deviation_out || (reinterpret_cast<uintptr_t>(deviation_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "deviation_out is NULL or not 4-byte aligned");
    fr_status st = need_device(ctx);
    if (st != FR_OK) return st;
    hipError_t e = launch_kv_deviation(ctx->shape, kv_a, kv_b, n_tokens, deviation_out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "kv deviation launch", e);
    return FR_OK;
}

fr_status fr_score_select(fr_ctx* ctx, const void* q_question, int32_t nq, const void* k_ctx,
                          const int32_t* chunk_offsets, int32_t n_chunks, int64_t k, int32_t norm, float* scores_out,
                          int32_t* q_index_out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    if (nq < 0) return fail(ctx, FR_ERR_INVALID_ARG, "nq = %d is negative", nq);
    if (nq > ctx->max_q) return fail(ctx, FR_ERR_WORKSPACE, "nq = %d exceeds max_question_tokens = %d", nq, ctx->max_q);
    ChunkTable ct;
    fr_status st = read_chunks(ctx, chunk_offsets, n_chunks, ctx->max_tokens - nq, &ct, nullptr);
    if (st != FR_OK) return st;
    const int64_t L_ctx = ct.off[ct.n];
    if (norm != FR_NORM_PER_CHUNK && norm != FR_NORM_GLOBAL && norm != FR_NORM_RAW)
        return fail(ctx, FR_ERR_INVALID_ARG, "unknown score norm %d", norm);
    if (k < 0 || k > L_ctx)
        return fail(ctx, FR_ERR_INVALID_ARG, "k = %lld outside [0, L_ctx = %lld]", (long long)k, (long long)L_ctx);
    if (k + nq > 0 && !q_index_out) return fail(ctx, FR_ERR_INVALID_ARG, "q_index_out is NULL");
    if (nq > 0 && (!q_question || !aligned16(q_question)))
        return fail(ctx, FR_ERR_INVALID_ARG, "q_question is NULL or not 16-byte aligned");
    if (L_ctx > 0 && (!k_ctx || !aligned16(k_ctx)))
        return fail(ctx, FR_ERR_INVALID_ARG, "k_ctx is NULL or not 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scores_out) & 3u) || (reinterpret_cast<uintptr_t>(q_index_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "scores_out / q_index_out must be 4-byte aligned");
    if (L_ctx == 0 && nq == 0) return FR_OK;
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    float* scores = scores_out ? scores_out : ctx->ws.scores;
    const bool need_scores = (scores_out != nullptr) || (k > 0 && k < L_ctx);
    if (L_ctx > 0 && need_scores) {
        hipError_t e;
        if (score_mfma_supported(s) && nq > 0 && norm != FR_NORM_RAW)
            e = launch_score_mfma(s, q_question, nq, k_ctx, ct, norm, ctx->ws, scores, hs);
        else if (norm == FR_NORM_RAW && score_raw_supported(s))
            e = launch_score_raw(s, q_question, nq, k_ctx, L_ctx, ctx->ws.qsum, scores, hs);
        else
            e = launch_score_simt(s, q_question, nq, k_ctx, ct, norm, ctx->ws, scores, hs);
        if (e != hipSuccess) return hip_fail(ctx, "score launch", e);
    }
    hipError_t e = launch_select(scores, L_ctx, k, nq, q_index_out, ctx->ws.select_tmp, select_workspace_bytes(), hs);
    if (e != hipSuccess) return hip_fail(ctx, "select launch", e);
    return FR_OK;
}

// Shapes the tiled kernels do not take: the query's keys (moved to their prompt positions, Appendix A) and, when
// v_store is given, its values are gathered from the chunk store into the workspace's [L, Hkv, d] copies, on which
// the generic kernels then run.  Values go through the same kernel with a rotation by zero positions, which is
// the identity in every arithmetic (cos 0 = 1, sin 0 = 0).  Rows [L_ctx, L) are cleared.
static fr_status gather_from_store(fr_ctx* ctx, const void* k_store, const void* v_store, const ChunkTable& ct,
                                   const int32_t* chunk_store_row0, const ChunkDeltas& dl, int64_t L, hipStream_t hs) {
    const Shape& s = ctx->shape;
    const int64_t L_ctx = ct.off[ct.n];
    ChunkRows rows{};
    int max_len = 0;
    for (int c = 0; c < ct.n; ++c) {
        rows.row0[c] = chunk_store_row0[c];
        max_len = std::max(max_len, ct.off[c + 1] - ct.off[c]);
    }
    hipError_t e = hipSuccess;
    if (v_store && L_ctx > 0) {
        const ChunkDeltas zero{};
        e = launch_rope_table(s, zero, ct.n, ctx->ws.rope_table, hs);
        if (e == hipSuccess) e = launch_rope_shift(s, v_store, ctx->ws.store_v, ct, max_len, ctx->ws.rope_table, 1, 0, 0, &rows, hs);
        if (e != hipSuccess) return hip_fail(ctx, "value gather launch", e);
    }
    if (L_ctx > 0) {
        e = launch_rope_table(s, dl, ct.n, ctx->ws.rope_table, hs);
        if (e == hipSuccess) e = launch_rope_shift(s, k_store, ctx->ws.store_k, ct, max_len, ctx->ws.rope_table, 1, 0, 0, &rows, hs);
        if (e != hipSuccess) return hip_fail(ctx, "key gather launch", e);
    }
    const int64_t row_words = (int64_t)s.Hkv * s.d * s.esize / 4;
    if (L > L_ctx) {
        e = launch_clear_words((uint32_t*)ctx->ws.store_k + L_ctx * row_words, (L - L_ctx) * row_words, hs);
        if (e == hipSuccess && v_store)
            e = launch_clear_words((uint32_t*)ctx->ws.store_v + L_ctx * row_words, (L - L_ctx) * row_words, hs);
        if (e != hipSuccess) return hip_fail(ctx, "clear launch", e);
    }
    return FR_OK;
}

fr_status fr_score_select_shared(fr_ctx* ctx, const void* q_question, int32_t nq, const void* k_store,
                                 int64_t n_store_rows, const int32_t* chunk_offsets, const int32_t* chunk_store_row0,
                                 const int32_t* chunk_src_pos0, int32_t n_chunks, int64_t k, int32_t norm,
                                 float* scores_out, int32_t* q_index_out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    if (nq < 0) return fail(ctx, FR_ERR_INVALID_ARG, "nq = %d is negative", nq);
    if (nq > ctx->max_q) return fail(ctx, FR_ERR_WORKSPACE, "nq = %d exceeds max_question_tokens = %d", nq, ctx->max_q);
    ChunkTable ct;
    fr_status st = read_chunks(ctx, chunk_offsets, n_chunks, ctx->max_tokens - nq, &ct, nullptr);
    if (st != FR_OK) return st;
    const int64_t L_ctx = ct.off[ct.n];
    if (norm != FR_NORM_PER_CHUNK && norm != FR_NORM_GLOBAL)
        return fail(ctx, FR_ERR_INVALID_ARG, "score norm %d: the shared-store scoring takes the two softmax scopes", norm);
    if (k < 0 || k > L_ctx)
        return fail(ctx, FR_ERR_INVALID_ARG, "k = %lld outside [0, L_ctx = %lld]", (long long)k, (long long)L_ctx);
    if (n_store_rows < 0) return fail(ctx, FR_ERR_INVALID_ARG, "n_store_rows is negative");
    if (n_chunks > 0 && (!chunk_store_row0 || !chunk_src_pos0))
        return fail(ctx, FR_ERR_INVALID_ARG, "chunk_store_row0 / chunk_src_pos0 is NULL");
    ChunkDeltas dl;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t len = (int64_t)ct.off[c + 1] - ct.off[c];
        if (chunk_store_row0[c] < 0 || (int64_t)chunk_store_row0[c] + len > n_store_rows)
            return fail(ctx, FR_ERR_INVALID_ARG, "chunk %d: store rows [%d, %lld) outside the store of %lld rows", c,
                        chunk_store_row0[c], (long long)chunk_store_row0[c] + len, (long long)n_store_rows);
        const int64_t delta = (int64_t)ct.off[c] - (int64_t)chunk_src_pos0[c];
        if (delta > INT32_MAX || delta < INT32_MIN) return fail(ctx, FR_ERR_INVALID_ARG, "position delta overflows");
        dl.delta[c] = (int32_t)delta;
    }
    if (k + nq > 0 && !q_index_out) return fail(ctx, FR_ERR_INVALID_ARG, "q_index_out is NULL");
    if (nq > 0 && (!q_question || !aligned16(q_question)))
        return fail(ctx, FR_ERR_INVALID_ARG, "q_question is NULL or not 16-byte aligned");
    if (L_ctx > 0 && (!k_store || !aligned16(k_store)))
        return fail(ctx, FR_ERR_INVALID_ARG, "k_store is NULL or not 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(scores_out) & 3u) || (reinterpret_cast<uintptr_t>(q_index_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "scores_out / q_index_out must be 4-byte aligned");
    if (L_ctx == 0 && nq == 0) return FR_OK;
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    float* scores = scores_out ? scores_out : ctx->ws.scores;
    const bool need_scores = (scores_out != nullptr) || (k > 0 && k < L_ctx);
    if (L_ctx > 0 && need_scores) {
        if (nq == 0) {   // no question rows: every score is an empty sum (the generic kernel writes the zeros; no key is read)
            hipError_t e = launch_score_simt(s, q_question, 0, k_store, ct, norm, ctx->ws, scores, hs);
            if (e != hipSuccess) return hip_fail(ctx, "score launch", e);
        } else if (!score_mfma_supported(s)) {   // no tiled kernel for this shape: gathered keys, generic kernel
            if ((st = gather_from_store(ctx, k_store, nullptr, ct, chunk_store_row0, dl, L_ctx, hs)) != FR_OK) return st;
            hipError_t e = launch_score_simt(s, q_question, nq, ctx->ws.store_k, ct, norm, ctx->ws, scores, hs);
            if (e != hipSuccess) return hip_fail(ctx, "score launch", e);
        } else {
            hipError_t e = launch_rope_table(s, dl, n_chunks, ctx->ws.rope_table, hs);
            if (e != hipSuccess) return hip_fail(ctx, "rope table launch", e);
            e = launch_score_mfma_shared(s, q_question, nq, k_store, ct, chunk_store_row0, ctx->ws.rope_table, norm, ctx->ws,
                                         scores, hs);
            if (e != hipSuccess) return hip_fail(ctx, "score launch", e);
        }
    }
    hipError_t e = launch_select(scores, L_ctx, k, nq, q_index_out, ctx->ws.select_tmp, select_workspace_bytes(), hs);
    if (e != hipSuccess) return hip_fail(ctx, "select launch", e);
    return FR_OK;
}

static fr_status check_rows(fr_ctx* ctx, int32_t R, int64_t L) {
    if (R < 0) return fail(ctx, FR_ERR_INVALID_ARG, "R = %d is negative", R);
    if (L < 0) return fail(ctx, FR_ERR_INVALID_ARG, "L = %lld is negative", (long long)L);
    if (L > ctx->max_tokens)
        return fail(ctx, FR_ERR_WORKSPACE, "L = %lld exceeds the context's max_tokens = %lld", (long long)L,
                    (long long)ctx->max_tokens);
    if (R > L) return fail(ctx, FR_ERR_INVALID_ARG, "R = %d rows but only L = %lld positions", R, (long long)L);
    return FR_OK;
}

static fr_status prefill_attn_impl(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                   const void* k_cache, const void* v_cache, int64_t L, const void* k_new,
                                   const void* v_new, void* out, float* lse_out, bool writeback, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    fr_status st = check_rows(ctx, R, L);
    if (st != FR_OK) return st;
    if (R == 0) return FR_OK;
    if (!q_rows || !q_index || !k_cache || !v_cache || !out)
        return fail(ctx, FR_ERR_INVALID_ARG, "q_rows / q_index / k_cache / v_cache / out is NULL");
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(ctx, FR_ERR_INVALID_ARG, "k_new and v_new must both be given or both be NULL");
    if (!aligned16(q_rows) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(k_new) ||
        !aligned16(v_new))
        return fail(ctx, FR_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(q_index) & 3u) || (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "q_index / lse_out must be 4-byte aligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    if (writeback && !k_new) return fail(ctx, FR_ERR_INVALID_ARG, "the write-back needs k_new / v_new");
    hipError_t e;
    if (attn_mfma_supported(s)) {   // (the tiled path finds the fresh rows of a key tile while it packs the tile)
        e = launch_attn_mfma(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse_out, ctx->ws,
                             ctx->attn_softmax_mode, ctx->attn_split_mode, nullptr, &ctx->attn_timer, writeback, hs);
    } else {
        const int32_t* inv = nullptr;   // position -> fresh row map
        if (k_new) {
            e = launch_inv_index(q_index, R, L, ctx->ws.inv_index, hs);
            if (e != hipSuccess) return hip_fail(ctx, "index map launch", e);
            inv = ctx->ws.inv_index;
        }
        e = launch_attn_simt(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, inv, out, lse_out, hs);
        if (e == hipSuccess && writeback)   // the generic kernel has no packing pass to fuse it into
            e = launch_kv_scatter(s, k_new, v_new, q_index, R, const_cast<void*>(k_cache), const_cast<void*>(v_cache), L, hs);
    }
    if (e != hipSuccess) return hip_fail(ctx, "attention launch", e);
    return FR_OK;
}

fr_status fr_sparse_prefill_attn(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                 const void* k_cache, const void* v_cache, int64_t L, const void* k_new,
                                 const void* v_new, void* out, float* lse_out, void* stream) {
    return prefill_attn_impl(ctx, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse_out, false, stream);
}

fr_status fr_sparse_prefill_attn_writeback(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                           void* k_cache, void* v_cache, int64_t L, const void* k_new,
                                           const void* v_new, void* out, float* lse_out, void* stream) {
    return prefill_attn_impl(ctx, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse_out, true, stream);
}

// Host-side checks of one query over the shared chunk store; fills the chunk table and the position deltas.
static fr_status check_shared_query(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                    const void* k_store, const void* v_store, int64_t n_store_rows,
                                    const int32_t* chunk_offsets, const int32_t* chunk_store_row0,
                                    const int32_t* chunk_src_pos0, int32_t n_chunks, int64_t L, const void* k_new,
                                    const void* v_new, const void* out, const float* lse_out, SharedStoreArgs* sh,
                                    ChunkDeltas* dl) {
    fr_status st = check_rows(ctx, R, L);
    if (st != FR_OK) return st;
    st = read_chunks(ctx, chunk_offsets, n_chunks, L, &sh->ct, nullptr);
    if (st != FR_OK) return st;
    if (n_store_rows < 0) return fail(ctx, FR_ERR_INVALID_ARG, "n_store_rows is negative");
    if (n_chunks > 0 && (!chunk_store_row0 || !chunk_src_pos0))
        return fail(ctx, FR_ERR_INVALID_ARG, "chunk_store_row0 / chunk_src_pos0 is NULL");
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t len = (int64_t)sh->ct.off[c + 1] - sh->ct.off[c];
        if (chunk_store_row0[c] < 0 || (int64_t)chunk_store_row0[c] + len > n_store_rows)
            return fail(ctx, FR_ERR_INVALID_ARG, "chunk %d: store rows [%d, %lld) outside the store of %lld rows", c,
                        chunk_store_row0[c], (long long)chunk_store_row0[c] + len, (long long)n_store_rows);
        const int64_t delta = (int64_t)sh->ct.off[c] - (int64_t)chunk_src_pos0[c];
        if (delta > INT32_MAX || delta < INT32_MIN) return fail(ctx, FR_ERR_INVALID_ARG, "position delta overflows");
        dl->delta[c] = (int32_t)delta;
    }
    if (R == 0) return FR_OK;
    if (!q_rows || !q_index || !out || !k_new || !v_new)
        return fail(ctx, FR_ERR_INVALID_ARG, "q_rows / q_index / k_new / v_new / out is NULL");
    if (sh->ct.off[sh->ct.n] > 0 && (!k_store || !v_store)) return fail(ctx, FR_ERR_INVALID_ARG, "k_store / v_store is NULL");
    if (!aligned16(q_rows) || !aligned16(k_store) || !aligned16(v_store) || !aligned16(out) || !aligned16(k_new) ||
        !aligned16(v_new))
        return fail(ctx, FR_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(q_index) & 3u) || (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "q_index / lse_out must be 4-byte aligned");
    sh->store_row0 = chunk_store_row0;
    return FR_OK;
}

fr_status fr_sparse_prefill_attn_shared(fr_ctx* ctx, const void* q_rows, const int32_t* q_index, int32_t R,
                                        const void* k_store, const void* v_store, int64_t n_store_rows,
                                        const int32_t* chunk_offsets, const int32_t* chunk_store_row0,
                                        const int32_t* chunk_src_pos0, int32_t n_chunks, int64_t L, const void* k_new,
                                        const void* v_new, void* out, float* lse_out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    SharedStoreArgs sh;
    ChunkDeltas dl;
    fr_status st = check_shared_query(ctx, q_rows, q_index, R, k_store, v_store, n_store_rows, chunk_offsets,
                                      chunk_store_row0, chunk_src_pos0, n_chunks, L, k_new, v_new, out, lse_out, &sh, &dl);
    if (st != FR_OK) return st;
    if (R == 0) return FR_OK;
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (!attn_mfma_supported(s)) {   // no tiled kernel for this shape: gathered keys and values, generic kernel
        e = launch_inv_index(q_index, R, L, ctx->ws.inv_index, hs);
        if (e != hipSuccess) return hip_fail(ctx, "index map launch", e);
        if ((st = gather_from_store(ctx, k_store, v_store, sh.ct, chunk_store_row0, dl, L, hs)) != FR_OK) return st;
        e = launch_attn_simt(s, q_rows, q_index, R, ctx->ws.store_k, ctx->ws.store_v, L, k_new, v_new, ctx->ws.inv_index, out,
                             lse_out, hs);
        if (e != hipSuccess) return hip_fail(ctx, "attention launch", e);
        return FR_OK;
    }
    e = launch_rope_table(s, dl, n_chunks, ctx->ws.rope_table, hs);
    if (e != hipSuccess) return hip_fail(ctx, "rope table launch", e);
    sh.table = ctx->ws.rope_table;
    e = launch_attn_mfma(s, q_rows, q_index, R, k_store, v_store, L, k_new, v_new, out, lse_out, ctx->ws,
                         ctx->attn_softmax_mode, ctx->attn_split_mode, &sh, &ctx->attn_timer, false, hs);
    if (e != hipSuccess) return hip_fail(ctx, "attention launch", e);
    return FR_OK;
}

// Scratch of one query of a batch inside the caller's workspace, every part 256-byte aligned.
namespace {
struct BatchScratch {
    size_t srow, cid, table, images, flags, end;
    size_t images_bytes, flags_elems;
};
BatchScratch batch_scratch(const Shape& s, int64_t L, int64_t R, size_t base) {
    BatchScratch b{};
    size_t off = base;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += round_up(bytes, 256);
        return o;
    };
    b.srow = take((size_t)L * 4);
    b.cid = take((size_t)L * 4);
    b.table = take((size_t)FR_MAX_CHUNKS * (s.d / 2) * sizeof(float2));
    b.images_bytes = attn_mfma_images_bytes(s, L);
    b.images = take(b.images_bytes);
    b.flags_elems = attn_mfma_flags_elems(s, R);
    b.flags = take(b.flags_elems * 4);
    b.end = off;
    return b;
}
}  // namespace

int64_t fr_shared_batch_workspace_bytes(const fr_ctx* ctx, int32_t n_queries, int64_t max_L) {
    if (!ctx || n_queries <= 0 || max_L <= 0) return 0;
    if (!attn_mfma_supported(ctx->shape)) return 0;   // such shapes are served query by query from the context's own workspace
    const int64_t group = n_queries < ATTN_MAX_BATCH ? n_queries : ATTN_MAX_BATCH;
    return group * (int64_t)batch_scratch(ctx->shape, max_L, max_L, 0).end;
}

fr_status fr_sparse_prefill_attn_shared_batch(fr_ctx* ctx, const fr_shared_query* queries, int32_t n_queries,
                                              const void* k_store, const void* v_store, int64_t n_store_rows,
                                              void* workspace, int64_t workspace_bytes, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    if (n_queries < 0) return fail(ctx, FR_ERR_INVALID_ARG, "n_queries = %d is negative", n_queries);
    if (n_queries == 0) return FR_OK;
    if (!queries) return fail(ctx, FR_ERR_INVALID_ARG, "queries is NULL");
    if (workspace_bytes < 0 || (workspace_bytes > 0 && !workspace) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ctx, FR_ERR_INVALID_ARG, "workspace is NULL or not 256-byte aligned");
    // every query is checked before anything is launched
    std::vector<SharedBatchQuery> work;
    std::vector<ChunkDeltas> deltas;
    work.reserve(n_queries);
    deltas.reserve(n_queries);
    for (int i = 0; i < n_queries; ++i) {
        const fr_shared_query& q = queries[i];
        SharedBatchQuery w{};
        ChunkDeltas dl;
        fr_status st = check_shared_query(ctx, q.q_rows, q.q_index, q.R, k_store, v_store, n_store_rows, q.chunk_offsets,
                                          q.chunk_store_row0, q.chunk_src_pos0, q.n_chunks, q.L, q.k_new, q.v_new, q.out,
                                          q.lse_out, &w.shared, &dl);
        if (st != FR_OK) {
            ctx->err = "query " + std::to_string(i) + ": " + ctx->err;
            return st;
        }
        if (q.R == 0) continue;   // nothing to compute for this query
        w.q_rows = q.q_rows; w.q_index = q.q_index; w.R = q.R; w.L = q.L;
        w.k_new = q.k_new; w.v_new = q.v_new; w.out = q.out; w.lse = q.lse_out;
        work.push_back(w);
        deltas.push_back(dl);
    }
    if (work.empty()) return FR_OK;
    if (!attn_mfma_supported(s)) {   // no tiled kernel for this shape: one query after the other, on the same stream
        for (int i = 0; i < n_queries; ++i) {
            const fr_shared_query& q = queries[i];
            if (q.R == 0) continue;
            fr_status st = fr_sparse_prefill_attn_shared(ctx, q.q_rows, q.q_index, q.R, k_store, v_store, n_store_rows,
                                                         q.chunk_offsets, q.chunk_store_row0, q.chunk_src_pos0, q.n_chunks, q.L,
                                                         q.k_new, q.v_new, q.out, q.lse_out, stream);
            if (st != FR_OK) return st;
        }
        return FR_OK;
    }
    // groups of at most ATTN_MAX_BATCH queries share one attention launch; the groups reuse the workspace (the
    // stream orders them)
    for (size_t g0 = 0; g0 < work.size(); g0 += ATTN_MAX_BATCH) {
        const size_t g1 = std::min(work.size(), g0 + (size_t)ATTN_MAX_BATCH);
        size_t off = 0;
        for (size_t i = g0; i < g1; ++i) off = batch_scratch(s, work[i].L, work[i].R, off).end;
        if ((int64_t)off > workspace_bytes)
            return fail(ctx, FR_ERR_WORKSPACE, "the batch needs %lld bytes of workspace, %lld given "
                        "(fr_shared_batch_workspace_bytes gives a sufficient size)", (long long)off, (long long)workspace_bytes);
    }
    fr_status st = need_device(ctx);
    if (st != FR_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    unsigned char* base = static_cast<unsigned char*>(workspace);
    for (size_t g0 = 0; g0 < work.size(); g0 += ATTN_MAX_BATCH) {
        const size_t g1 = std::min(work.size(), g0 + (size_t)ATTN_MAX_BATCH);
        size_t off = 0;
        for (size_t i = g0; i < g1; ++i) {
            SharedBatchQuery& w = work[i];
            const BatchScratch b = batch_scratch(s, w.L, w.R, off);
            off = b.end;
            float2* table = reinterpret_cast<float2*>(base + b.table);
            hipError_t e = launch_rope_table(s, deltas[i], w.shared.ct.n, table, hs);
            if (e != hipSuccess) return hip_fail(ctx, "rope table launch", e);
            w.shared.table = table;
            w.store_row_map = reinterpret_cast<int32_t*>(base + b.srow);
            w.chunk_id_map = reinterpret_cast<int32_t*>(base + b.cid);
            w.images = base + b.images;
            w.images_bytes = b.images_bytes;
            w.flags = reinterpret_cast<int32_t*>(base + b.flags);
            w.flags_elems = b.flags_elems;
        }
        hipError_t e = launch_attn_mfma_shared_batch(s, (int)(g1 - g0), &work[g0], k_store, v_store, ctx->attn_softmax_mode,
                                                     &ctx->attn_timer, hs);
        if (e != hipSuccess) return hip_fail(ctx, "attention launch", e);
    }
    return FR_OK;
}

fr_status fr_decode_attn(fr_ctx* ctx, const void* q, int32_t n_queries, const void* k_shared, const void* v_shared,
                         int64_t n_shared_rows, const int32_t* seg_offsets, const int32_t* seg_row0,
                         const int32_t* seg_len, const int32_t* seg_delta, int32_t n_segments,
                         const uint32_t* stale_bits, int64_t stale_words, const void* k_pages, const void* v_pages,
                         int64_t page_stride_rows, const int32_t* page_len, void* out, float* lse_out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (n_queries < 0 || n_segments < 0 || n_shared_rows < 0 || page_stride_rows < 0 || stale_words < 0)
        return fail(ctx, FR_ERR_INVALID_ARG, "negative size");
    if (n_queries == 0) return FR_OK;
    if ((int64_t)n_queries + n_segments > DECODE_MAX_UNITS)
        return fail(ctx, FR_ERR_WORKSPACE, "n_segments + n_queries = %lld exceeds %d", (long long)n_queries + n_segments,
                    DECODE_MAX_UNITS);
    auto bad16 = [](const void* p) { return !p || (reinterpret_cast<uintptr_t>(p) & 15u); };
    auto bad4 = [](const void* p) { return !p || (reinterpret_cast<uintptr_t>(p) & 3u); };
    if (bad16(q) || bad16(out) || bad16(k_pages) || bad16(v_pages))
        return fail(ctx, FR_ERR_INVALID_ARG, "q / out / k_pages / v_pages is NULL or not 16-byte aligned");
    if (n_segments > 0 && (bad16(k_shared) || bad16(v_shared)))
        return fail(ctx, FR_ERR_INVALID_ARG, "k_shared / v_shared is NULL or not 16-byte aligned");
    if (bad4(seg_offsets) || bad4(page_len) || (n_segments > 0 && (bad4(seg_row0) || bad4(seg_len) || bad4(seg_delta))))
        return fail(ctx, FR_ERR_INVALID_ARG, "a descriptor array is NULL or not 4-byte aligned");
    if ((stale_bits && (reinterpret_cast<uintptr_t>(stale_bits) & 3u)) || (lse_out && (reinterpret_cast<uintptr_t>(lse_out) & 3u)))
        return fail(ctx, FR_ERR_INVALID_ARG, "stale_bits / lse_out not 4-byte aligned");
    if (!decode_supported(ctx->shape)) return fail(ctx, FR_ERR_UNSUPPORTED, "group size %d", ctx->shape.G);
    fr_status st = need_device(ctx);
    if (st != FR_OK) return st;
    DecodeArgs a;
    a.q = q; a.B = n_queries;
    a.k_shared = k_shared; a.v_shared = v_shared; a.n_shared = n_shared_rows;
    a.seg_offsets = seg_offsets; a.seg_row0 = seg_row0; a.seg_len = seg_len; a.seg_delta = seg_delta; a.n_seg = n_segments;
    a.stale_bits = stale_bits; a.stale_words = stale_words;
    a.k_pages = k_pages; a.v_pages = v_pages; a.page_stride = page_stride_rows; a.page_len = page_len;
    a.out = out; a.lse_out = lse_out;
    a.force_generic = ctx->decode_generic;
    hipError_t e = launch_decode_attn(ctx->shape, a, ctx->ws.decode_partials, ctx->ws.decode_rot, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "decode attention launch", e);
    return FR_OK;
}

fr_status fr_mark_stale_rows(fr_ctx* ctx, uint32_t* stale_bits, int64_t n_words, const int32_t* rows, int32_t n_rows,
                             int32_t clear, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (n_words < 0 || n_rows < 0) return fail(ctx, FR_ERR_INVALID_ARG, "negative size");
    if (n_words == 0 || (n_rows == 0 && !clear)) return FR_OK;
    if (!stale_bits || (reinterpret_cast<uintptr_t>(stale_bits) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "stale_bits is NULL or not 4-byte aligned");
    if (n_rows > 0 && (!rows || (reinterpret_cast<uintptr_t>(rows) & 3u)))
        return fail(ctx, FR_ERR_INVALID_ARG, "rows is NULL or not 4-byte aligned");
    fr_status st = need_device(ctx);
    if (st != FR_OK) return st;
    hipError_t e = launch_mark_stale(stale_bits, n_words, rows, n_rows, clear, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "mark stale launch", e);
    return FR_OK;
}

fr_status fr_kv_scatter(fr_ctx* ctx, const void* k_new, const void* v_new, const int32_t* q_index, int32_t R,
                        void* k_cache, void* v_cache, int64_t L, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    fr_status st = check_rows(ctx, R, L);
    if (st != FR_OK) return st;
    if (R == 0) return FR_OK;
    if (!k_new || !v_new || !q_index || !k_cache || !v_cache)
        return fail(ctx, FR_ERR_INVALID_ARG, "k_new / v_new / q_index / k_cache / v_cache is NULL");
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return fail(ctx, FR_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(q_index) & 3u) return fail(ctx, FR_ERR_INVALID_ARG, "q_index must be 4-byte aligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipError_t e = launch_kv_scatter(ctx->shape, k_new, v_new, q_index, R, k_cache, v_cache, L, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "scatter launch", e);
    return FR_OK;
}

// ---- model steps around the path -------------------------------------------------------------------

static fr_status check_stack(fr_ctx* ctx, const char* what) {
    if (ctx->shape.dtype != FR_BF16) return fail(ctx, FR_ERR_UNSUPPORTED, "%s: bf16 contexts only", what);
    return FR_OK;
}

fr_status fr_rmsnorm(fr_ctx* ctx, const void* x, const void* gain, int32_t R, int32_t hidden, float eps, void* out,
                     void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    fr_status st = check_stack(ctx, "fr_rmsnorm");
    if (st != FR_OK) return st;
    if (R < 0 || hidden <= 0 || hidden % 8 != 0) return fail(ctx, FR_ERR_INVALID_ARG, "bad R = %d / hidden = %d", R, hidden);
    if (!(eps >= 0.f)) return fail(ctx, FR_ERR_INVALID_ARG, "eps must be non-negative");
    if (R == 0) return FR_OK;
    if (!x || !gain || !out || !aligned16(x) || !aligned16(gain) || !aligned16(out))
        return fail(ctx, FR_ERR_INVALID_ARG, "x / gain / out is NULL or not 16-byte aligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipError_t e = launch_rmsnorm(x, gain, R, hidden, eps, out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "rmsnorm launch", e);
    return FR_OK;
}

static fr_status check_gemm(fr_ctx* ctx, const char* what, const void* a, const void* w, int32_t M, int32_t N, int32_t K) {
    fr_status st = check_stack(ctx, what);
    if (st != FR_OK) return st;
    if (M < 0 || N <= 0 || K <= 0) return fail(ctx, FR_ERR_INVALID_ARG, "%s: bad M = %d, N = %d, K = %d", what, M, N, K);
    if (N % 128 != 0 || K % 64 != 0)
        return fail(ctx, FR_ERR_UNSUPPORTED, "%s: N = %d must be a multiple of 128 and K = %d of 64", what, N, K);
    if (K > (1 << 22))   // the kernel addresses a tile's rows with 32-bit byte offsets: 256 rows of K elements
        return fail(ctx, FR_ERR_UNSUPPORTED, "%s: K = %d exceeds 2^22", what, K);
    if (M > 0 && (!a || !w || !aligned16(a) || !aligned16(w)))
        return fail(ctx, FR_ERR_INVALID_ARG, "%s: a / w is NULL or not 16-byte aligned", what);
    return FR_OK;
}

fr_status fr_linear(fr_ctx* ctx, const void* a, const void* w, int32_t M, int32_t N, int32_t K, const void* residual,
                    void* out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    fr_status st = check_gemm(ctx, "fr_linear", a, w, M, N, K);
    if (st != FR_OK) return st;
    if (M == 0) return FR_OK;
    if (!out || !aligned16(out) || !aligned16(residual))
        return fail(ctx, FR_ERR_INVALID_ARG, "fr_linear: out is NULL or out / residual not 16-byte aligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipError_t e = launch_linear(a, w, M, N, K, residual, out, ctx->ws.gemm_partials, ctx->ws.gemm_partials_bytes, ctx->gemm_tuning, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "linear launch", e);
    return FR_OK;
}

fr_status fr_linear_swiglu(fr_ctx* ctx, const void* a, const void* w_gate_up, int32_t M, int32_t F, int32_t K,
                           void* out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    if (F <= 0 || F > INT32_MAX / 2) return fail(ctx, FR_ERR_INVALID_ARG, "fr_linear_swiglu: bad F = %d", F);
    fr_status st = check_gemm(ctx, "fr_linear_swiglu", a, w_gate_up, M, 2 * F, K);
    if (st != FR_OK) return st;
    if (M == 0) return FR_OK;
    if (!out || !aligned16(out)) return fail(ctx, FR_ERR_INVALID_ARG, "fr_linear_swiglu: out is NULL or misaligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipError_t e = launch_linear_swiglu(a, w_gate_up, M, F, K, out, ctx->ws.gemm_partials, ctx->ws.gemm_partials_bytes, ctx->gemm_tuning, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "swiglu launch", e);
    return FR_OK;
}

fr_status fr_qkv_rope(fr_ctx* ctx, const void* a, const void* w_qkv, int32_t M, int32_t K, const int32_t* positions,
                      void* q_out, void* k_out, void* v_out, void* stream) {
    if (!ctx) return FR_ERR_INVALID_ARG;
    ctx->err.clear();
    const Shape& s = ctx->shape;
    if (s.d != 128 || s.rope_layout != FR_ROPE_INTERLEAVED)
        return fail(ctx, FR_ERR_UNSUPPORTED, "fr_qkv_rope: head_dim 128 with interleaved rotary pairs only");
    fr_status st = check_gemm(ctx, "fr_qkv_rope", a, w_qkv, M, (s.Hq + 2 * s.Hkv) * s.d, K);
    if (st != FR_OK) return st;
    if (M > ctx->max_tokens) return fail(ctx, FR_ERR_WORKSPACE, "fr_qkv_rope: M = %d exceeds max_tokens", M);
    if (M == 0) return FR_OK;
    if (!positions || !q_out || !k_out || !v_out || !aligned16(q_out) || !aligned16(k_out) || !aligned16(v_out) ||
        (reinterpret_cast<uintptr_t>(positions) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "fr_qkv_rope: positions / q_out / k_out / v_out is NULL or misaligned");
    if ((st = need_device(ctx)) != FR_OK) return st;
    hipError_t e = launch_qkv_rope(s, a, w_qkv, M, K, positions, ctx->ws.rope_rows, q_out, k_out, v_out, ctx->ws.gemm_partials,
                                   ctx->ws.gemm_partials_bytes, ctx->gemm_tuning, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, "qkv launch", e);
    return FR_OK;
}

}  // extern "C"
