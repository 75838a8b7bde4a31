// Internal declarations shared by the translation units of libfusionrag (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "fusionrag.h"

namespace fr {

// Chunk boundaries travel to the kernels by value (kernel arguments are captured at launch, so a
// call never depends on host memory or a staging buffer after it returns).
struct ChunkTable {
    int32_t n;
    int32_t off[FR_MAX_CHUNKS + 1];
};
struct ChunkDeltas {
    int32_t delta[FR_MAX_CHUNKS];
};
// Store row of prompt position j inside chunk c of a query over a shared chunk store: row0[c] + (j - chunk offset).
struct ChunkRows {
    int32_t row0[FR_MAX_CHUNKS];
};

struct Shape {
    int Hq, Hkv, d, G;
    int dtype;       // fr_dtype
    int esize;       // bytes per element
    double rope_base;
    int rope_layout;
    int rope_index_base;
};

// Device workspace, carved from one allocation.
struct Workspace {
    char* base = nullptr;
    size_t bytes = 0;
    float2* rope_table = nullptr;   // [max_chunks][d/2] (cos, sin)
    float* lse = nullptr;           // [Hq][max_chunks + 1][max_q]  natural-log row normalisers
    float* col_partial = nullptr;   // [Hkv][max_ctx] per-KV-head column sums
    float* scores = nullptr;        // [max_tokens]
    int32_t* inv_index = nullptr;   // [max_tokens] position -> row of k_new / -1
    int32_t* store_row_map = nullptr;   // [max_tokens] prompt position -> row of the shared chunk store / -1
    int32_t* chunk_id_map = nullptr;    // [max_tokens] prompt position -> chunk
    float* qsum = nullptr;              // [Hkv][d] question queries summed per KV head (raw scores), then partial sums
    uint32_t* select_tmp = nullptr; // state, histogram, per-wave counts and candidate list of the selection kernels
    int32_t* attn_flags = nullptr;  // per (row tile, KV head) of an attention launch: 1 = redo with a running maximum
    size_t attn_flags_elems = 0;
    int n_cu = 0;                   // compute units of the device
    void* store_k = nullptr;        // shapes without a tiled path: a query's keys / values gathered from a shared
    void* store_v = nullptr;        // chunk store ([max_tokens, Hkv, d] each), for the generic kernels
    float* gemm_partials = nullptr; // partial sums of the GEMM tiles that are split along K
    size_t gemm_partials_bytes = 0;
    float2* rope_rows = nullptr;    // [max_tokens][d/2] (cos, sin) of the recomputed rows' positions
    float* decode_partials = nullptr;    // [DECODE_MAX_UNITS][Hq][d + 2] partial softmax results of fr_decode_attn
    float2* decode_rot = nullptr;        // [DECODE_MAX_UNITS][d/2] (cos, sin) of the segments' position shifts
    float* attn_partials = nullptr;      // partial results of an attention launch whose items are computed in parts
    size_t attn_partials_bytes = 0;
    unsigned char* kv_images = nullptr;  // [Hkv][ceil(max_tokens / 64)] LDS-ready K / V^T tile images, 32 KB each
    size_t kv_images_bytes = 0;
};

}  // namespace fr

namespace fr {
// Optional timing of the dominant attention kernel: a ring of event pairs recorded on the launch stream around it.
struct KernelTimer {
    static constexpr int MAX_SLOTS = 256;
    int n_slots = 0;            // 0 = off
    int64_t n_recorded = 0;     // launches recorded since it was switched on
    hipEvent_t start[MAX_SLOTS] = {};
    hipEvent_t stop[MAX_SLOTS] = {};
};
}  // namespace fr

namespace fr {
// Tuning switches of the projection kernels, kept per context (FR_OPT_GEMM_TILE, FR_OPT_GEMM_TAIL_SPLIT).
struct GemmTuning {
    int tile = 0;         // output features per workgroup: 0 = choose, 128, 256
    int tail_split = 1;   // 0 = the tiles of a launch's last, partly filled round are never split along K
};
}  // namespace fr

struct fr_ctx {
    fr::Shape shape;
    int64_t max_tokens = 0;
    int32_t max_chunks = 0;
    int32_t max_q = 0;
    bool has_device = false;
    int device = -1;
    fr::Workspace ws;
    int attn_softmax_mode = FR_ATTN_SOFTMAX_AUTO;
    int attn_split_mode = FR_ATTN_SPLIT_AUTO;
    int decode_generic = 0;
    fr::GemmTuning gemm_tuning;
    fr::KernelTimer attn_timer;
    std::string err;
};

namespace fr {

// Launchers.  Each returns hipSuccess or the launch error; none synchronises.
hipError_t launch_rope_table(const Shape& s, const ChunkDeltas& deltas, int n_chunks, float2* table,
                             hipStream_t st);
// src_rows != NULL: chunk c's source rows start at src row src_rows->row0[c] (a chunk store) instead of at its
// prompt offset.
hipError_t launch_rope_shift(const Shape& s, const void* src, void* dst, const ChunkTable& ct,
                             int max_chunk_len, const float2* table, int n_batch, int64_t src_stride,
                             int64_t dst_stride, const ChunkRows* src_rows, hipStream_t st);
hipError_t launch_clear_words(uint32_t* words, int64_t n_words, hipStream_t st);
hipError_t launch_kv_scatter(const Shape& s, const void* k_new, const void* v_new, const int32_t* q_index,
                             int R, void* k_cache, void* v_cache, int64_t L, hipStream_t st);

hipError_t launch_score_simt(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct,
                             int norm, const Workspace& ws, float* scores, hipStream_t st);
bool score_raw_supported(const Shape& s);
size_t score_raw_workspace_bytes(const Shape& s);
hipError_t launch_score_raw(const Shape& s, const void* q, int nq, const void* k_ctx, int64_t L_ctx, float* qsum,
                            float* scores, hipStream_t st);
bool score_mfma_supported(const Shape& s);
hipError_t launch_score_mfma(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct,
                             int norm, const Workspace& ws, float* scores, hipStream_t st);

hipError_t launch_score_mfma_shared(const Shape& s, const void* q, int nq, const void* k_store, const ChunkTable& ct,
                                    const int32_t* store_row0, const float2* table, int norm, const Workspace& ws,
                                    float* scores, hipStream_t st);

// `tmp` (tmp_bytes bytes of device scratch) is used beyond SELECT_ONE_WORKGROUP_MAX scores only; a scratch too small
// for n gives hipErrorInvalidValue before anything is launched.
constexpr int64_t SELECT_ONE_WORKGROUP_MAX = 32768;
hipError_t launch_select(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index,
                         uint32_t* tmp, size_t tmp_bytes, hipStream_t st);
// Scratch layout of the multi-workgroup selection, in 32-bit words: state and histograms (fixed), two words per tile of
// SELECT_TILE scores (the tiles' status words), candidate list.
constexpr int64_t SELECT_TILE = 32768;
constexpr size_t SELECT_FIXED_WORDS = 16 + 2 * 16384 + 16;
constexpr size_t SELECT_CAND_WORDS = (size_t)1 << 20;
constexpr size_t select_workspace_words(int64_t max_n) {   // scratch that serves every n <= max_n
    return SELECT_FIXED_WORDS + 2 * (size_t)((max_n + SELECT_TILE - 1) / SELECT_TILE) + SELECT_CAND_WORDS;
}
size_t select_workspace_bytes();                    // scratch for any n up to 2^31 - 1
size_t select_zeroed_bytes();                       // its leading part that must be zero when handed over (calls leave it zero)
// Resolves this device's copy of the static scratch of fr_select_topk_static (once per device; no allocation).
hipError_t select_static_prepare();
hipError_t launch_select_large(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* tmp,
                               size_t tmp_bytes, hipStream_t st);   // n beyond one workgroup's registers

hipError_t launch_kv_deviation(const Shape& s, const void* kv_a, const void* kv_b, int64_t n_tokens, float* out,
                               hipStream_t st);

// Batch decoding (all pointers device memory unless noted; see fr_decode_attn in the public header).
struct DecodeArgs {
    const void* q; int B;
    const void *k_shared, *v_shared; int64_t n_shared;
    const int32_t *seg_offsets, *seg_row0, *seg_len, *seg_delta; int n_seg;
    const uint32_t* stale_bits; int64_t stale_words;
    const void *k_pages, *v_pages; int64_t page_stride; const int32_t* page_len;
    void* out; float* lse_out;
    int force_generic;   // 1: the all-vector-ALU kernel also where the matrix-core one applies (tests)
};
constexpr int DECODE_MAX_UNITS = 4096;   // segments + queries of one call (sizes the partial-result buffer)
bool decode_supported(const Shape& s);
size_t decode_partials_bytes(const Shape& s);
size_t decode_rot_table_bytes(const Shape& s);
hipError_t launch_decode_attn(const Shape& s, const DecodeArgs& a, float* partials, float2* rot_table, hipStream_t st);
hipError_t launch_mark_stale(uint32_t* bits, int64_t n_words, const int32_t* rows, int n_rows, int clear, hipStream_t st);

// When given to launch_attn_mfma, k_cache / v_cache are a chunk store shared between queries: prompt position
// j in [ct.off[c], ct.off[c+1]) reads store row store_row0[c] + j - ct.off[c], its key rotated by the chunk's
// (cos, sin) row of `table` (device, [chunks][d/2]); store_row0 is a host array.
struct SharedStoreArgs {
    ChunkTable ct;
    const int32_t* store_row0;
    const float2* table;
};

hipError_t launch_inv_index(const int32_t* q_index, int R, int64_t L, int32_t* inv, hipStream_t st);
hipError_t launch_attn_simt(const Shape& s, const void* q_rows, const int32_t* q_index, int R,
                            const void* k_cache, const void* v_cache, int64_t L, const void* k_new,
                            const void* v_new, const int32_t* inv, void* out, float* lse, hipStream_t st);
bool attn_mfma_supported(const Shape& s);
hipError_t launch_attn_mfma(const Shape& s, const void* q_rows, const int32_t* q_index, int R,
                            const void* k_cache, const void* v_cache, int64_t L, const void* k_new,
                            const void* v_new, void* out, float* lse,
                            const Workspace& ws, int softmax_mode, int split_mode, const struct SharedStoreArgs* shared,
                            struct KernelTimer* timer, bool writeback, hipStream_t st);
// Several queries over one shared chunk store in one attention launch (Sec. 4.3).  Each query brings its scratch:
// prompt maps, rotation table, tile images and recompute flags (sizes: attn_mfma_images_bytes, attn_mfma_flags_elems).
// R > 0 for every query.
constexpr int ATTN_MAX_BATCH = 16;
struct SharedBatchQuery {
    const void* q_rows; const int32_t* q_index; int R; int64_t L;
    const void* k_new; const void* v_new; void* out; float* lse;
    SharedStoreArgs shared;          // chunk table, store rows (host), rotation table (device)
    int32_t* store_row_map; int32_t* chunk_id_map;   // device [L] each
    unsigned char* images; size_t images_bytes;
    int32_t* flags; size_t flags_elems;
};
size_t attn_mfma_images_bytes(const Shape& s, int64_t L);
size_t attn_mfma_flags_elems(const Shape& s, int64_t R);
hipError_t launch_attn_mfma_shared_batch(const Shape& s, int n, const SharedBatchQuery* qs, const void* k_store,
                                         const void* v_store, int softmax_mode, struct KernelTimer* timer, hipStream_t st);
// A one-query attention launch with few (row tile, KV head) items deals every item's key tiles to several workgroups
// (parts), on its own up to ATTN_SPLIT_AUTO_ITEMS items (beyond that the items alone keep the chip busy and the partial
// results' traffic costs more than the better balance gains): two parts, more (up to ATTN_MAX_PARTS) while that still
// leaves at most one piece per compute unit.  FR_ATTN_SPLIT_ON asks for two parts at any size the partial-result buffer
// takes.
constexpr int ATTN_SPLIT_AUTO_ITEMS = 400;
constexpr int ATTN_MAX_PARTS = 4;
size_t attn_mfma_partials_bytes(const Shape& s, int64_t max_tokens);

// `partials` (gemm_partials_bytes() bytes, or NULL: no split) holds the partial sums of the tiles of a launch's last,
// partly filled round, which are computed by several workgroups each.
size_t gemm_partials_bytes();
hipError_t launch_linear(const void* a, const void* w, int M, int N, int K, const void* residual, void* out,
                         float* partials, size_t partials_bytes, const GemmTuning& tune, hipStream_t st);
hipError_t launch_linear_swiglu(const void* a, const void* w_gate_up, int M, int F, int K, void* out, float* partials,
                                size_t partials_bytes, const GemmTuning& tune, hipStream_t st);
hipError_t launch_qkv_rope(const Shape& s, const void* a, const void* w_qkv, int M, int K, const int32_t* positions,
                           float2* rope_rows, void* q_out, void* k_out, void* v_out, float* partials,
                           size_t partials_bytes, const GemmTuning& tune, hipStream_t st);
hipError_t launch_rmsnorm(const void* x, const void* gain, int R, int hidden, float eps, void* out, hipStream_t st);

// ---- element helpers (device) ------------------------------------------------------------
template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <>
struct Elem<__bf16> {
    static __device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }
    static __device__ __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }  // nearest-even
};

}  // namespace fr
