// Sparse prefill attention (eq. 9, Sec. 4.3) on the gfx950 matrix cores: bf16, head_dim 128.
//
// Work split.  One workgroup (4 waves) owns one KV head and a tile of consecutive Q-index rows;
// each wave owns 64 "query columns" = (64 / G) token rows x the G query heads that share the KV
// head, so every K/V tile staged in LDS is reused by the whole grouped-query group and by all
// four waves.  Rows are sorted by position, so a tile needs keys 0 .. (position of its last row);
// tiles are issued longest first.
//
// Orientation.  The kernel computes the transposed products S^T = K Q^T and O^T = V^T P^T with
// v_mfma_f32_32x32x16_bf16:
//   * keys run along the M (register) dimension of S^T and query columns along N (lanes), so the
//     softmax statistics of a query column live in one lane (plus its partner lane + 32);
//   * the fp32 accumulator layout of S^T is, after conversion to bf16, exactly the B-operand
//     layout of the second product (contraction over keys), so P never leaves registers;
//   * V is transposed once per (KV head, key tile) by the packing pre-pass (4 keys x 8 dims per lane,
//     repacked with byte permutes), so the A operand of the second product is a 16-byte LDS read.
// The key order inside every block of 16 keys is permuted identically in P^T and V^T
// ([0-3, 8-11, 4-7, 12-15]); a contraction does not care about the order of its terms.
//
// Softmax.  exp(s - m) / sum exp(s - m) does not depend on m, and fp32 / bf16 leave about 2^127 of
// headroom, so the fast kernel fixes each query column's reference m once (the maximum over the
// column's first 32 visible keys) and never rescales: the tile loop holds no maximum, no
// comparison and no branch.  If a later logit exceeds the reference by more than that headroom
// the sums overflow to inf; the workgroup then raises a flag, and the safe kernel (classic online
// softmax with a running maximum) recomputes exactly the flagged workgroups.
//
// K/V tile images.  Every row tile of a KV head walks the same K/V stream (47 row tiles per head at 17k
// tokens / 15 %), so the work that does not depend on the rows is done once, by a packing pre-pass: for each
// (KV head, 64-key tile) it resolves stale / fresh rows (key j comes from k_new/v_new when inv[j] >= 0, i.e.
// its token is in the Q index, and from the cache otherwise: the cache is never written and stale rows are
// never read), transposes V, applies the LDS bank swizzle and writes a 32 KB image that is byte for byte what
// the attention kernels want in LDS.  The fast kernel's tile loop then stages a tile with direct-to-LDS
// copies: no lookups, no pointer selects, no permutes, no address arithmetic, no staging registers.
#include "fr_internal.hpp"
#include "k_rotate.hpp"

#include <hip/hip_ext.h>

#include <algorithm>

#ifndef FR_SCHED_HINTS
#define FR_SCHED_HINTS 1
#endif

namespace fr {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int D = 128;           // head_dim
constexpr int KT = 64;           // keys per tile
constexpr int O_PITCH = D + 8;   // bf16 elements per output row in the epilogue's LDS staging
constexpr float NEG_BIG = -1.0e30f;

// Tile image = [K image 18 KB][V^T image 18 KB], padded so that 16-byte operand reads (one lane per row, 16
// lanes per LDS pass) fall into 16 distinct bank groups and every fragment address is base + constant:
//   K image:   64 rows (keys) of 272 B (256 B of data + 16 B pad), then 1 KB of tail pad;
//   V^T image: 128 rows (dims) of 144 B (64 key slots = 128 B of data + 16 B pad), slot order see key_slot.
constexpr int K_ROW = 272, V_ROW = 144;
constexpr int K_IMG_BYTES = 18432;
constexpr int V_IMG_BYTES = D * V_ROW;   // 18432
constexpr int IMG_BYTES = K_IMG_BYTES + V_IMG_BYTES;
static_assert(KT * K_ROW <= K_IMG_BYTES && K_IMG_BYTES % 1024 == 0 && V_IMG_BYTES % 1024 == 0, "image layout");
// Inside every block of 16 keys the order is [0-3, 8-11, 4-7, 12-15]: the order in which the accumulator
// layout of S^T hands the keys to the second product.  Slot of key t (0..63) of a tile:
__device__ __forceinline__ int key_slot(int t) { return 16 * (t >> 4) + 4 * ((0x3120 >> (4 * ((t >> 2) & 3))) & 3) + (t & 3); }

// The fast kernel keeps separate rings of three K images and three V^T images (see its tile loop).
struct __attribute__((aligned(16))) Rings {
    unsigned char k[3][K_IMG_BYTES];
    unsigned char vt[3][V_IMG_BYTES];
};
constexpr size_t EPILOGUE_LDS = 4 * 64 * O_PITCH * sizeof(__bf16);   // four waves x [64 columns][d] bf16

__device__ __forceinline__ uint32_t perm_lo(uint32_t a, uint32_t b) {  // (a.lo16, b.lo16) -> a in low half
    return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t perm_hi(uint32_t a, uint32_t b) {  // (a.hi16, b.hi16)
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// ---- what a lane knows about its workgroup, wave and two query columns ---------------------------
template <int G>
struct Geometry {
    static constexpr int TRW = 64 / G;   // token rows per wave
    static constexpr int TR = 4 * TRW;   // token rows per workgroup
    int g, tile, row0;
    int x, h, wave;
    int col_row[2], col_head[2], col_pos[2];
    int wp_max;    // no key beyond it is visible to any row of this wave
    int n_kt;      // key tiles the workgroup walks
    int n_plain;   // leading tiles whose keys are visible to every row of the workgroup

    // ordinal counts the row tiles of a query from the longest one; ordinal < n_row_tiles
    __device__ __forceinline__ void init(const int32_t* __restrict__ q_index, int R, int Hkv, int n_row_tiles,
                                         int n_img_tiles, int g_, int ordinal) {
        init_rows(Hkv, n_row_tiles, g_, ordinal);
        init_positions(q_index, R, n_img_tiles);
    }
    // The part that does not read the Q index: which rows and heads the lane's two columns are.
    __device__ __forceinline__ void init_rows(int Hkv, int n_row_tiles, int g_, int ordinal) {
        const int tid = threadIdx.x, lane = tid & 63;
        wave = tid >> 6;
        x = lane & 31;
        h = lane >> 5;
        g = g_;
        tile = n_row_tiles - 1 - ordinal;                   // longest tiles first
        row0 = tile * TR;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int col = 32 * nb + x;
            const int r = row0 + wave * TRW + (col % TRW);
            col_row[nb] = r;                                 // rows past the end compute a copy of the last
            col_head[nb] = g * G + col / TRW;                // row and are never stored
        }
    }
    // The positions of the rows, from the Q index.
    // (a position beyond the prompt breaks the caller's contract; the walk then ends with the last image that exists)
    __device__ __forceinline__ void init_positions(const int32_t* __restrict__ q_index, int R, int n_img_tiles) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) col_pos[nb] = q_index[min(col_row[nb], R - 1)];
        const int p_first = q_index[row0];                   // rows ascend: every key <= p_first is visible to all
        const int p_max = q_index[min(R, row0 + TR) - 1];    // the workgroup's furthest key
        wp_max = q_index[min(row0 + wave * TRW + TRW, R) - 1];   // a wave past the end copies the last row
        n_kt = min(p_max / KT + 1, n_img_tiles);
        n_plain = min((p_first + 1) / KT, n_kt - 1);
    }
};

// ---- which keys of a 64-key tile are fresh ---------------------------------------------------------------
// fresh[t] = row r of k_new / v_new that holds the recomputed entry of position 64 kt + t (q_index[r] == that
// position), else -1.  The Q index is strictly ascending: wave 0 finds the first row at or behind the tile's first
// position by a 64-ary search (every round probes 64 evenly spaced rows at once: two dependent loads for up to 4096
// rows, where a binary search needs twelve), then the at most 64 rows that can fall into the tile are read in one go.
// All 256 threads call it; `fresh` is LDS, valid after the call's closing barrier.
__device__ __forceinline__ void tile_fresh_rows(const int32_t* __restrict__ q_index, int R, int kt, int32_t* fresh) {
    const int tid = threadIdx.x;
    if (tid < KT) fresh[tid] = -1;
    __syncthreads();
    if (tid < 64) {
        const int target = kt * KT;
        int lo = 0, hi = R;   // the first row with q_index[row] >= target lies in [lo, hi]
        while (lo < hi) {
            const int step = (hi - lo + 63) >> 6;
            const int probe = lo + tid * step;
            const bool below = probe < hi && q_index[probe] < target;
            const int cnt = __popcll(__ballot(below));   // probes are ascending, so the ones below the target come first
            if (cnt == 0) { hi = lo; break; }
            const int last_below = lo + (cnt - 1) * step;
            hi = min(hi, last_below + step);
            lo = last_below + 1;
        }
        const int row = lo + tid;
        if (row < R) {
            const int pos = q_index[row];
            if (pos >= target && pos < target + KT) fresh[pos - target] = row;   // (pos < target only for an index that is not ascending)
        }
    }
    __syncthreads();
}

// ---- packing pre-pass: grid (key tiles, KV heads) ---------------------------------------------------------
// Second half of both packing kernels: the thread's 4 key vectors and 4 value vectors (st_vec = 16-byte vector
// within the 256-byte head row; K: keys st_key + 16 i, V: keys 4 st_key + i) go into the LDS image, which is then
// written out as it is.
__device__ __forceinline__ void write_image(const u32x4 (&kreg)[4], const u32x4 (&vreg)[4], unsigned char* img,
                                            unsigned char* __restrict__ dst) {
    const int tid = threadIdx.x;
    const int st_vec = tid & 15, st_key = tid >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(&img[(st_key + 16 * i) * K_ROW + 16 * st_vec]) = kreg[i];
    {   // pads: K row tails, K image tail, V^T row tails (never read by the matrix operands; kept zero)
        const u32x4 z = {0u, 0u, 0u, 0u};
        if (tid < KT) *reinterpret_cast<u32x4*>(&img[tid * K_ROW + 256]) = z;
        if (tid < (K_IMG_BYTES - KT * K_ROW) / 16) *reinterpret_cast<u32x4*>(&img[KT * K_ROW + 16 * tid]) = z;
        if (tid < D) *reinterpret_cast<u32x4*>(&img[K_IMG_BYTES + tid * V_ROW + 128]) = z;
    }
    const int slot = key_slot(4 * st_key);   // the 4 keys of this lane occupy slots slot .. slot + 3
#pragma unroll
    for (int c = 0; c < 4; ++c) {   // dims 8 st_vec + 2c and + 2c + 1: gather the 4 keys of each
        u32x2 lo, hi;
        lo[0] = perm_lo(vreg[0][c], vreg[1][c]);
        lo[1] = perm_lo(vreg[2][c], vreg[3][c]);
        hi[0] = perm_hi(vreg[0][c], vreg[1][c]);
        hi[1] = perm_hi(vreg[2][c], vreg[3][c]);
        const int d0 = 8 * st_vec + 2 * c, d1 = d0 + 1;
        *reinterpret_cast<u32x2*>(&img[K_IMG_BYTES + d0 * V_ROW + 2 * slot]) = lo;
        *reinterpret_cast<u32x2*>(&img[K_IMG_BYTES + d1 * V_ROW + 2 * slot]) = hi;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < IMG_BYTES / 4096; ++i)
        *reinterpret_cast<u32x4*>(dst + i * 4096 + tid * 16) = *reinterpret_cast<const u32x4*>(&img[i * 4096 + tid * 16]);
}

// WRITEBACK: the fresh rows are also stored at their positions of the cache (the write-back of Sec. 4.3 fused into
// this pass: the row is in registers anyway).  No workgroup reads a cache row that another one writes: a position
// with a fresh row is never read from the cache.
template <bool WRITEBACK>
__global__ __launch_bounds__(256) void pack_kv_images_kernel(const __bf16* k_cache, const __bf16* v_cache, int L,
                                                             const __bf16* __restrict__ k_new,
                                                             const __bf16* __restrict__ v_new,
                                                             const int32_t* __restrict__ q_index, int R, int Hkv,
                                                             int n_img_tiles, unsigned char* __restrict__ images) {
    __shared__ __attribute__((aligned(16))) unsigned char img[IMG_BYTES];
    __shared__ int32_t fresh[KT];
    const int tid = threadIdx.x, kt = blockIdx.x, g = blockIdx.y;
    const int st_vec = tid & 15;   // 16-byte vector (8 dims) within a 256-byte head row
    const int st_key = tid >> 4;   // K: keys st_key + 16 i;  V: keys 4 st_key + i
    const bool have_new = k_new != nullptr;   // else the cache already holds the fresh rows
    if (have_new) tile_fresh_rows(q_index, R, kt, fresh);
    u32x4 kreg[4], vreg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {   // a key past the end is clamped: it lies beyond every row's position
        const int tk = st_key + 16 * i, tv = 4 * st_key + i;
        const int jk = min(kt * KT + tk, L - 1), jv = min(kt * KT + tv, L - 1);
        const int rk = have_new ? fresh[jk - kt * KT] : -1, rv = have_new ? fresh[jv - kt * KT] : -1;
        const __bf16* pk = rk >= 0 ? k_new + ((size_t)rk * Hkv + g) * D : k_cache + ((size_t)jk * Hkv + g) * D;
        const __bf16* pv = rv >= 0 ? v_new + ((size_t)rv * Hkv + g) * D : v_cache + ((size_t)jv * Hkv + g) * D;
        kreg[i] = *reinterpret_cast<const u32x4*>(pk + 8 * st_vec);
        vreg[i] = *reinterpret_cast<const u32x4*>(pv + 8 * st_vec);
        if (WRITEBACK) {   // (a clamped key past the end repeats key L-1: the same bytes again)
            if (rk >= 0)
                *reinterpret_cast<u32x4*>(const_cast<__bf16*>(k_cache) + ((size_t)jk * Hkv + g) * D + 8 * st_vec) = kreg[i];
            if (rv >= 0)
                *reinterpret_cast<u32x4*>(const_cast<__bf16*>(v_cache) + ((size_t)jv * Hkv + g) * D + 8 * st_vec) = vreg[i];
        }
    }
    write_image(kreg, vreg, img, images + ((size_t)g * n_img_tiles + kt) * IMG_BYTES);
}

// The same images built from a chunk store that is shared between queries and never written (Sec. 4.3): position
// j < L_ctx of the prompt belongs to chunk c = (the chunk whose offsets contain j) and reads store row
// row0[c] + j - off[c]; its key is moved to the prompt position on the way (Appendix A: one more rotation by
// Delta_c, from the (cos, sin) rows of `table`, same arithmetic as the stand-alone position shift).  Positions
// listed in the Q index (inv[j] >= 0: recomputed context tokens and all question tokens) read the query's own
// fresh rows instead, so the store's stale entries of those tokens are never read and no per-query copy of the
// cache exists.  Positions >= L_ctx that are not in the Q index have no data: they read as zero.

// Prompt position -> (store row, chunk) for the packing kernel, so that it needs no search and no dependent loads:
// grid (position tiles of the longest chunk, chunks + 1); the extra y index covers the positions behind the context
// (no store row: -1).
__global__ __launch_bounds__(256) void prompt_map_kernel(ChunkTable ct, ChunkRows rows, int L,
                                                         int32_t* __restrict__ store_row, int32_t* __restrict__ chunk_id) {
    const int c = blockIdx.y;
    const int begin = (c < ct.n) ? ct.off[c] : ct.off[ct.n];
    const int end = (c < ct.n) ? ct.off[c + 1] : L;
    for (int j = begin + blockIdx.x * 256 + threadIdx.x; j < end; j += gridDim.x * 256) {
        store_row[j] = (c < ct.n) ? rows.row0[c] + (j - begin) : -1;
        chunk_id[j] = (c < ct.n) ? c : 0;
    }
}

template <int LAYOUT>
__global__ __launch_bounds__(256) void pack_kv_images_shared_kernel(const __bf16* __restrict__ k_store,
                                                                    const __bf16* __restrict__ v_store,
                                                                    const int32_t* __restrict__ store_row,
                                                                    const int32_t* __restrict__ chunk_id,
                                                                    const float2* __restrict__ table,
                                                                    int L, const __bf16* __restrict__ k_new,
                                                                    const __bf16* __restrict__ v_new,
                                                                    const int32_t* __restrict__ q_index, int R, int Hkv,
                                                                    int n_img_tiles, unsigned char* __restrict__ images) {
    __shared__ __attribute__((aligned(16))) unsigned char img[IMG_BYTES];
    __shared__ int32_t fresh[KT];
    const int tid = threadIdx.x, kt = blockIdx.x, g = blockIdx.y;
    const int st_vec = tid & 15, st_key = tid >> 4;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    tile_fresh_rows(q_index, R, kt, fresh);
    int jk[4], jv[4], rk[4], rv[4], sk[4], sv[4], ck[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {   // the maps first, all at once: no load below depends on more than one of them
        jk[i] = min(kt * KT + st_key + 16 * i, L - 1);
        jv[i] = min(kt * KT + 4 * st_key + i, L - 1);
        rk[i] = fresh[jk[i] - kt * KT];
        rv[i] = fresh[jv[i] - kt * KT];
        sk[i] = store_row[jk[i]];
        sv[i] = store_row[jv[i]];
        ck[i] = chunk_id[jk[i]];
    }
    u32x4 kreg[4], vreg[4], kpart[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {   // positions that are neither fresh nor in a chunk read row 0 of the page and become zero
        const __bf16* pk = (rk[i] >= 0 || sk[i] < 0) ? k_new + ((size_t)max(rk[i], 0) * Hkv + g) * D
                                                      : k_store + ((size_t)sk[i] * Hkv + g) * D;
        const __bf16* pv = (rv[i] >= 0 || sv[i] < 0) ? v_new + ((size_t)max(rv[i], 0) * Hkv + g) * D
                                                      : v_store + ((size_t)sv[i] * Hkv + g) * D;
        kreg[i] = *reinterpret_cast<const u32x4*>(pk + 8 * st_vec);
        if (LAYOUT != FR_ROPE_INTERLEAVED) kpart[i] = *reinterpret_cast<const u32x4*>(pk + 8 * (st_vec ^ 8));
        vreg[i] = *reinterpret_cast<const u32x4*>(pv + 8 * st_vec);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (rk[i] < 0) {
            if (sk[i] >= 0)
                kreg[i] = rotate_key_vector<LAYOUT>(kreg[i], LAYOUT != FR_ROPE_INTERLEAVED ? kpart[i] : kreg[i],
                                                    table + (size_t)ck[i] * (D / 2), st_vec);
            else
                kreg[i] = zero;
        }
        if (rv[i] < 0 && sv[i] < 0) vreg[i] = zero;
    }
    write_image(kreg, vreg, img, images + ((size_t)g * n_img_tiles + kt) * IMG_BYTES);
}

// ---- staging in the fast kernel: image -> LDS directly (global_load_lds_dwordx4: lane i of a wave deposits its
//      16 bytes at the wave's LDS base + 16 i), no registers involved.  An image is 18 chunks of 1 KB; wave w
//      moves chunks w, w + 4, ...  Completion: the issuing wave's vmcnt, then a workgroup barrier. ----------
__device__ __forceinline__ void dma_image(const unsigned char* src, unsigned char* lds_dst, int wave, int lane) {
    // Written out rather than left to the builtin: the compiler treats a pending direct-to-LDS load as an access
    // that may complete out of order with the LDS reads, and from then on waits for *all* outstanding fragment
    // reads before every use (lgkmcnt(0)), which puts a full LDS round trip in front of the matrix pipe every few
    // fragments.  Completion is waited for explicitly anyway (wait_dma + workgroup barrier), so nothing is lost.
    // The image address is the same for the whole workgroup, so it travels in scalar registers (base + 16 lane):
    // the copies cost the vector ALU nothing.  `wave` must be wave-uniform in the compiler's eyes (readfirstlane).
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_dst);
    const uint32_t lane_off = (uint32_t)lane * 16u;
    static_assert(K_IMG_BYTES / 1024 == 18, "chunks 0..15 by all four waves, 16 and 17 by waves 0 and 1");
#pragma unroll
    for (int c = 0; c < 5; ++c) {
        const int chunk = wave + 4 * c;
        if (c < 4 || wave < 2) {
            const unsigned char* g = src + chunk * 1024;
            const uint32_t l = lds_base + (uint32_t)chunk * 1024u;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(g), "s"(l) : "memory");
        }
    }
}
__device__ __forceinline__ void wait_dma() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0)

// ---- staging in the safe kernel: image -> registers -> LDS, 9 copies of 16 bytes per lane ----------------
struct ImageStager {
    const unsigned char* head_images;   // images of this KV head
    int lane_off;                       // threadIdx.x * 16
    u32x4 reg[IMG_BYTES / 4096];
    __device__ __forceinline__ void init(const unsigned char* images, int g, int n_img_tiles) {
        head_images = images + (size_t)g * n_img_tiles * IMG_BYTES;
        lane_off = threadIdx.x * 16;
    }
    __device__ __forceinline__ void load(int kt) {
        const unsigned char* p = head_images + (size_t)kt * IMG_BYTES + lane_off;
#pragma unroll
        for (int i = 0; i < IMG_BYTES / 4096; ++i) reg[i] = *reinterpret_cast<const u32x4*>(p + i * 4096);
    }
    __device__ __forceinline__ void write(unsigned char* img) const {
#pragma unroll
        for (int i = 0; i < IMG_BYTES / 4096; ++i) *reinterpret_cast<u32x4*>(img + i * 4096 + lane_off) = reg[i];
    }
};

// Per-lane byte offsets of the operand fragments inside an image: row x, 16-byte half h.
struct FragOffsets {
    int k;   // K fragment: + 32 ks (16 dims per step) + 32 * K_ROW for the second half of the tile
    int v;   // V^T fragment: + 32 kb (16 key slots per block) + 32 * V_ROW * md for dim block md
    __device__ __forceinline__ void init(int x, int h) {
        k = x * K_ROW + 16 * h;
        v = x * V_ROW + 16 * h;
    }
};

// S^T for 32 keys (half mb of a staged tile) against this wave's 64 query columns.
__device__ __forceinline__ void qk_half(const unsigned char* k, int mb, const bf16x8 (&qf)[2][8], const FragOffsets& fo,
                                        f32x16 (&s)[2]) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(k + fo.k + 32 * ks + mb * (32 * K_ROW));
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], s[nb], 0, 0, 0);
    }
}

template <bool MASK>
__device__ __forceinline__ void mask_half(f32x16 (&s)[2], const int (&col_pos)[2], int key_base, int h) {
    if (!MASK) return;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = key_base + 8 * (v >> 2) + 4 * h + (v & 3);
            if (key > col_pos[nb]) s[nb][v] = -INFINITY;
        }
}

// O^T += V^T P^T for the 32 keys of half mb.
__device__ __forceinline__ void pv_half(const unsigned char* vt, int mb, const bf16x8 (&pf)[2][2], const FragOffsets& fo,
                                        f32x16 (&o)[4][2]) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int kb = 2 * mb + kk;
#pragma unroll
        for (int md = 0; md < 4; ++md) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(vt + fo.v + 32 * kb + md * (32 * V_ROW));
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) o[md][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nb][kk], o[md][nb], 0, 0, 0);
        }
    }
}

// One step of the fast kernel's software pipeline, at the granularity of 32 keys ("a half").  It turns the
// logits of half j (s_cur) into bf16 weights (pf_cur), while the matrix cores form the logits of half j+1
// (s_nxt = K Q^T, 16 instructions) and add half j-1 to the output (O^T += V^T P^T with pf_prev, 16
// instructions).  The three strands are independent, so the vector ALU's exp work runs in the shadow of the
// matrix instructions.  The exponent reference is fixed per column: no maximum, no rescale, no branch.
template <bool MASK, bool DO_QK>
__device__ __forceinline__ void pipeline_step(const unsigned char* k_next, int mb_next, const unsigned char* vt_prev,
                                              int mb_prev, const FragOffsets& fo, const bf16x8 (&qf)[2][8],
                                              f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2],
                                              const bf16x8 (&pf_prev)[2][2], bf16x8 (&pf_cur)[2][2], f32x16 (&o)[4][2],
                                              float (&lsum)[2], const float (&mref)[2], const int (&col_pos)[2],
                                              int key_base, int h, float scale_log2e) {
    mask_half<MASK>(s_cur, col_pos, key_base, h);
    if (DO_QK) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s_nxt[nb][v] = 0.f;
    }
    // Operand fragments are requested from LDS PF matrix steps before their use (rotating register buffer), so the
    // LDS latency overlaps the matrix and vector work already in flight.
    constexpr int PF = 4;
    bf16x8 fr[PF + 1];
    auto frag = [&](int i) -> bf16x8 {   // i < 8: K fragment ks = i of the next half;  i >= 8: V fragment (kk, md)
        if (i < 8) return *reinterpret_cast<const bf16x8*>(k_next + fo.k + 32 * i + mb_next * (32 * K_ROW));
        const int j = i - 8, kk = j >> 2, md = j & 3;
        return *reinterpret_cast<const bf16x8*>(vt_prev + fo.v + 32 * (2 * mb_prev + kk) + md * (32 * V_ROW));
    };
    constexpr int first = DO_QK ? 0 : 8;
#pragma unroll
    for (int i = 0; i < PF; ++i) fr[i] = frag(first + i);
    float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
    for (int i = first; i < 16; ++i) {
        if (i + PF < 16) fr[(i - first + PF) % (PF + 1)] = frag(i + PF);
        const bf16x8 a = fr[(i - first) % (PF + 1)];
        if (i < 8) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) s_nxt[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][i], s_nxt[nb], 0, 0, 0);
        } else {
            const int j = i - 8, kk = j >> 2, md = j & 3;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                o[md][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf_prev[nb][kk], o[md][nb], 0, 0, 0);
        }
        if (DO_QK || i >= 8) {   // two weights per matrix step: column block 0 during the logits, block 1 during the output
            const int nb = (i < 8) ? 0 : 1;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int v = 2 * (i & 7) + e;
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[nb][v], scale_log2e, -mref[nb]));
                if (nb == 0) psum0 += p; else psum1 += p;
                pf_cur[nb][v >> 3][v & 7] = (__bf16)p;
            }
        }
    }
    if (!DO_QK) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[0][v], scale_log2e, -mref[0]));
            psum0 += p;
            pf_cur[0][v >> 3][v & 7] = (__bf16)p;
        }
    }
    lsum[0] += psum0;
    lsum[1] += psum1;
#if FR_SCHED_HINTS
    // Ask the scheduler for: every fragment read PF matrix steps ahead of its use, and matrix and transcendental
    // instructions (the two long-latency strands) alternating.  Measured: several per cent over its own order;
    // patterns that also place the remaining vector work lose.
    __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);       // the first PF fragment reads
#pragma unroll
    for (int i = first; i < 16; ++i) {
        if (i + PF < 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // fragment i + PF
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // matrix
        __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);   // transcendental
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
    }
#endif
}

// Normalise, transpose through LDS and store 16 bytes per lane; lse = (m + log2 l) ln 2.
template <int G>
__device__ __forceinline__ void store_output(const Geometry<G>& ge, f32x16 (&o)[4][2], const float (&l)[2],
                                             const float (&mref)[2], int R, int Hq, unsigned char* smem,
                                             __bf16* __restrict__ out, float* __restrict__ lse_out) {
    constexpr int TRW = Geometry<G>::TRW;
    __bf16* ob = reinterpret_cast<__bf16*>(smem) + ge.wave * 64 * O_PITCH;   // this wave's [64 columns][d]
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float inv_l = 1.0f / l[nb];
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[md][nb][4 * q4 + e] * inv_l);
                *reinterpret_cast<bf16x4*>(&ob[(32 * nb + ge.x) * O_PITCH + 32 * md + 8 * q4 + 4 * ge.h]) = w;
            }
        if (lse_out != nullptr && ge.h == 0 && ge.col_row[nb] < R)
            lse_out[(size_t)ge.col_row[nb] * Hq + ge.col_head[nb]] =
                (mref[nb] + __builtin_amdgcn_logf(l[nb])) * 0.6931471805599453f;
    }
    __syncthreads();   // (each wave reads back only its own region; the barrier orders its LDS writes and reads)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int col = 4 * i + (lane >> 4), vec = lane & 15;
        const int r = ge.row0 + ge.wave * TRW + (col % TRW);
        if (r < R) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(&ob[col * O_PITCH + 8 * vec]);
            *reinterpret_cast<u32x4*>(out + ((size_t)r * Hq + ge.g * G + col / TRW) * D + 8 * vec) = w;
        }
    }
}

// Partial result of one part of an item, per lane: its 128 output accumulators as half-precision pairs (the 64 of a
// column block scaled by a power of two that brings the largest of them into [0.5, 1): 11 significant bits of that
// column's largest value, four times finer than the bf16 the output is rounded to), the two sums, the two exponent
// references and the two scale exponents as 32-bit words: 70 words instead of 132.  Register-major (word r of thread t
// at [r * 256 + t]: every store and load is one coalesced 1 KB line per wave).  Part p of item (ordinal, KV head g)
// lives at ((ordinal * n_parts + p) * Hkv + g) * PART_FLOATS.  Infinities and NaNs survive the packing (the combine
// pass must still see an overflow).
constexpr int PART_REGS = 70;
constexpr int PART_FLOATS = PART_REGS * 256;   // 32-bit words
typedef _Float16 __attribute__((ext_vector_type(2))) f16x2;

__device__ __forceinline__ void store_partial(float* __restrict__ dst_f, const f32x16 (&o)[4][2], const float (&lsum)[2],
                                              const float (&mref)[2]) {
    uint32_t* dst = reinterpret_cast<uint32_t*>(dst_f);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        float m = 0.f;
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
            for (int v = 0; v < 16; ++v) m = fmaxf(m, fabsf(o[md][nb][v]));
        // m = f 2^e with f in [0.5, 1); an infinite m keeps e = 0: the infinity is stored as it is
        const int e = (m < INFINITY) ? __builtin_amdgcn_frexp_expf(m) : 0;
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                f16x2 h;
                h[0] = (_Float16)__builtin_ldexpf(o[md][nb][v], -e);
                h[1] = (_Float16)__builtin_ldexpf(o[md][nb][v + 1], -e);
                dst[(nb * 32 + md * 8 + v / 2) * 256] = __builtin_bit_cast(uint32_t, h);
            }
        dst[(64 + nb) * 256] = __float_as_uint(lsum[nb]);
        dst[(66 + nb) * 256] = __float_as_uint(mref[nb]);
        dst[(68 + nb) * 256] = (uint32_t)e;
    }
}

// One launch serves up to ATTN_MAX_BATCH queries with their own rows, index sets, tile images and outputs (Sec. 4.3:
// queries of a batch share nothing but the chunk store the images were built from).  The table travels as a kernel
// argument.  blockIdx.x = (query * max_row_tiles + ordinal) * Hkv + KV head (launches without parts): consecutive blocks land
// on different XCDs, so with 8 KV heads each XCD's L2 serves the images of one head; the queries follow one another,
// each with its row tiles longest first, so that the short tiles at the end of one query run beside the long ones of
// the next and no more than about two queries' images are in use at a time (interleaving the queries was measured:
// their images then compete for the caches and the batch gains nothing over one launch per query).  A query with fewer
// row tiles than the longest one leaves its surplus blocks empty.
struct AttnQuery {
    const __bf16* q_rows;
    const int32_t* q_index;
    const unsigned char* images;
    __bf16* out;
    float* lse;
    int32_t* flags;        // per (row tile, KV head): 1 = redo with a running maximum
    int R, n_row_tiles, n_img_tiles, pad;
};
struct AttnBatch {
    AttnQuery q[ATTN_MAX_BATCH];
    int n, max_row_tiles;
};
struct BlockWork {
    int g, ordinal, query;
    __device__ __forceinline__ void init(int max_row_tiles, int Hkv) {
        int t = (int)blockIdx.x;
        g = t % Hkv; t /= Hkv;
        ordinal = t % max_row_tiles;
        query = t / max_row_tiles;
    }
};

// ---- classic online softmax (running maximum) for one (row tile, KV head): the whole key range, one workgroup.
//      Runs where the fixed exponent reference overflowed, and everywhere under FR_ATTN_SOFTMAX_RUNNING_MAX.
//      `smem` holds max(IMG_BYTES, EPILOGUE_LDS) bytes; every thread of the workgroup calls it. ------------------------
template <int G>
__device__ __forceinline__ void running_max_item(const AttnQuery& aq, int g, int ordinal, int Hq, int Hkv,
                                                 float scale_log2e, unsigned char* smem) {
    const __bf16* __restrict__ q_rows = aq.q_rows;
    const int R = aq.R, n_img_tiles = aq.n_img_tiles;
    unsigned char* k_img = smem;
    unsigned char* v_img = smem + K_IMG_BYTES;
    Geometry<G> ge;
    ge.init(aq.q_index, R, Hkv, aq.n_row_tiles, n_img_tiles, g, ordinal);
    const int h = ge.h;
    FragOffsets fo;
    fo.init(ge.x, h);
    bf16x8 qf[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const __bf16* qp = q_rows + ((size_t)min(ge.col_row[nb], R - 1) * Hq + ge.col_head[nb]) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }
    f32x16 o[4][2];
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[md][nb][v] = 0.f;
    float lsum[2] = {0.f, 0.f};
    float m2[2] = {NEG_BIG, NEG_BIG};
    ImageStager sg;
    sg.init(aq.images, ge.g, n_img_tiles);
    for (int kt = 0; kt < ge.n_kt; ++kt) {
        sg.load(kt);
        __syncthreads();
        sg.write(k_img);
        __syncthreads();
        if (kt * KT > ge.wp_max) continue;   // wave-uniform; the barriers stay outside
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            f32x16 s[2];
            qk_half(k_img, mb, qf, fo, s);
            mask_half<true>(s, ge.col_pos, kt * KT + 32 * mb, h);
            bf16x8 pf[2][2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float t = s[nb][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) t = fmaxf(t, s[nb][v]);
                t = fmaxf(t, __shfl_xor(t, 32));
                const float m_new = fmaxf(m2[nb], t * scale_log2e);
                const float alpha = __builtin_amdgcn_exp2f(m2[nb] - m_new);
                m2[nb] = m_new;
                float psum = 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nb][v], scale_log2e, -m_new));
                    psum += p;
                    pf[nb][v >> 3][v & 7] = (__bf16)p;
                }
                lsum[nb] = lsum[nb] * alpha + psum;
#pragma unroll
                for (int md = 0; md < 4; ++md)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[md][nb][v] *= alpha;
            }
            pv_half(v_img, mb, pf, fo, o);
        }
    }
    float l[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) l[nb] = lsum[nb] + __shfl_xor(lsum[nb], 32);
    __syncthreads();
    store_output<G>(ge, o, l, m2, R, Hq, smem, aq.out, aq.lse);
}

// Overflow check of a finished item: with a fixed reference a runaway logit shows up as inf / nan in the sums.
// Returns (workgroup-uniform) whether any column of the workgroup is affected; l = the columns' softmax sums.
__device__ __forceinline__ int sums_overflowed(const f32x16 (&o)[4][2], const float (&lsum)[2], float (&l)[2]) {
    bool bad = false;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        l[nb] = lsum[nb] + __shfl_xor(lsum[nb], 32);
        float chk = l[nb];
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
            for (int v = 0; v < 16; ++v) chk += fabsf(o[md][nb][v]);
        bad = bad || !(chk < INFINITY) || !(l[nb] > 0.f);
    }
    return __syncthreads_or(bad ? 1 : 0);   // also: every wave is done with the rings
}

// ---- fast path: key tiles [kb, ke) of one (row tile, KV head) ---------------------------------------------
// part < 0: the piece is the whole item; the workgroup finishes it: overflow check, then either the output or the
// item's flag (the kernel that follows recomputes flagged items with a running maximum).  part >= 0: the piece is
// share `part` of `n_parts` of the item's key tiles; it leaves its partial sums, and attn_combine_kernel finishes
// the item.  Every part uses the same exponent reference (each derives it from keys 0..31), so the parts simply add up.
template <int G>
__device__ __forceinline__ void process_piece(const AttnQuery& aq, int g, int ordinal, int part, int n_parts,
                                              float* __restrict__ partials, int Hq, int Hkv, float scale_log2e,
                                              unsigned char* smem_raw) {
    Rings& rg = *reinterpret_cast<Rings*>(smem_raw);
    const __bf16* __restrict__ q_rows = aq.q_rows;
    const int R = aq.R, n_img_tiles = aq.n_img_tiles;
    // ---- prologue.  Everything that does not depend on the Q index is requested first (the query fragments, and K
    //      image 0 for the exponent reference), then the Q index itself, so that the three memory round trips of the
    //      prologue overlap instead of following one another. ------------------------------------------------------
    Geometry<G> ge;
    ge.init_rows(Hkv, aq.n_row_tiles, g, ordinal);
    const int x = ge.x, h = ge.h;
    FragOffsets fo;
    fo.init(x, h);
    const unsigned char* head_images = aq.images + (size_t)ge.g * n_img_tiles * IMG_BYTES;
    const int wave = __builtin_amdgcn_readfirstlane(ge.wave), lane = threadIdx.x & 63;
    dma_image(head_images, rg.k[2], wave, lane);   // K image 0 into ring slot 2: the exponent reference comes from it

    // Q fragments: B operand of S^T = K Q^T, kept in registers for the whole loop
    bf16x8 qf[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const __bf16* qp = q_rows + ((size_t)min(ge.col_row[nb], R - 1) * Hq + ge.col_head[nb]) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }
    ge.init_positions(aq.q_index, R, n_img_tiles);
    const int n_kt = ge.n_kt;
    // this piece's key tiles [kb, ke): shares of ceil(n_kt / n_parts) tiles, so part 0 is never empty
    const int per_part = part < 0 ? n_kt : (n_kt + n_parts - 1) / n_parts;
    const int kb = part < 0 ? 0 : part * per_part, ke = min(n_kt, kb + per_part);
    float* part_dst = part < 0 ? nullptr : partials + (((size_t)ordinal * n_parts + part) * Hkv + g) * PART_FLOATS + threadIdx.x;
    if (kb >= ke) {   // fewer key tiles than parts: this one adds nothing
        for (int r = 0; r < PART_REGS; ++r) part_dst[r * 256] = 0.f;
        return;       // (the hardware waits for the outstanding copy before it retires the wave)
    }
    f32x16 o[4][2];
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[md][nb][v] = 0.f;
    float lsum[2] = {0.f, 0.f};

    // K images kb and kb + 1 and V image kb land in LDS
    const unsigned char* first_image = head_images + (size_t)kb * IMG_BYTES;
    dma_image(first_image, rg.k[0], wave, lane);
    dma_image(first_image + K_IMG_BYTES, rg.vt[0], wave, lane);
    if (kb + 1 < n_kt) dma_image(first_image + IMG_BYTES, rg.k[1], wave, lane);
    {   // V ring slot 2 is read (against all-zero weights) by the very first step: it must hold finite numbers
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = threadIdx.x; i < V_IMG_BYTES / 16; i += 256) *reinterpret_cast<u32x4*>(&rg.vt[2][16 * i]) = z;
    }
    wait_dma();
    __syncthreads();

    // exponent reference of each column = the maximum of its logits over the visible ones of keys 0..31
    f32x16 s_a[2], s_b[2];
    qk_half(rg.k[2], 0, qf, fo, s_a);
    float mref[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        float t = NEG_BIG;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = 8 * (v >> 2) + 4 * h + (v & 3);
            t = fmaxf(t, key <= ge.col_pos[nb] ? s_a[nb][v] : NEG_BIG);
        }
        t = fmaxf(t, __shfl_xor(t, 32));   // key 0 (held by the h = 0 lane) is visible to every row
        mref[nb] = t * scale_log2e;
    }
    __syncthreads();                                // ring slot 2 is free again before the loop copies into it
    if (kb > 0) qk_half(rg.k[0], 0, qf, fo, s_a);   // logits of this part's first 32 keys (else: those above)
    bf16x8 pf_a[2][2], pf_b[2][2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf_b[nb][kk][e] = (__bf16)0.0f;

    // ---- tile loop ------------------------------------------------------------------------------------
    // Iteration kt: wait for the own direct-to-LDS copies issued one iteration ago, barrier (now K image kt+1
    // and V image kt are complete and visible, and nobody reads the slots of K image kt-1 / V image kt-2 any
    // more), issue the copies of K image kt+2 and V image kt+1 into those slots, and run two pipeline steps:
    //   step (kt, 0): weights of keys [64kt, 64kt+32)    | logits of (kt, 1) from K[kt]     | O += half (kt-1, 1), V[kt-1]
    //   step (kt, 1): weights of keys [64kt+32, 64kt+64) | logits of (kt+1, 0) from K[kt+1] | O += half (kt, 0),   V[kt]
    int k0 = 0, k1 = 1, k2 = 2;   // ring slots of K images kt, kt+1, kt+2; V images kt-1, kt, kt+1 sit in k2, k0, k1
    int kt = kb;
    const int plain_end = min(ge.n_plain, ke);
    for (; kt < plain_end; ++kt) {   // plain tiles: every key visible to every row; image kt+1 always exists
        if (kt > kb) {
            wait_dma();
            __syncthreads();
        }
        const unsigned char* nxt = head_images + (size_t)(kt + 1) * IMG_BYTES;
        if (kt + 2 < n_kt) dma_image(nxt + IMG_BYTES, rg.k[k2], wave, lane);
        dma_image(nxt + K_IMG_BYTES, rg.vt[k1], wave, lane);
        pipeline_step<false, true>(rg.k[k0], 1, rg.vt[k2], 1, fo, qf, s_a, s_b, pf_b, pf_a, o, lsum, mref, ge.col_pos,
                                   kt * KT, h, scale_log2e);
        pipeline_step<false, true>(rg.k[k1], 0, rg.vt[k0], 0, fo, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref, ge.col_pos,
                                   kt * KT + 32, h, scale_log2e);
        const int t = k0; k0 = k1; k1 = k2; k2 = t;
    }
    for (; kt < ke; ++kt) {           // tiles that cross some row's own position
        if (kt > kb) {
            wait_dma();
            __syncthreads();
        }
        const unsigned char* nxt = head_images + (size_t)(kt + 1) * IMG_BYTES;
        if (kt + 2 < ke) dma_image(nxt + IMG_BYTES, rg.k[k2], wave, lane);
        if (kt + 1 < ke) dma_image(nxt + K_IMG_BYTES, rg.vt[k1], wave, lane);
        pipeline_step<true, true>(rg.k[k0], 1, rg.vt[k2], 1, fo, qf, s_a, s_b, pf_b, pf_a, o, lsum, mref, ge.col_pos,
                                  kt * KT, h, scale_log2e);
        if (kt + 1 < ke)
            pipeline_step<true, true>(rg.k[k1], 0, rg.vt[k0], 0, fo, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref,
                                      ge.col_pos, kt * KT + 32, h, scale_log2e);
        else
            pipeline_step<true, false>(rg.k[k1], 0, rg.vt[k0], 0, fo, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref,
                                       ge.col_pos, kt * KT + 32, h, scale_log2e);
        const int t = k0; k0 = k1; k1 = k2; k2 = t;
    }
    pv_half(rg.vt[k2], 1, pf_b, fo, o);   // the last half: V image ke-1 now sits in slot k2

    if (part >= 0) {   // leave the partial result; attn_combine_kernel adds the parts, checks and stores
        store_partial(part_dst, o, lsum, mref);
        return;
    }
    float l[2];
    const int any_bad = sums_overflowed(o, lsum, l);
    if (threadIdx.x == 0) aq.flags[ordinal * Hkv + g] = any_bad;   // raised: the item is recomputed with a running maximum
    if (any_bad) return;
    store_output<G>(ge, o, l, mref, R, Hq, smem_raw, aq.out, aq.lse);
}

// blockIdx.x = ((query * max_row_tiles + ordinal) * n_parts + part) * Hkv + KV head.  n_parts = 1: every item whole.
// n_parts > 1 (one query, few items: the chip would idle behind the longest ones): the key tiles of every item are
// dealt to n_parts workgroups in equal consecutive shares; items are launched longest first, so the pieces are too.
// Dynamic LDS: the larger of the K/V rings and the epilogue's staging.
template <int G>
__global__ __launch_bounds__(256) void attn_fixed_ref_kernel(const AttnBatch batch, float* __restrict__ partials, int n_parts,
                                                             int Hq, int Hkv, float scale_log2e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    int t = (int)blockIdx.x;
    const int g = t % Hkv; t /= Hkv;
    const int part = t % n_parts; t /= n_parts;
    const int ordinal = t % batch.max_row_tiles, query = t / batch.max_row_tiles;
    const AttnQuery& aq = batch.q[query];
    if (ordinal >= aq.n_row_tiles) return;
    process_piece<G>(aq, g, ordinal, n_parts > 1 ? part : -1, n_parts, partials, Hq, Hkv, scale_log2e, smem_raw);
}

// ---- combine: adds the parts of every item, then checks and stores like the fast path's own epilogue; on overflow
//      the item is recomputed with a running maximum.  grid.x = n_row_tiles * Hkv, LDS = max(epilogue staging, one image).
template <int G>
__global__ __launch_bounds__(256, 2) void attn_combine_kernel(const AttnQuery aq, const float* __restrict__ partials,
                                                              int n_parts, int Hq, int Hkv, float scale_log2e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int g = (int)blockIdx.x % Hkv, ordinal = (int)blockIdx.x / Hkv;
    {
        Geometry<G> ge;
        ge.init(aq.q_index, aq.R, Hkv, aq.n_row_tiles, aq.n_img_tiles, g, ordinal);
        const uint32_t* p0 = reinterpret_cast<const uint32_t*>(partials + (((size_t)ordinal * n_parts) * Hkv + g) * PART_FLOATS) + threadIdx.x;
        const size_t part_stride = (size_t)Hkv * PART_FLOATS;
        f32x16 o[4][2];
        float lsum[2] = {0.f, 0.f}, mref[2];
#pragma unroll
        for (int md = 0; md < 4; ++md)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[md][nb][v] = 0.f;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) mref[nb] = __uint_as_float(p0[(66 + nb) * 256]);   // part 0 is never empty; every part derives the same reference
        for (int part = 0; part < n_parts; ++part) {   // a part's 70 loads are in flight together, then unpacked and added
            const uint32_t* pp = p0 + part * part_stride;
            uint32_t w[2][32];
            uint32_t tail[2][2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
                for (int j2 = 0; j2 < 32; ++j2) w[nb][j2] = pp[(nb * 32 + j2) * 256];
                tail[nb][0] = pp[(64 + nb) * 256];
                tail[nb][1] = pp[(68 + nb) * 256];
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int e = (int)tail[nb][1];
#pragma unroll
                for (int md = 0; md < 4; ++md)
#pragma unroll
                    for (int v = 0; v < 16; v += 2) {
                        const f16x2 h = __builtin_bit_cast(f16x2, w[nb][md * 8 + v / 2]);
                        o[md][nb][v] += __builtin_ldexpf((float)h[0], e);
                        o[md][nb][v + 1] += __builtin_ldexpf((float)h[1], e);
                    }
                lsum[nb] += __uint_as_float(tail[nb][0]);
            }
        }
        float l[2];
        if (!sums_overflowed(o, lsum, l)) {
            store_output<G>(ge, o, l, mref, aq.R, Hq, smem_raw, aq.out, aq.lse);
            return;
        }
    }
    // the sums overflowed the fixed exponent reference (rare): the item again, with a running maximum
    __syncthreads();
    running_max_item<G>(aq, g, ordinal, Hq, Hkv, scale_log2e, smem_raw);
}

// ---- the items of a launch without parts with the running maximum: the flagged ones (use_flags), or all of them
//      (FR_ATTN_SOFTMAX_RUNNING_MAX) ---------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(256) void attn_running_max_kernel(const AttnBatch batch, int use_flags, int Hq, int Hkv,
                                                               float scale_log2e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    BlockWork bw;
    bw.init(batch.max_row_tiles, Hkv);
    const AttnQuery& aq = batch.q[bw.query];
    if (bw.ordinal >= aq.n_row_tiles) return;
    if (use_flags && aq.flags[bw.ordinal * Hkv + bw.g] == 0) return;
    running_max_item<G>(aq, bw.g, bw.ordinal, Hq, Hkv, scale_log2e, smem_raw);
}

// Where one query's packing pass leaves its results.
struct QueryScratch {
    int32_t* store_row_map;   // [L], shared-store queries only
    int32_t* chunk_id_map;    // [L], shared-store queries only
    unsigned char* images;
    size_t images_bytes;
    int32_t* flags;
    size_t flags_elems;
};

constexpr size_t LDS_FAST = sizeof(Rings) > EPILOGUE_LDS ? sizeof(Rings) : EPILOGUE_LDS;
constexpr size_t LDS_SAFE = (size_t)IMG_BYTES > EPILOGUE_LDS ? (size_t)IMG_BYTES : EPILOGUE_LDS;

// Raises the kernels' dynamic LDS limit, once per process (C++ initialises a function-local static exactly once,
// also when several host threads arrive together).
template <int G>
hipError_t set_kernel_attributes() {
    static const hipError_t once = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fixed_ref_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_FAST);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_combine_kernel<G>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_SAFE);
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_running_max_kernel<G>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_SAFE);
    }();
    return once;
}

// Packing pass of one query: tile images of its effective K/V into sc.images; fills the query's line of the table.
template <int G>
hipError_t pack_query(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                      const void* v_cache, int64_t L, const void* k_new, const void* v_new, void* out, float* lse,
                      const QueryScratch& sc, const SharedStoreArgs* shared, bool writeback, AttnQuery* aq, hipStream_t st) {
    constexpr int TR = Geometry<G>::TR;
    const int n_row_tiles = (R + TR - 1) / TR;
    const int n_img_tiles = (int)((L + KT - 1) / KT);
    const dim3 block(256);
    if ((size_t)n_row_tiles * s.Hkv > sc.flags_elems) return hipErrorInvalidValue;
    if ((size_t)n_img_tiles * s.Hkv * IMG_BYTES > sc.images_bytes) return hipErrorInvalidValue;
    if (shared == nullptr) {
        if (writeback)
            pack_kv_images_kernel<true><<<dim3(n_img_tiles, s.Hkv), block, 0, st>>>(
                (const __bf16*)k_cache, (const __bf16*)v_cache, (int)L, (const __bf16*)k_new, (const __bf16*)v_new, q_index, R,
                s.Hkv, n_img_tiles, sc.images);
        else
            pack_kv_images_kernel<false><<<dim3(n_img_tiles, s.Hkv), block, 0, st>>>(
                (const __bf16*)k_cache, (const __bf16*)v_cache, (int)L, (const __bf16*)k_new, (const __bf16*)v_new, q_index, R,
                s.Hkv, n_img_tiles, sc.images);
    } else {   // k_cache / v_cache are the shared chunk store
        ChunkRows rows;
        int max_len = (int)L - shared->ct.off[shared->ct.n];
        for (int c = 0; c < shared->ct.n; ++c) {
            rows.row0[c] = shared->store_row0[c];
            max_len = std::max(max_len, shared->ct.off[c + 1] - shared->ct.off[c]);
        }
        prompt_map_kernel<<<dim3(std::max(1, (max_len + 255) / 256), shared->ct.n + 1), block, 0, st>>>(
            shared->ct, rows, (int)L, sc.store_row_map, sc.chunk_id_map);
        if (s.rope_layout == FR_ROPE_INTERLEAVED)
            pack_kv_images_shared_kernel<FR_ROPE_INTERLEAVED><<<dim3(n_img_tiles, s.Hkv), block, 0, st>>>(
                (const __bf16*)k_cache, (const __bf16*)v_cache, sc.store_row_map, sc.chunk_id_map, shared->table, (int)L,
                (const __bf16*)k_new, (const __bf16*)v_new, q_index, R, s.Hkv, n_img_tiles, sc.images);
        else
            pack_kv_images_shared_kernel<FR_ROPE_HALF><<<dim3(n_img_tiles, s.Hkv), block, 0, st>>>(
                (const __bf16*)k_cache, (const __bf16*)v_cache, sc.store_row_map, sc.chunk_id_map, shared->table, (int)L,
                (const __bf16*)k_new, (const __bf16*)v_new, q_index, R, s.Hkv, n_img_tiles, sc.images);
    }
    aq->q_rows = (const __bf16*)q_rows;
    aq->q_index = q_index;
    aq->images = sc.images;
    aq->out = (__bf16*)out;
    aq->lse = lse;
    aq->flags = sc.flags;
    aq->R = R;
    aq->n_row_tiles = n_row_tiles;
    aq->n_img_tiles = n_img_tiles;
    aq->pad = 0;
    return hipGetLastError();
}

// Launches the key-tile loop; with a live timer its event pair rides on the kernel's own dispatch (start and end of its
// execution), so the stream carries no extra marker packets and the kernels before and after it are not held up.
template <int G>
void launch_tile_loop(const AttnBatch& batch, dim3 grid, float* partials, int n_parts, const Shape& s, float scale_log2e,
                      KernelTimer* timer, bool timed, hipStream_t st) {
    if (timed) {
        const int slot = (int)(timer->n_recorded % timer->n_slots);
        hipExtLaunchKernelGGL((attn_fixed_ref_kernel<G>), grid, dim3(256), (uint32_t)LDS_FAST, st, timer->start[slot],
                              timer->stop[slot], 0u, batch, partials, n_parts, s.Hq, s.Hkv, scale_log2e);
        ++timer->n_recorded;
    } else {
        attn_fixed_ref_kernel<G><<<grid, dim3(256), LDS_FAST, st>>>(batch, partials, n_parts, s.Hq, s.Hkv, scale_log2e);
    }
}

// Parts per item of a one-query launch of `items` (row tile, KV head) items over n_img_tiles key tiles.  With few items
// the chip would idle behind the longest ones (rows ascend by position: the question rows' tiles walk the whole prompt),
// so every item's key tiles are dealt to several workgroups.  Measured on a 17k-token prompt (256 compute units, one
// workgroup each): two parts pay up to about 400 items (recompute ratios up to 15 %; at 30 %, 680 items, the partial
// results' traffic and the combine pass cost more than the balance gains); below half a workgroup per compute unit more
// parts pay until there is about one piece per compute unit (question-only prefill, 64 items: 4 parts, 0.24 -> 0.17 ms);
// in between two parts stay best (168 items at 5 %, 128 items of the offline stage: three or four parts lose 3-15 %).
int choose_parts(int split_mode, int items, int n_img_tiles, int n_cu, size_t partials_bytes) {
    int parts = 1;
    if (split_mode == FR_ATTN_SPLIT_ON) parts = 2;
    if (split_mode == FR_ATTN_SPLIT_AUTO && n_img_tiles >= 32 && items <= ATTN_SPLIT_AUTO_ITEMS)
        parts = std::max(2, std::min(ATTN_MAX_PARTS, n_cu / std::max(items, 1)));
    while (parts > 1 && (size_t)items * parts * PART_FLOATS * sizeof(float) > partials_bytes) --parts;
    return parts;
}

template <int G>
hipError_t launch(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                  const void* v_cache, int64_t L, const void* k_new, const void* v_new, void* out, float* lse,
                  const Workspace& ws, int mode, int split_mode, const SharedStoreArgs* shared, KernelTimer* timer,
                  bool writeback, hipStream_t st) {
    hipError_t e = set_kernel_attributes<G>();
    if (e != hipSuccess) return e;
    const float scale_log2e = (1.0f / sqrtf((float)s.d)) * 1.4426950408889634f;
    const QueryScratch sc{ws.store_row_map, ws.chunk_id_map, ws.kv_images, ws.kv_images_bytes, ws.attn_flags,
                          ws.attn_flags_elems};
    AttnBatch batch;
    batch.n = 1;
    e = pack_query<G>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse, sc, shared, writeback, &batch.q[0], st);
    if (e != hipSuccess) return e;
    batch.max_row_tiles = batch.q[0].n_row_tiles;
    const int items = batch.q[0].n_row_tiles * s.Hkv;
    const dim3 grid(items);
    if (mode == FR_ATTN_SOFTMAX_RUNNING_MAX) {   // every item with the running maximum
        attn_running_max_kernel<G><<<grid, dim3(256), LDS_SAFE, st>>>(batch, 0, s.Hq, s.Hkv, scale_log2e);
        return hipGetLastError();
    }
    const int n_parts = choose_parts(split_mode, items, batch.q[0].n_img_tiles, ws.n_cu, ws.attn_partials_bytes);
    const bool timed = timer != nullptr && timer->n_slots > 0;
    launch_tile_loop<G>(batch, dim3(items * n_parts), ws.attn_partials, n_parts, s, scale_log2e, timer, timed, st);
    if (n_parts > 1)   // adds the parts, stores, and recomputes the items whose sums overflowed
        attn_combine_kernel<G><<<grid, dim3(256), LDS_SAFE, st>>>(batch.q[0], ws.attn_partials, n_parts, s.Hq, s.Hkv, scale_log2e);
    else               // recomputes the items whose workgroups raised their flag
        attn_running_max_kernel<G><<<grid, dim3(256), LDS_SAFE, st>>>(batch, 1, s.Hq, s.Hkv, scale_log2e);
    return hipGetLastError();
}

template <int G>
hipError_t launch_shared_batch(const Shape& s, int n, const SharedBatchQuery* qs, const void* k_store,
                               const void* v_store, int mode, KernelTimer* timer, hipStream_t st) {
    hipError_t e = set_kernel_attributes<G>();
    if (e != hipSuccess) return e;
    const float scale_log2e = (1.0f / sqrtf((float)s.d)) * 1.4426950408889634f;
    AttnBatch batch;
    batch.n = n;
    batch.max_row_tiles = 0;
    for (int i = 0; i < n; ++i) {
        const SharedBatchQuery& q = qs[i];
        const QueryScratch sc{q.store_row_map, q.chunk_id_map, q.images, q.images_bytes, q.flags, q.flags_elems};
        e = pack_query<G>(s, q.q_rows, q.q_index, q.R, k_store, v_store, q.L, q.k_new, q.v_new, q.out, q.lse, sc, &q.shared,
                          false, &batch.q[i], st);
        if (e != hipSuccess) return e;
        batch.max_row_tiles = std::max(batch.max_row_tiles, batch.q[i].n_row_tiles);
    }
    // a batch of queries fills the chip by itself: every item whole, one workgroup each
    const dim3 grid(batch.max_row_tiles * n * s.Hkv);
    if (mode == FR_ATTN_SOFTMAX_RUNNING_MAX) {
        attn_running_max_kernel<G><<<grid, dim3(256), LDS_SAFE, st>>>(batch, 0, s.Hq, s.Hkv, scale_log2e);
    } else {
        launch_tile_loop<G>(batch, grid, nullptr, 1, s, scale_log2e, timer, timer != nullptr && timer->n_slots > 0, st);
        attn_running_max_kernel<G><<<grid, dim3(256), LDS_SAFE, st>>>(batch, 1, s.Hq, s.Hkv, scale_log2e);
    }
    return hipGetLastError();
}

}  // namespace

// Partial results of a launch in parts: one slot of 132 KB per piece.
size_t attn_mfma_partials_bytes(const Shape& s, int64_t max_tokens) {
    const int64_t tr = 4 * (64 / s.G);   // token rows per workgroup
    const int64_t items = std::min<int64_t>(((max_tokens + tr - 1) / tr) * s.Hkv, ATTN_SPLIT_AUTO_ITEMS);
    return (size_t)(2 * items) * PART_FLOATS * sizeof(float);   // two parts of the most items that are split without being asked
}

bool attn_mfma_supported(const Shape& s) {
    return s.dtype == FR_BF16 && s.d == 128 && (s.G == 1 || s.G == 2 || s.G == 4 || s.G == 8);
}

hipError_t launch_attn_mfma(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                            const void* v_cache, int64_t L, const void* k_new, const void* v_new, void* out, float* lse,
                            const Workspace& ws, int mode, int split_mode, const SharedStoreArgs* shared,
                            KernelTimer* timer, bool writeback, hipStream_t st) {
    if (R == 0) return hipSuccess;
    switch (s.G) {
        case 1: return launch<1>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse, ws, mode, split_mode, shared, timer, writeback, st);
        case 2: return launch<2>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse, ws, mode, split_mode, shared, timer, writeback, st);
        case 4: return launch<4>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse, ws, mode, split_mode, shared, timer, writeback, st);
        default: return launch<8>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, out, lse, ws, mode, split_mode, shared, timer, writeback, st);
    }
}

size_t attn_mfma_images_bytes(const Shape& s, int64_t L) { return (size_t)((L + KT - 1) / KT) * s.Hkv * IMG_BYTES; }
size_t attn_mfma_flags_elems(const Shape& s, int64_t R) { return (size_t)(R / 32 + 1) * s.Hkv; }

hipError_t launch_attn_mfma_shared_batch(const Shape& s, int n, const SharedBatchQuery* qs, const void* k_store,
                                         const void* v_store, int mode, KernelTimer* timer, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (n > ATTN_MAX_BATCH) return hipErrorInvalidValue;
    switch (s.G) {
        case 1: return launch_shared_batch<1>(s, n, qs, k_store, v_store, mode, timer, st);
        case 2: return launch_shared_batch<2>(s, n, qs, k_store, v_store, mode, timer, st);
        case 4: return launch_shared_batch<4>(s, n, qs, k_store, v_store, mode, timer, st);
        default: return launch_shared_batch<8>(s, n, qs, k_store, v_store, mode, timer, st);
    }
}

}  // namespace fr
