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
//   * V is transposed once per tile while it is staged into LDS (4 keys x 8 dims per lane,
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
// Stale entries.  Key j is read from k_new/v_new when inv[j] >= 0 (its token is in the Q index)
// and from the cache otherwise: the cache is never written and stale rows are never read.
#include "fr_internal.hpp"

namespace fr {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int D = 128;           // head_dim
constexpr int KT = 64;           // keys per tile
constexpr int K_PITCH = D + 8;   // bf16 elements per K row in LDS (272 B: 16-byte reads hit distinct banks)
constexpr int O_PITCH = D + 8;   // bf16 elements per output row in the epilogue's LDS staging
constexpr float NEG_BIG = -1.0e30f;

struct __attribute__((aligned(16))) Stage {
    __bf16 k[KT * K_PITCH];   // [key][d], rows padded to 272 B
    __bf16 vt[D * KT];        // [d][key slot], 128-byte rows, 16-byte chunks XOR-swizzled (see vt_chunk)
};
// The fast kernel keeps separate rings of three K tiles and three V^T tiles (see its tile loop).
struct __attribute__((aligned(16))) Rings {
    __bf16 k[3][KT * K_PITCH];
    __bf16 vt[3][D * KT];
};
constexpr size_t EPILOGUE_LDS = 4 * 64 * O_PITCH * sizeof(__bf16);   // four waves x [64 columns][d] bf16

// V^T rows are exactly 128 bytes (all 32 LDS banks), so both the transposing writes (one lane per 8-dim
// group, rows 8 apart) and the operand reads (one lane per row, 32 consecutive rows) would pile onto the
// same banks.  The 16-byte chunk index is therefore XORed with a key that differs between rows 1 apart
// and between rows 8 apart.
__device__ __forceinline__ int vt_chunk(int dd, int chunk) { return chunk ^ ((dd ^ (dd >> 3)) & 7); }

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

    __device__ __forceinline__ void init(const int32_t* __restrict__ q_index, int R, int Hkv, int n_row_tiles) {
        const int tid = threadIdx.x, lane = tid & 63;
        wave = tid >> 6;
        x = lane & 31;
        h = lane >> 5;
        g = blockIdx.x % Hkv;                               // consecutive blocks land on different XCDs
        tile = n_row_tiles - 1 - (int)(blockIdx.x / Hkv);   // longest tiles first
        row0 = tile * TR;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int col = 32 * nb + x;
            const int r = row0 + wave * TRW + (col % TRW);
            col_row[nb] = r;                                 // rows past the end compute a copy of the last
            col_head[nb] = g * G + col / TRW;                // row and are never stored
            col_pos[nb] = q_index[min(r, R - 1)];
        }
        const int p_first = q_index[row0];                   // rows ascend: every key <= p_first is visible to all
        const int p_max = q_index[min(R, row0 + TR) - 1];    // the workgroup's furthest key
        wp_max = q_index[min(row0 + wave * TRW + TRW, R) - 1];   // a wave past the end copies the last row
        n_kt = p_max / KT + 1;
        n_plain = min((p_first + 1) / KT, n_kt - 1);
    }
};

// ---- staging: global -> registers -> LDS ------------------------------------------------------------
// Loads never branch: a key past the end of the cache is clamped to the last row (it lies beyond every
// row's position, so the causal mask removes it), and the cache / fresh-row choice is a pointer select.
template <bool HAS_NEW>
struct Stager {
    const __bf16 *k_cache, *v_cache, *k_new, *v_new;
    const int32_t* inv;
    int L, Hkv, g;
    int st_vec, st_key, kslot;
    u32x4 kreg[4], vreg[4];

    __device__ __forceinline__ void init(const __bf16* kc, const __bf16* vc, const __bf16* kn, const __bf16* vn,
                                         const int32_t* iv, int L_, int Hkv_, int g_) {
        k_cache = kc; v_cache = vc; k_new = kn; v_new = vn; inv = iv; L = L_; Hkv = Hkv_; g = g_;
        st_vec = threadIdx.x & 15;   // 16-byte vector within a 256-byte head row
        st_key = threadIdx.x >> 4;   // K: keys st_key + 16 i;  V: key group st_key (4 consecutive keys)
        kslot = 16 * (st_key >> 2) + 4 * ((0x3120 >> (4 * (st_key & 3))) & 3);   // permuted slot of key 4*st_key
    }
    // The position -> fresh-row map is read one step ahead of the rows themselves (fetch_inv_* for tile kt+1
    // right after load_* of tile kt), so that a row load never waits on the lookup that addresses it.
    int inv_k[4], inv_v[4];
    __device__ __forceinline__ void fetch_inv_k(int kt) {
        if (!HAS_NEW) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) inv_k[i] = inv[min(kt * KT + st_key + 16 * i, L - 1)];
    }
    __device__ __forceinline__ void fetch_inv_v(int kt) {
        if (!HAS_NEW) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) inv_v[i] = inv[min(kt * KT + 4 * st_key + i, L - 1)];
    }
    __device__ __forceinline__ void load_k(int kt) {   // needs fetch_inv_k(kt) before
        const int key0 = kt * KT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jk = min(key0 + st_key + 16 * i, L - 1);
            const __bf16* pk = k_cache + ((size_t)jk * Hkv + g) * D;
            if (HAS_NEW) {
                const int rk = inv_k[i];
                const __bf16* nk = k_new + ((size_t)max(rk, 0) * Hkv + g) * D;
                pk = (rk >= 0) ? nk : pk;
            }
            kreg[i] = *reinterpret_cast<const u32x4*>(pk + 8 * st_vec);
        }
    }
    __device__ __forceinline__ void load_v(int kt) {   // needs fetch_inv_v(kt) before
        const int key0 = kt * KT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jv = min(key0 + 4 * st_key + i, L - 1);
            const __bf16* pv = v_cache + ((size_t)jv * Hkv + g) * D;
            if (HAS_NEW) {
                const int rv = inv_v[i];
                const __bf16* nv = v_new + ((size_t)max(rv, 0) * Hkv + g) * D;
                pv = (rv >= 0) ? nv : pv;
            }
            vreg[i] = *reinterpret_cast<const u32x4*>(pv + 8 * st_vec);
        }
    }
    __device__ __forceinline__ void load(int kt) { fetch_inv_k(kt); fetch_inv_v(kt); load_k(kt); load_v(kt); }
    __device__ __forceinline__ void write_k(__bf16* k) const {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<u32x4*>(&k[(st_key + 16 * i) * K_PITCH + 8 * st_vec]) = kreg[i];
    }
    __device__ __forceinline__ void write_v(__bf16* vt) const {
#pragma unroll
        for (int c = 0; c < 4; ++c) {   // dims 8*st_vec + 2c, +2c+1: gather the 4 keys of each
            u32x2 lo, hi;
            lo[0] = perm_lo(vreg[0][c], vreg[1][c]);
            lo[1] = perm_lo(vreg[2][c], vreg[3][c]);
            hi[0] = perm_hi(vreg[0][c], vreg[1][c]);
            hi[1] = perm_hi(vreg[2][c], vreg[3][c]);
            const int d0 = 8 * st_vec + 2 * c, d1 = d0 + 1;
            *reinterpret_cast<u32x2*>(&vt[d0 * KT + 8 * vt_chunk(d0, kslot >> 3) + (kslot & 4)]) = lo;
            *reinterpret_cast<u32x2*>(&vt[d1 * KT + 8 * vt_chunk(d1, kslot >> 3) + (kslot & 4)]) = hi;
        }
    }
    __device__ __forceinline__ void write(Stage& st) const { write_k(st.k); write_v(st.vt); }
};

// S^T for 32 keys (half mb of a staged tile) against this wave's 64 query columns.
__device__ __forceinline__ void qk_half(const __bf16* k, int mb, const bf16x8 (&qf)[2][8], int x, int h, f32x16 (&s)[2]) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&k[(32 * mb + x) * K_PITCH + 16 * ks + 8 * h]);
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
__device__ __forceinline__ void pv_half(const __bf16* vt, int mb, const bf16x8 (&pf)[2][2], int x, int h, f32x16 (&o)[4][2]) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int kb = 2 * mb + kk;
#pragma unroll
        for (int md = 0; md < 4; ++md) {
            const int dd = 32 * md + x;
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&vt[dd * KT + 8 * vt_chunk(dd, 2 * kb + h)]);
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
__device__ __forceinline__ void pipeline_step(const __bf16* k_next, int mb_next, const __bf16* vt_prev, int mb_prev,
                                              const bf16x8 (&qf)[2][8], f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2],
                                              const bf16x8 (&pf_prev)[2][2], bf16x8 (&pf_cur)[2][2], f32x16 (&o)[4][2],
                                              float (&lsum)[2], const float (&mref)[2], const int (&col_pos)[2],
                                              int key_base, int x, int h, float scale_log2e) {
    mask_half<MASK>(s_cur, col_pos, key_base, h);
    if (DO_QK) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s_nxt[nb][v] = 0.f;
    }
    // strand 1 + first half of the weights (query column block 0)
    float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        if (DO_QK) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&k_next[(32 * mb_next + x) * K_PITCH + 16 * ks + 8 * h]);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                s_nxt[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], s_nxt[nb], 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int v = 2 * ks + e;
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[0][v], scale_log2e, -mref[0]));
            psum0 += p;
            pf_cur[0][v >> 3][v & 7] = (__bf16)p;
        }
    }
    // strand 2 + second half of the weights (query column block 1)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int kb = 2 * mb_prev + kk;
#pragma unroll
        for (int md = 0; md < 4; ++md) {
            const int dd = 32 * md + x;
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(&vt_prev[dd * KT + 8 * vt_chunk(dd, 2 * kb + h)]);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                o[md][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf_prev[nb][kk], o[md][nb], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int v = 8 * kk + 2 * md + e;
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[1][v], scale_log2e, -mref[1]));
                psum1 += p;
                pf_cur[1][v >> 3][v & 7] = (__bf16)p;
            }
        }
    }
    lsum[0] += psum0;
    lsum[1] += psum1;
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

// ---- fast kernel ---------------------------------------------------------------------------------
// grid.x = n_row_tiles * Hkv.  Dynamic LDS: the larger of the K/V rings and the epilogue's staging.
template <int G, bool HAS_NEW>
__global__ __launch_bounds__(256) void attn_fixed_ref_kernel(const __bf16* __restrict__ q_rows,
                                                             const int32_t* __restrict__ q_index, int R,
                                                             const __bf16* __restrict__ k_cache,
                                                             const __bf16* __restrict__ v_cache, int L,
                                                             const __bf16* __restrict__ k_new,
                                                             const __bf16* __restrict__ v_new,
                                                             const int32_t* __restrict__ inv, __bf16* __restrict__ out,
                                                             float* __restrict__ lse_out, int32_t* __restrict__ redo_flags,
                                                             int Hq, int Hkv, int n_row_tiles, float scale_log2e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Rings& rg = *reinterpret_cast<Rings*>(smem_raw);
    Geometry<G> ge;
    ge.init(q_index, R, Hkv, n_row_tiles);
    const int x = ge.x, h = ge.h;

    // Q fragments: B operand of S^T = K Q^T, kept in registers for the whole loop
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

    // ---- prologue: K tiles 0 and 1 and V tile 0 in LDS, K tile 2 and V tile 1 in flight -----------------
    Stager<HAS_NEW> sg;
    sg.init(k_cache, v_cache, k_new, v_new, inv, L, Hkv, ge.g);
    const int n_kt = ge.n_kt;
    sg.fetch_inv_k(0);
    sg.fetch_inv_v(0);
    sg.load_k(0);
    sg.load_v(0);
    sg.fetch_inv_k(1);
    sg.fetch_inv_v(1);
    {   // V ring slot 2 is read (against all-zero weights) by the very first step: it must hold finite numbers
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 4; ++i) reinterpret_cast<u32x4*>(rg.vt[2])[threadIdx.x + 256 * i] = z;
    }
    sg.write_k(rg.k[0]);
    sg.write_v(rg.vt[0]);
    if (n_kt > 1) {
        sg.load_k(1);
        sg.fetch_inv_k(2);
        sg.write_k(rg.k[1]);
        sg.load_v(1);
        sg.fetch_inv_v(2);
    }
    if (n_kt > 2) {
        sg.load_k(2);
        sg.fetch_inv_k(3);
    }
    __syncthreads();

    // logits of the first 32 keys; exponent reference of each column = their maximum over the visible ones
    f32x16 s_a[2], s_b[2];
    qk_half(rg.k[0], 0, qf, x, h, s_a);
    float mref[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        float t = s_a[nb][0];   // key 0 (h = 0) or key 4 (h = 1); key 0 is visible to every row
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = 8 * (v >> 2) + 4 * h + (v & 3);
            t = fmaxf(t, key <= ge.col_pos[nb] ? s_a[nb][v] : NEG_BIG);
        }
        if (h == 1 && ge.col_pos[nb] < 4) t = NEG_BIG;
        t = fmaxf(t, __shfl_xor(t, 32));
        mref[nb] = t * scale_log2e;
    }
    bf16x8 pf_a[2][2], pf_b[2][2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf_b[nb][kk][e] = (__bf16)0.0f;

    // ---- tile loop ------------------------------------------------------------------------------------
    // Iteration kt, after its barrier: K tile kt+2 and V tile kt+1 move from registers into their rings, the
    // loads of K tile kt+3 and V tile kt+2 are issued, and two pipeline steps run:
    //   step (kt, 0): weights of keys [64kt, 64kt+32)    | logits of (kt, 1) from K[kt]     | O += half (kt-1, 1), V[kt-1]
    //   step (kt, 1): weights of keys [64kt+32, 64kt+64) | logits of (kt+1, 0) from K[kt+1] | O += half (kt, 0),   V[kt]
    // A ring slot is rewritten two iterations after its last reader, so one barrier per tile suffices.
    int k0 = 0, k1 = 1, k2 = 2;   // ring slots of tiles kt, kt+1, kt+2 (K);  V tile kt-1 sits in slot k2, kt in k0, kt+1 in k1
    int kt = 0;
    for (; kt < ge.n_plain; ++kt) {   // plain tiles: every key visible to every row; a next tile always exists
        if (kt > 0) __syncthreads();
        if (kt + 2 < n_kt) sg.write_k(rg.k[k2]);
        sg.write_v(rg.vt[k1]);
        if (kt + 3 < n_kt) { sg.load_k(kt + 3); sg.fetch_inv_k(kt + 4); }
        if (kt + 2 < n_kt) { sg.load_v(kt + 2); sg.fetch_inv_v(kt + 3); }
        pipeline_step<false, true>(rg.k[k0], 1, rg.vt[k2], 1, qf, s_a, s_b, pf_b, pf_a, o, lsum, mref, ge.col_pos,
                                   kt * KT, x, h, scale_log2e);
        // (V tile kt+1 was just written to slot k1; slot k2 is free for K tile kt+2 -- written above -- because the
        //  K and V rings are separate arrays)
        pipeline_step<false, true>(rg.k[k1], 0, rg.vt[k0], 0, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref, ge.col_pos,
                                   kt * KT + 32, x, h, scale_log2e);
        const int t = k0; k0 = k1; k1 = k2; k2 = t;
    }
    for (; kt < n_kt; ++kt) {         // tiles that cross some row's own position
        if (kt > 0) __syncthreads();
        if (kt + 2 < n_kt) sg.write_k(rg.k[k2]);
        if (kt + 1 < n_kt) sg.write_v(rg.vt[k1]);
        if (kt + 3 < n_kt) { sg.load_k(kt + 3); sg.fetch_inv_k(kt + 4); }
        if (kt + 2 < n_kt) { sg.load_v(kt + 2); sg.fetch_inv_v(kt + 3); }
        pipeline_step<true, true>(rg.k[k0], 1, rg.vt[k2], 1, qf, s_a, s_b, pf_b, pf_a, o, lsum, mref, ge.col_pos,
                                  kt * KT, x, h, scale_log2e);
        if (kt + 1 < n_kt)
            pipeline_step<true, true>(rg.k[k1], 0, rg.vt[k0], 0, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref, ge.col_pos,
                                      kt * KT + 32, x, h, scale_log2e);
        else
            pipeline_step<true, false>(rg.k[k1], 0, rg.vt[k0], 0, qf, s_b, s_a, pf_a, pf_b, o, lsum, mref, ge.col_pos,
                                       kt * KT + 32, x, h, scale_log2e);
        const int t = k0; k0 = k1; k1 = k2; k2 = t;
    }
    pv_half(rg.vt[k2], 1, pf_b, x, h, o);   // the last half: tile n_kt-1 now sits in slot k2

    // overflow check: with a fixed reference a runaway logit shows up as inf / nan in the sums
    float l[2];
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
    const int any_bad = __syncthreads_or(bad ? 1 : 0);   // also: every wave is done with the stages
    if (threadIdx.x == 0) redo_flags[blockIdx.x] = any_bad;
    if (any_bad) return;
    store_output<G>(ge, o, l, mref, R, Hq, smem_raw, out, lse_out);
}

// ---- safe kernel: classic online softmax, runs only where the fast kernel raised its flag ----------
template <int G, bool HAS_NEW>
__global__ __launch_bounds__(256) void attn_running_max_kernel(const __bf16* __restrict__ q_rows,
                                                               const int32_t* __restrict__ q_index, int R,
                                                               const __bf16* __restrict__ k_cache,
                                                               const __bf16* __restrict__ v_cache, int L,
                                                               const __bf16* __restrict__ k_new,
                                                               const __bf16* __restrict__ v_new,
                                                               const int32_t* __restrict__ inv, __bf16* __restrict__ out,
                                                               float* __restrict__ lse_out,
                                                               const int32_t* __restrict__ redo_flags, int Hq, int Hkv,
                                                               int n_row_tiles, float scale_log2e) {
    if (redo_flags != nullptr && redo_flags[blockIdx.x] == 0) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Stage* stages = reinterpret_cast<Stage*>(smem_raw);
    Geometry<G> ge;
    ge.init(q_index, R, Hkv, n_row_tiles);
    const int x = ge.x, h = ge.h;
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
    Stager<HAS_NEW> sg;
    sg.init(k_cache, v_cache, k_new, v_new, inv, L, Hkv, ge.g);
    for (int kt = 0; kt < ge.n_kt; ++kt) {
        sg.load(kt);
        __syncthreads();
        sg.write(stages[0]);
        __syncthreads();
        if (kt * KT > ge.wp_max) continue;   // wave-uniform; the barriers stay outside
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            f32x16 s[2];
            qk_half(stages[0].k, mb, qf, x, h, s);
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
            pv_half(stages[0].vt, mb, pf, x, h, o);
        }
    }
    float l[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) l[nb] = lsum[nb] + __shfl_xor(lsum[nb], 32);
    __syncthreads();
    store_output<G>(ge, o, l, m2, R, Hq, smem_raw, out, lse_out);
}

template <int G, bool HAS_NEW>
hipError_t launch(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                  const void* v_cache, int64_t L, const void* k_new, const void* v_new, const int32_t* inv, void* out,
                  float* lse, const Workspace& ws, int mode, hipStream_t st) {
    const float scale_log2e = (1.0f / sqrtf((float)s.d)) * 1.4426950408889634f;
    constexpr int TR = Geometry<G>::TR;
    const int n_row_tiles = (R + TR - 1) / TR;
    const size_t lds_fast = sizeof(Rings) > EPILOGUE_LDS ? sizeof(Rings) : EPILOGUE_LDS;
    const size_t lds_safe = sizeof(Stage) > EPILOGUE_LDS ? sizeof(Stage) : EPILOGUE_LDS;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fixed_ref_kernel<G, HAS_NEW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_fast);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_running_max_kernel<G, HAS_NEW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_safe);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(n_row_tiles * s.Hkv), block(256);
    if ((size_t)grid.x > ws.attn_flags_elems) return hipErrorInvalidValue;
    const int32_t* flags = ws.attn_flags;
    if (mode != FR_ATTN_SOFTMAX_RUNNING_MAX)
        attn_fixed_ref_kernel<G, HAS_NEW><<<grid, block, lds_fast, st>>>(
            (const __bf16*)q_rows, q_index, R, (const __bf16*)k_cache, (const __bf16*)v_cache, (int)L,
            (const __bf16*)k_new, (const __bf16*)v_new, inv, (__bf16*)out, lse, ws.attn_flags, s.Hq, s.Hkv, n_row_tiles,
            scale_log2e);
    else
        flags = nullptr;   // recompute every workgroup with the running maximum
    attn_running_max_kernel<G, HAS_NEW><<<grid, block, lds_safe, st>>>(
        (const __bf16*)q_rows, q_index, R, (const __bf16*)k_cache, (const __bf16*)v_cache, (int)L, (const __bf16*)k_new,
        (const __bf16*)v_new, inv, (__bf16*)out, lse, flags, s.Hq, s.Hkv, n_row_tiles, scale_log2e);
    return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(const Shape& s) {
    return s.dtype == FR_BF16 && s.d == 128 && (s.G == 1 || s.G == 2 || s.G == 4 || s.G == 8);
}

hipError_t launch_attn_mfma(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                            const void* v_cache, int64_t L, const void* k_new, const void* v_new, const int32_t* inv,
                            void* out, float* lse, const Workspace& ws, int mode, hipStream_t st) {
    if (R == 0) return hipSuccess;
#define FR_GO(GG)                                                                                                    \
    return (k_new != nullptr)                                                                                        \
               ? launch<GG, true>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, inv, out, lse, ws, mode, st) \
               : launch<GG, false>(s, q_rows, q_index, R, k_cache, v_cache, L, k_new, v_new, inv, out, lse, ws, mode, st)
    switch (s.G) {
        case 1: FR_GO(1);
        case 2: FR_GO(2);
        case 4: FR_GO(4);
        default: FR_GO(8);
    }
#undef FR_GO
}

}  // namespace fr
