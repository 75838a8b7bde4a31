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
constexpr int V_PITCH = KT + 8;  // bf16 elements per V^T row in LDS (144 B)
constexpr float NEG_BIG = -1.0e30f;

struct __attribute__((aligned(16))) Smem {
    __bf16 k[KT * K_PITCH];   // [key][d]
    __bf16 vt[D * V_PITCH];   // [d][key slot]
};

__device__ __forceinline__ uint32_t perm_lo(uint32_t a, uint32_t b) {  // (a.lo16, b.lo16) -> a in low half
    return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t perm_hi(uint32_t a, uint32_t b) {  // (a.hi16, b.hi16)
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// G = query heads per KV head.  grid.x = n_row_tiles * Hkv.
template <int G>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const __bf16* __restrict__ q_rows,
                                                        const int32_t* __restrict__ q_index, int R,
                                                        const __bf16* __restrict__ k_cache,
                                                        const __bf16* __restrict__ v_cache, int L,
                                                        const __bf16* __restrict__ k_new,
                                                        const __bf16* __restrict__ v_new,
                                                        const int32_t* __restrict__ inv, __bf16* __restrict__ out,
                                                        float* __restrict__ lse_out, int Hq, int Hkv, int n_row_tiles,
                                                        float scale_log2e) {
    constexpr int TRW = 64 / G;   // token rows per wave
    constexpr int TR = 4 * TRW;   // token rows per workgroup
    __shared__ Smem sm;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int x = lane & 31, h = lane >> 5;
    const int g = blockIdx.x % Hkv;                             // consecutive blocks land on different XCDs
    const int tile = n_row_tiles - 1 - (int)(blockIdx.x / Hkv);  // longest tiles first
    const int row0 = tile * TR;

    // ---- this lane's two query columns (one per 32-wide N block) ---------------------------------
    int col_row[2], col_head[2], col_pos[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int col = 32 * nb + x;
        const int r = row0 + wave * TRW + (col % TRW);
        col_row[nb] = r;
        col_head[nb] = g * G + col / TRW;
        col_pos[nb] = (r < R) ? q_index[r] : -1;
    }
    const int last_row = min(R, row0 + TR) - 1;
    const int p_max = q_index[last_row];                        // rows ascend: the tile's furthest key
    const int w_first = row0 + wave * TRW, w_last = min(R, w_first + TRW) - 1;
    const int wp_min = (w_first < R) ? q_index[w_first] : -1;   // every key <= wp_min is visible to the whole wave
    const int wp_max = (w_first < R) ? q_index[w_last] : -1;    // no key > wp_max is visible to any of its rows
    const int n_kt = p_max / KT + 1;

    // ---- Q fragments: B operand of S^T = K Q^T, kept in registers for the whole loop -------------
    bf16x8 qf[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const __bf16* qp = q_rows + ((size_t)col_row[nb] * Hq + col_head[nb]) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (col_row[nb] < R) {
                qf[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[nb][ks][e] = (__bf16)0.0f;
            }
        }
    }

    f32x16 o[4][2];
#pragma unroll
    for (int md = 0; md < 4; ++md)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[md][nb][v] = 0.f;
    float m2[2] = {NEG_BIG, NEG_BIG};   // running max of the scaled (log2 domain) logits, per column
    float lsum[2] = {0.f, 0.f};         // this lane's share of the running denominator

    // staging assignments
    const int st_vec = tid & 15;            // 16-byte vector within a 256-byte head row
    const int st_key = tid >> 4;            // K: keys st_key + 16 i;  V: key group st_key (4 keys)
    const int kslot = 16 * (st_key >> 2) + 4 * ((0x3120 >> (4 * (st_key & 3))) & 3);  // permuted slot of key 4*st_key

    for (int kt = 0; kt < n_kt; ++kt) {
        const int key0 = kt * KT;
        // ---- stage K [key][d] and V^T [d][slot] ------------------------------------------------
        u32x4 kreg[4], vreg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jk = key0 + st_key + 16 * i;
            const int jv = key0 + 4 * st_key + i;
            u32x4 zk = {0u, 0u, 0u, 0u};
            kreg[i] = zk;
            vreg[i] = zk;
            if (jk < L) {
                const int rr = inv ? inv[jk] : -1;
                const __bf16* p = (rr >= 0) ? k_new + ((size_t)rr * Hkv + g) * D : k_cache + ((size_t)jk * Hkv + g) * D;
                kreg[i] = *reinterpret_cast<const u32x4*>(p + 8 * st_vec);
            }
            if (jv < L) {
                const int rr = inv ? inv[jv] : -1;
                const __bf16* p = (rr >= 0) ? v_new + ((size_t)rr * Hkv + g) * D : v_cache + ((size_t)jv * Hkv + g) * D;
                vreg[i] = *reinterpret_cast<const u32x4*>(p + 8 * st_vec);
            }
        }
        __syncthreads();   // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<u32x4*>(&sm.k[(st_key + 16 * i) * K_PITCH + 8 * st_vec]) = kreg[i];
#pragma unroll
        for (int c = 0; c < 4; ++c) {   // dims 8*st_vec + 2c, +2c+1: gather the 4 keys of each
            u32x2 lo, hi;
            lo[0] = perm_lo(vreg[0][c], vreg[1][c]);
            lo[1] = perm_lo(vreg[2][c], vreg[3][c]);
            hi[0] = perm_hi(vreg[0][c], vreg[1][c]);
            hi[1] = perm_hi(vreg[2][c], vreg[3][c]);
            *reinterpret_cast<u32x2*>(&sm.vt[(8 * st_vec + 2 * c) * V_PITCH + kslot]) = lo;
            *reinterpret_cast<u32x2*>(&sm.vt[(8 * st_vec + 2 * c + 1) * V_PITCH + kslot]) = hi;
        }
        __syncthreads();

        if (key0 <= wp_max) {   // otherwise nothing in this tile is visible to this wave
            // ---- S^T = K Q^T -------------------------------------------------------------------
            f32x16 s[2][2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) s[mb][nb][v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sm.k[(32 * mb + x) * K_PITCH + 16 * ks + 8 * h]);
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], s[mb][nb], 0, 0, 0);
                }
            }
            // ---- causal mask by position (only tiles that reach past the wave's first row) ------
            if (key0 + KT - 1 > wp_min) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int key = key0 + 32 * mb + 8 * (v >> 2) + 4 * h + (v & 3);
                            if (key > col_pos[nb]) s[mb][nb][v] = -INFINITY;
                        }
            }
            // ---- online softmax per query column -------------------------------------------------
            bf16x8 pf[2][4];   // P^T as B operand: [nb][16-key block]
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float mx = NEG_BIG;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[mb][nb][v]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m2[nb], mx * scale_log2e);
                const float alpha = __builtin_amdgcn_exp2f(m2[nb] - m_new);
                m2[nb] = m_new;
                float psum = 0.f;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][nb][v], scale_log2e, -m_new));
                        s[mb][nb][v] = p;
                        psum += p;
                    }
                lsum[nb] = lsum[nb] * alpha + psum;
#pragma unroll
                for (int md = 0; md < 4; ++md)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[md][nb][v] *= alpha;
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[nb][kb][e] = (__bf16)s[kb >> 1][nb][8 * (kb & 1) + e];
            }
            // ---- O^T += V^T P^T ------------------------------------------------------------------
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
                for (int md = 0; md < 4; ++md) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sm.vt[(32 * md + x) * V_PITCH + 16 * kb + 8 * h]);
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        o[md][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nb][kb], o[md][nb], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: normalise and store ---------------------------------------------------------
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float l = lsum[nb] + __shfl_xor(lsum[nb], 32);
        if (col_row[nb] < R) {
            const float inv_l = 1.0f / l;
            __bf16* op = out + ((size_t)col_row[nb] * Hq + col_head[nb]) * D;
#pragma unroll
            for (int md = 0; md < 4; ++md)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[md][nb][4 * q4 + e] * inv_l);
                    *reinterpret_cast<bf16x4*>(op + 32 * md + 8 * q4 + 4 * h) = w;
                }
            if (lse_out != nullptr && h == 0)
                lse_out[(size_t)col_row[nb] * Hq + col_head[nb]] = (m2[nb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
        }
    }
}

}  // namespace

bool attn_mfma_supported(const Shape& s) {
    return s.dtype == FR_BF16 && s.d == 128 && (s.G == 1 || s.G == 2 || s.G == 4 || s.G == 8);
}

hipError_t launch_attn_mfma(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                            const void* v_cache, int64_t L, const void* k_new, const void* v_new, const int32_t* inv,
                            void* out, float* lse, const Workspace& ws, hipStream_t st) {
    (void)ws;
    if (R == 0) return hipSuccess;
    const float scale_log2e = (1.0f / sqrtf((float)s.d)) * 1.4426950408889634f;
    const int TR = 4 * (64 / s.G);
    const int n_row_tiles = (R + TR - 1) / TR;
    dim3 grid(n_row_tiles * s.Hkv), block(256);
#define FR_LAUNCH(GG)                                                                                             \
    attn_mfma_kernel<GG><<<grid, block, 0, st>>>((const __bf16*)q_rows, q_index, R, (const __bf16*)k_cache,      \
                                                 (const __bf16*)v_cache, (int)L, (const __bf16*)k_new,           \
                                                 (const __bf16*)v_new, inv, (__bf16*)out, lse, s.Hq, s.Hkv,      \
                                                 n_row_tiles, scale_log2e)
    switch (s.G) {
        case 1: FR_LAUNCH(1); break;
        case 2: FR_LAUNCH(2); break;
        case 4: FR_LAUNCH(4); break;
        default: FR_LAUNCH(8); break;
    }
#undef FR_LAUNCH
    return hipGetLastError();
}

}  // namespace fr
