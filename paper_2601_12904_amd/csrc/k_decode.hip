// Batch decoding attention over shared chunk caches and per-query exclusive pages (Sec. 4.3; decoding
// step of Sec. 2.1: the last token attends to all past K/V).
//
// The chunk store is shared by the batch and never written.  A query's prompt is a list of segments of store
// rows; the keys of a segment were cached `delta` positions away from where they sit in this prompt.  Instead
// of rotating the keys (which would need a private copy per query), the kernel rotates the query the other way
// once per segment: <RoPE(k, +delta), q> = <k, RoPE(q, -delta)> (Appendix A: RoPE is a rotation, additive in the
// position).  Store rows whose tokens the query recomputed are skipped by a per-query bit mask; their fresh
// K/V, the question's and the generated tokens' live in the query's exclusive page, which is one more segment
// (delta 0, no mask).
//
// HBM-bound streaming (2 flop per byte): one workgroup per (segment or page, KV head), every lane reads 16
// bytes of a key row and of the matching value row, the LPK lanes of a row reduce their partial dot products
// by shuffles, all vector-ALU work is in fp32.  Every lane keeps an online-softmax state for the rows it has
// seen; lanes, waves and finally the segments of a query are merged in a fixed order (reproducible results).
#include "fr_internal.hpp"

namespace fr {

namespace {

constexpr float NEG_BIG = -1.0e30f;
constexpr int UNROLL = 4;   // key rows in flight per lane group

template <typename T>
struct Row16;
template <>
struct Row16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& w, float (&f)[4]) {
        f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y); f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
    }
};
template <>
struct Row16<__bf16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& w, float (&f)[8]) {   // a bf16 is the upper half of an fp32
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(u[e] << 16);
            f[2 * e + 1] = __uint_as_float(u[e] & 0xFFFF0000u);
        }
    }
};

// Sum over the LPK consecutive lanes that share a key row, left in every one of them.  Data-parallel-primitive
// moves inside a row of 16 lanes (no LDS round trip): swap neighbours, swap pairs, mirror within 8, mirror within 16.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float t) {
    return t + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), CTRL, 0xF, 0xF, true));
}
template <int LPK>
__device__ __forceinline__ float row_group_sum(float t) {
    t = dpp_add<0xB1>(t);                     // quad_perm [1,0,3,2]
    t = dpp_add<0x4E>(t);                     // quad_perm [2,3,0,1]
    t = dpp_add<0x141>(t);                    // row_half_mirror: the other quad of the 8
    if (LPK >= 16) t = dpp_add<0x140>(t);     // row_mirror: the other half of the 16
    if (LPK >= 32) t += __shfl_xor(t, 16);
    return t;
}

// Partial result of one (unit, query head): [m (base-2 exponent reference), l, o[D]] in fp32.
template <int D>
constexpr int part_floats() { return D + 2; }

// What a workgroup streams.  unit u < n_seg: segment u of the shared store; unit n_seg + b: the exclusive page of
// query b.  The pages are usually the longest units, so the grid starts with them (blockIdx.x < B) and the tail
// consists of segments.  Rows outside the tensors are never read, whatever the descriptors say.
template <typename T>
struct Unit {
    int unit, b, delta;
    int64_t row0, len;
    const T *kbase, *vbase;
    const uint32_t* stale;
    __device__ __forceinline__ void resolve(int B, const T* k_shared, const T* v_shared, int64_t n_shared,
                                            const int32_t* seg_offsets, const int32_t* seg_row0, const int32_t* seg_len,
                                            const int32_t* seg_delta, int n_seg, const uint32_t* stale_bits,
                                            int64_t stale_words, const T* k_pages, const T* v_pages, int64_t page_stride,
                                            const int32_t* page_len, size_t row_elems) {
        unit = ((int)blockIdx.x < B) ? n_seg + (int)blockIdx.x : (int)blockIdx.x - B;
        stale = nullptr;
        int64_t limit;
        if (unit < n_seg) {
            int lo = 0, hi = B;   // largest b with seg_offsets[b] <= unit
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (seg_offsets[mid] <= unit) lo = mid; else hi = mid;
            }
            b = lo;
            row0 = seg_row0[unit];
            len = seg_len[unit];
            delta = seg_delta[unit];
            kbase = k_shared;
            vbase = v_shared;
            limit = n_shared;
            if (stale_bits != nullptr && stale_words > 0) stale = stale_bits + (size_t)b * stale_words;
        } else {
            b = unit - n_seg;
            row0 = 0;
            len = page_len[b];
            delta = 0;
            kbase = k_pages + (size_t)b * page_stride * row_elems;
            vbase = v_pages + (size_t)b * page_stride * row_elems;
            limit = page_stride;
        }
        if (row0 < 0) { len += row0; row0 = 0; }
        if (row0 + len > limit) len = limit - row0;
        if (len < 0) len = 0;
    }
};

// Generic streaming kernel (any dtype / head_dim): all arithmetic on the vector ALU.
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_partial_kernel(
    const T* __restrict__ q, int B, const T* __restrict__ k_shared, const T* __restrict__ v_shared, int64_t n_shared,
    const int32_t* __restrict__ seg_offsets, const int32_t* __restrict__ seg_row0, const int32_t* __restrict__ seg_len,
    const int32_t* __restrict__ seg_delta, int n_seg, const uint32_t* __restrict__ stale_bits, int64_t stale_words,
    const T* __restrict__ k_pages, const T* __restrict__ v_pages, int64_t page_stride, const int32_t* __restrict__ page_len,
    int Hq, int Hkv, const float2* __restrict__ rot_table, int rope_layout, float scale_log2e,
    float* __restrict__ partials) {
    constexpr int N = Row16<T>::N;              // elements per 16-byte vector
    constexpr int LPK = D / N;                  // lanes per key row (8, 16 or 32)
    constexpr int KPW = 64 / LPK;               // key rows per wave and step
    constexpr int PF = part_floats<D>();
    __shared__ float merge[4][G][PF];           // per-wave results

    const int g = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = lane % LPK, r = lane / LPK;
    const size_t row_elems = (size_t)Hkv * D;
    Unit<T> un;
    un.resolve(B, k_shared, v_shared, n_shared, seg_offsets, seg_row0, seg_len, seg_delta, n_seg, stale_bits, stale_words,
               k_pages, v_pages, page_stride, page_len, row_elems);
    const int unit = un.unit, b = un.b, delta = un.delta;
    const int64_t row0 = un.row0, len = un.len;
    const T *kbase = un.kbase, *vbase = un.vbase;
    const uint32_t* stale = un.stale;

    // ---- this lane's slice of the G query heads, rotated by -delta ---------------------------------------
    float qr[G][N];
    {
        const int e0 = c * N;
        float cs[N], sn[N];   // per element: cos / signed sin of its pair's angle
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const int idx = e0 + e;
            const int pair = (rope_layout == FR_ROPE_INTERLEAVED) ? (idx >> 1) : (idx % (D / 2));
            const bool first = (rope_layout == FR_ROPE_INTERLEAVED) ? ((idx & 1) == 0) : (idx < D / 2);
            float2 t = make_float2(1.f, 0.f);
            if (delta != 0) t = rot_table[(size_t)unit * (D / 2) + pair];   // (cos, sin)(delta theta_pair)
            cs[e] = t.x;
            sn[e] = first ? t.y : -t.y;   // RoPE(q, -delta): a' = a cos + b sin, b' = b cos - a sin
        }
#pragma unroll
        for (int col = 0; col < G; ++col) {
            const T* qp = q + ((size_t)b * Hq + g * G + col) * D;
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const int idx = e0 + e;
                const int partner = (rope_layout == FR_ROPE_INTERLEAVED) ? (idx ^ 1) : ((idx + D / 2) % D);
                qr[col][e] = Elem<T>::to_f32(qp[idx]) * cs[e] + Elem<T>::to_f32(qp[partner]) * sn[e];
            }
        }
    }

    // ---- stream the rows -------------------------------------------------------------------------------
    float m[G], l[G], o[G][N];
#pragma unroll
    for (int col = 0; col < G; ++col) {
        m[col] = NEG_BIG;
        l[col] = 0.f;
#pragma unroll
        for (int e = 0; e < N; ++e) o[col][e] = 0.f;
    }
    const T* kp = kbase + (size_t)g * D + c * N;
    const T* vp = vbase + (size_t)g * D + c * N;
    // row i of the unit belongs to (step, wave, r) with i = (step * 4 + wave) * KPW + r; the trip count is the same
    // for all lanes of a wave (the shuffles below need every lane)
    for (int64_t w0 = (int64_t)wave * KPW; w0 < len; w0 += (int64_t)UNROLL * 4 * KPW) {
        uint4 kw[UNROLL], vw[UNROLL];
        bool ok[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = w0 + r + (int64_t)u * 4 * KPW;
            const int64_t row = row0 + min(i, len - 1);   // clamped: the load is always in bounds
            const int64_t wd = row >> 5;
            uint32_t word = 0u;   // (uniform branch; the per-lane part is branch-free so that the loads stay in flight)
            if (stale != nullptr) word = stale[min(wd, stale_words - 1)];
            ok[u] = (i < len) && !((wd < stale_words) && ((word >> (row & 31)) & 1u));
            kw[u] = *reinterpret_cast<const uint4*>(kp + (size_t)row * row_elems);
            vw[u] = *reinterpret_cast<const uint4*>(vp + (size_t)row * row_elems);
        }
        float s[UNROLL][G];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float kf[N];
            Row16<T>::unpack(kw[u], kf);
#pragma unroll
            for (int col = 0; col < G; ++col) {
                float t = 0.f;
#pragma unroll
                for (int e = 0; e < N; ++e) t = __builtin_fmaf(kf[e], qr[col][e], t);
                t = row_group_sum<LPK>(t);
                s[u][col] = ok[u] ? t * scale_log2e : -INFINITY;
            }
        }
#pragma unroll
        for (int col = 0; col < G; ++col) {
            float m_new = m[col];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) m_new = fmaxf(m_new, s[u][col]);
            const float alpha = __builtin_amdgcn_exp2f(m[col] - m_new);
            m[col] = m_new;
            l[col] *= alpha;
#pragma unroll
            for (int e = 0; e < N; ++e) o[col][e] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float vf[N];
            Row16<T>::unpack(vw[u], vf);
#pragma unroll
            for (int col = 0; col < G; ++col) {
                const float p = __builtin_amdgcn_exp2f(s[u][col] - m[col]);
                l[col] += p;
#pragma unroll
                for (int e = 0; e < N; ++e) o[col][e] = __builtin_fmaf(p, vf[e], o[col][e]);
            }
        }
    }

    // ---- merge the KPW lane groups of the wave (same slice c, different rows) ------------------------------
#pragma unroll
    for (int col = 0; col < G; ++col) {
        float mt = m[col];
        for (int sft = LPK; sft < 64; sft <<= 1) mt = fmaxf(mt, __shfl_xor(mt, sft));
        const float a = __builtin_amdgcn_exp2f(m[col] - mt);
        float lt = l[col] * a;
        for (int sft = LPK; sft < 64; sft <<= 1) lt += __shfl_xor(lt, sft);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            float t = o[col][e] * a;
            for (int sft = LPK; sft < 64; sft <<= 1) t += __shfl_xor(t, sft);
            o[col][e] = t;
        }
        m[col] = mt;
        l[col] = lt;
        if (r == 0) {
            if (c == 0) { merge[wave][col][0] = mt; merge[wave][col][1] = lt; }
#pragma unroll
            for (int e = 0; e < N; ++e) merge[wave][col][2 + c * N + e] = o[col][e];
        }
    }
    __syncthreads();
    // ---- merge the four waves, in wave order; thread t handles element t of the G x D outputs ---------------
    for (int idx = tid; idx < G * D; idx += 256) {
        const int col = idx / D, e = idx % D;
        float mt = NEG_BIG;
#pragma unroll
        for (int w = 0; w < 4; ++w) mt = fmaxf(mt, merge[w][col][0]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = __builtin_amdgcn_exp2f(merge[w][col][0] - mt);
            lt += merge[w][col][1] * a;
            ot += merge[w][col][2 + e] * a;
        }
        float* dst = partials + ((size_t)unit * Hq + g * G + col) * PF;
        if (e == 0) { dst[0] = mt; dst[1] = lt; }
        dst[2 + e] = ot;
    }
}


// bf16, head_dim 128: the logits come from the matrix cores, the value product stays on the vector ALU.
// Per wave and block of 32 key rows:
//   * S^T = K q^T with v_mfma_f32_32x32x16_bf16: the A operand (32 key rows x 16 dims per step) is read straight
//     from memory, 16 bytes per lane (lane = (row x, 8-dim half h)); the B operand holds the G rotated queries in
//     columns 0..G-1 (the other columns are zero);
//   * the G lanes that own a query column (and their partners for the other 4-row groups) run the online softmax
//     and leave the 32 x G weights and the G rescale factors in LDS;
//   * O += P V with the lanes regrouped as (row r of 4, 16-byte slice c of the value row): coalesced value loads,
//     one 16-byte LDS read of the row's G weights, G x 8 multiply-adds.
// Against the all-vector-ALU kernel this removes the dot products, their cross-lane reductions and the 16-fold
// redundant exponentials: about 14 instead of 31 vector instructions per key row and lane.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int G>
__global__ __launch_bounds__(256, 2) void decode_partial_mfma_kernel(
    const __bf16* __restrict__ q, int B, const __bf16* __restrict__ k_shared, const __bf16* __restrict__ v_shared,
    int64_t n_shared, const int32_t* __restrict__ seg_offsets, const int32_t* __restrict__ seg_row0,
    const int32_t* __restrict__ seg_len, const int32_t* __restrict__ seg_delta, int n_seg,
    const uint32_t* __restrict__ stale_bits, int64_t stale_words, const __bf16* __restrict__ k_pages,
    const __bf16* __restrict__ v_pages, int64_t page_stride, const int32_t* __restrict__ page_len, int Hq, int Hkv,
    const float2* __restrict__ rot_table, int rope_layout, float scale_log2e, float* __restrict__ partials) {
    constexpr int D = 128, PF = part_floats<D>();
    constexpr int GP = G < 4 ? 4 : G;                       // weights per row in LDS, padded to a 16-byte read
    __shared__ float merge[4][G][PF];
    __shared__ __attribute__((aligned(16))) float p_lds[4][32][GP];
    __shared__ float alpha_lds[4][GP];
    __shared__ __attribute__((aligned(16))) __bf16 q_rot[G][D];

    const int g = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int x = lane & 31, h = lane >> 5;                 // matrix view: key row (or query column) x, half h
    const int r = lane >> 4, c = lane & 15;                 // value view: row r of a step, 16-byte slice c
    const size_t row_elems = (size_t)Hkv * D;
    Unit<__bf16> un;
    un.resolve(B, k_shared, v_shared, n_shared, seg_offsets, seg_row0, seg_len, seg_delta, n_seg, stale_bits, stale_words,
               k_pages, v_pages, page_stride, page_len, row_elems);
    const int64_t row0 = un.row0, len = un.len;
    const uint32_t* stale = un.stale;

    // ---- the G queries of this KV head, rotated by -delta, rounded to bf16, through LDS into B-operand fragments ----
    for (int idx = tid; idx < G * D; idx += 256) {
        const int col = idx / D, e = idx % D;
        const int pair = (rope_layout == FR_ROPE_INTERLEAVED) ? (e >> 1) : (e % (D / 2));
        const bool first = (rope_layout == FR_ROPE_INTERLEAVED) ? ((e & 1) == 0) : (e < D / 2);
        const int partner = (rope_layout == FR_ROPE_INTERLEAVED) ? (e ^ 1) : ((e + D / 2) % D);
        float2 t = make_float2(1.f, 0.f);
        if (un.delta != 0) t = rot_table[(size_t)un.unit * (D / 2) + pair];
        const __bf16* qp = q + ((size_t)un.b * Hq + g * G + col) * D;
        // RoPE(q, -delta): a' = a cos + b sin, b' = b cos - a sin
        q_rot[col][e] = (__bf16)((float)qp[e] * t.x + (float)qp[partner] * (first ? t.y : -t.y));
    }
    __syncthreads();
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        if (x < G) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(&q_rot[x < G ? x : 0][16 * ks + 8 * h]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[ks][e] = (__bf16)0.0f;
        }
    }

    float m = NEG_BIG, l = 0.f;        // of query column x (lanes x < G; the two halves h keep the same m)
    float o[G][8];                     // value view: this lane's slice of the G output rows, over its key rows
#pragma unroll
    for (int col = 0; col < G; ++col)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[col][e] = 0.f;

    const __bf16* kp = un.kbase + (size_t)g * D + 8 * h;    // + row * row_elems + 16 ks
    const __bf16* vp = un.vbase + (size_t)g * D + 8 * c;    // + row * row_elems
    const int64_t n_blocks = (len + 31) / 32;
    uint4 kw[8], vw[8];
    // which of the 32 rows of block bi count: inside the unit and not stale for this query (bit i = row 32 bi + i)
    auto rows_that_count = [&](int64_t bi) -> uint32_t {
        if (bi >= n_blocks) return 0u;
        const int64_t rowb = row0 + 32 * bi;
        const int64_t left = len - 32 * bi;
        uint32_t okbits = (left >= 32) ? 0xFFFFFFFFu : ((1u << (int)left) - 1u);
        if (stale != nullptr) {
            const int64_t wd = rowb >> 5;
            const int sh = (int)(rowb & 31);
            const uint32_t w0 = (wd < stale_words) ? stale[wd] : 0u;
            const uint32_t w1 = (wd + 1 < stale_words) ? stale[wd + 1] : 0u;
            okbits &= ~(uint32_t)((((uint64_t)w1 << 32) | w0) >> sh);
        }
        return okbits;
    };
    // Rows that do not count (stale for this query, or past the end) are not fetched: their lanes read the unit's
    // first row instead, which stays in the cache, so the skipped rows cost no memory traffic (their logits are masked
    // and their weights are zero).  No branch: the address is chosen, not the load.
    auto load_block = [&](int64_t bi, uint32_t okbits) {
        const int64_t rk = ((okbits >> x) & 1u) ? row0 + 32 * bi + x : row0;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kw[ks] = *reinterpret_cast<const uint4*>(kp + (size_t)rk * row_elems + 16 * ks);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t rv = ((okbits >> (4 * t + r)) & 1u) ? row0 + 32 * bi + 4 * t + r : row0;
            vw[t] = *reinterpret_cast<const uint4*>(vp + (size_t)rv * row_elems);
        }
    };
    // the masks run one block ahead of the loads, the loads one block ahead of the arithmetic
    uint32_t ok_cur = rows_that_count(wave), ok_next = rows_that_count(wave + 4);
    if (wave < n_blocks) load_block(wave, ok_cur);
    for (int64_t bi = wave; bi < n_blocks; bi += 4) {
        // ---- logits of the block's 32 rows -----------------------------------------------------------------
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kw[ks]), qf[ks], s, 0, 0, 0);
        uint4 vcur[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) vcur[t] = vw[t];
        const uint32_t okbits = ok_cur;
        if (bi + 4 < n_blocks) load_block(bi + 4, ok_next);  // the next block of this wave travels during the rest
        ok_cur = ok_next;
        ok_next = rows_that_count(bi + 8);

        // ---- online softmax of column x over the 16 rows this lane holds: 8 (v / 4) + 4 h + v % 4 -----------
        float mx = NEG_BIG;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = 8 * (v >> 2) + 4 * h + (v & 3);
            s[v] = ((okbits >> key) & 1u) ? s[v] * scale_log2e : -INFINITY;
            mx = fmaxf(mx, s[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = __builtin_amdgcn_exp2f(s[v] - m_new);
            psum += p;
            if (x < G) p_lds[wave][8 * (v >> 2) + 4 * h + (v & 3)][x] = p;
        }
        l = l * alpha + psum;
        if (x < G && h == 0) alpha_lds[wave][x] = alpha;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the wave's LDS writes precede its LDS reads below
        __builtin_amdgcn_wave_barrier();

        // ---- O += P V, value view ----------------------------------------------------------------------------
        float al[G];
#pragma unroll
        for (int col = 0; col < G; ++col) al[col] = alpha_lds[wave][col];
#pragma unroll
        for (int col = 0; col < G; ++col)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[col][e] *= al[col];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float vf[8];
            Row16<__bf16>::unpack(vcur[t], vf);
            float pw[GP];
#pragma unroll
            for (int j = 0; j < GP; j += 4) {
                const float4 p4 = *reinterpret_cast<const float4*>(&p_lds[wave][4 * t + r][j]);
                pw[j] = p4.x; pw[j + 1] = p4.y; pw[j + 2] = p4.z; pw[j + 3] = p4.w;
            }
#pragma unroll
            for (int col = 0; col < G; ++col)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[col][e] = __builtin_fmaf(pw[col], vf[e], o[col][e]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // ... and these reads precede the next block's writes
        __builtin_amdgcn_wave_barrier();
    }

    // ---- merge inside the wave, then the four waves in wave order (as in the generic kernel) -----------------
    l += __shfl_xor(l, 32);
    if (x < G && h == 0) { merge[wave][x][0] = m; merge[wave][x][1] = l; }
#pragma unroll
    for (int col = 0; col < G; ++col)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = o[col][e];
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            if (r == 0) merge[wave][col][2 + 8 * c + e] = t;
        }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += 256) {
        const int col = idx / D, e = idx % D;
        float mt = NEG_BIG;
#pragma unroll
        for (int w = 0; w < 4; ++w) mt = fmaxf(mt, merge[w][col][0]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = __builtin_amdgcn_exp2f(merge[w][col][0] - mt);
            lt += merge[w][col][1] * a;
            ot += merge[w][col][2 + e] * a;
        }
        float* dst = partials + ((size_t)un.unit * Hq + g * G + col) * PF;
        if (e == 0) { dst[0] = mt; dst[1] = lt; }
        dst[2 + e] = ot;
    }
}

// rot_table[u][p] = (cos, sin)(seg_delta[u] * theta_p), theta_p = base^(-2 (p + index_base) / d): fp64, rounded once.
__global__ void decode_rot_table_kernel(const int32_t* __restrict__ seg_delta, int half_d, int d, double base,
                                        int index_base, float2* __restrict__ table) {
    const int u = blockIdx.x;
    const double delta = (double)seg_delta[u];
    for (int p = threadIdx.x; p < half_d; p += blockDim.x) {
        const double theta = pow(base, -2.0 * (double)(p + index_base) / (double)d);
        double sn, cs;
        sincos(delta * theta, &sn, &cs);
        table[(size_t)u * half_d + p] = make_float2((float)cs, (float)sn);
    }
}

// One wave per (query, query head): merges the units of the query in a fixed order (its segments, then its page).
template <typename T, int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const float* __restrict__ partials,
                                                            const int32_t* __restrict__ seg_offsets, int n_seg, int Hq,
                                                            T* __restrict__ out, float* __restrict__ lse_out) {
    constexpr int PF = part_floats<D>();
    constexpr int EPT = D / 64;   // elements per lane
    const int b = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    int s0 = seg_offsets[b], s1 = seg_offsets[b + 1];
    s0 = max(0, min(s0, n_seg));
    s1 = max(s0, min(s1, n_seg));
    float mt = NEG_BIG, lt = 0.f, ot[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) ot[e] = 0.f;
    for (int u = s0; u <= s1; ++u) {   // u == s1 stands for the page
        const int unit = (u < s1) ? u : n_seg + b;
        const float* p = partials + ((size_t)unit * Hq + h) * PF;
        const float mu = p[0], lu = p[1];
        const float m_new = fmaxf(mt, mu);
        const float a_old = __builtin_amdgcn_exp2f(mt - m_new), a_new = __builtin_amdgcn_exp2f(mu - m_new);
        lt = lt * a_old + lu * a_new;
#pragma unroll
        for (int e = 0; e < EPT; ++e) ot[e] = ot[e] * a_old + p[2 + lane * EPT + e] * a_new;
        mt = m_new;
    }
    const float inv = 1.0f / lt;
#pragma unroll
    for (int e = 0; e < EPT; ++e) out[((size_t)b * Hq + h) * D + lane * EPT + e] = Elem<T>::from_f32(ot[e] * inv);
    if (lse_out != nullptr && lane == 0) lse_out[(size_t)b * Hq + h] = (mt + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
}

// Sets the bits of the listed store rows in one query's mask (optionally clearing the mask first).
__global__ void mark_stale_kernel(uint32_t* __restrict__ bits, int64_t n_words, const int32_t* __restrict__ rows,
                                  int n_rows) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int64_t row = rows[i];
    if (row < 0 || (row >> 5) >= n_words) return;
    atomicOr(&bits[row >> 5], 1u << (row & 31));
}
__global__ void clear_words_kernel(uint32_t* __restrict__ bits, int64_t n_words) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) bits[i] = 0u;
}

template <typename T, int D, int G>
hipError_t run(const Shape& s, const DecodeArgs& a, float* partials, float2* rot_table, hipStream_t st) {
    const float scale_log2e = (1.0f / sqrtf((float)D)) * 1.4426950408889634f;
    const int units = a.n_seg + a.B;
    if (a.n_seg > 0)
        decode_rot_table_kernel<<<dim3(a.n_seg), dim3(64), 0, st>>>(a.seg_delta, D / 2, D, s.rope_base, s.rope_index_base,
                                                                    rot_table);
    if constexpr (sizeof(T) == 2 && D == 128) {
        if (!a.force_generic) {
            decode_partial_mfma_kernel<G><<<dim3(units, s.Hkv), dim3(256), 0, st>>>(
                (const __bf16*)a.q, a.B, (const __bf16*)a.k_shared, (const __bf16*)a.v_shared, a.n_shared, a.seg_offsets,
                a.seg_row0, a.seg_len, a.seg_delta, a.n_seg, a.stale_bits, a.stale_words, (const __bf16*)a.k_pages,
                (const __bf16*)a.v_pages, a.page_stride, a.page_len, s.Hq, s.Hkv, rot_table, s.rope_layout, scale_log2e,
                partials);
            decode_combine_kernel<T, D><<<dim3(a.B, s.Hq), dim3(64), 0, st>>>(partials, a.seg_offsets, a.n_seg, s.Hq,
                                                                              (T*)a.out, a.lse_out);
            return hipGetLastError();
        }
    }
    decode_partial_kernel<T, D, G><<<dim3(units, s.Hkv), dim3(256), 0, st>>>(
        (const T*)a.q, a.B, (const T*)a.k_shared, (const T*)a.v_shared, a.n_shared, a.seg_offsets, a.seg_row0, a.seg_len,
        a.seg_delta, a.n_seg, a.stale_bits, a.stale_words, (const T*)a.k_pages, (const T*)a.v_pages, a.page_stride,
        a.page_len, s.Hq, s.Hkv, rot_table, s.rope_layout, scale_log2e, partials);
    decode_combine_kernel<T, D><<<dim3(a.B, s.Hq), dim3(64), 0, st>>>(partials, a.seg_offsets, a.n_seg, s.Hq, (T*)a.out,
                                                                      a.lse_out);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t run_g(const Shape& s, const DecodeArgs& a, float* partials, float2* rot_table, hipStream_t st) {
    switch (s.G) {
        case 1: return run<T, D, 1>(s, a, partials, rot_table, st);
        case 2: return run<T, D, 2>(s, a, partials, rot_table, st);
        case 4: return run<T, D, 4>(s, a, partials, rot_table, st);
        case 8: return run<T, D, 8>(s, a, partials, rot_table, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool decode_supported(const Shape& s) { return s.G == 1 || s.G == 2 || s.G == 4 || s.G == 8; }

size_t decode_partials_bytes(const Shape& s) {
    return (size_t)DECODE_MAX_UNITS * s.Hq * (s.d + 2) * sizeof(float);
}

size_t decode_rot_table_bytes(const Shape& s) { return (size_t)DECODE_MAX_UNITS * (s.d / 2) * sizeof(float2); }

hipError_t launch_decode_attn(const Shape& s, const DecodeArgs& a, float* partials, float2* rot_table, hipStream_t st) {
    if (a.B == 0) return hipSuccess;
    if (s.dtype == FR_BF16)
        return s.d == 128 ? run_g<__bf16, 128>(s, a, partials, rot_table, st) : run_g<__bf16, 64>(s, a, partials, rot_table, st);
    return s.d == 128 ? run_g<float, 128>(s, a, partials, rot_table, st) : run_g<float, 64>(s, a, partials, rot_table, st);
}

hipError_t launch_clear_words(uint32_t* words, int64_t n_words, hipStream_t st) {
    if (n_words > 0) clear_words_kernel<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st>>>(words, n_words);
    return hipGetLastError();
}

hipError_t launch_mark_stale(uint32_t* bits, int64_t n_words, const int32_t* rows, int n_rows, int clear, hipStream_t st) {
    if (clear && n_words > 0)
        clear_words_kernel<<<dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, st>>>(bits, n_words);
    if (n_rows > 0) mark_stale_kernel<<<dim3((n_rows + 255) / 256), dim3(256), 0, st>>>(bits, n_words, rows, n_rows);
    return hipGetLastError();
}

}  // namespace fr
