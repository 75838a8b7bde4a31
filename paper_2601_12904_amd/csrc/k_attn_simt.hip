// Sparse prefill attention (eq. 9, Sec. 4.3) -- generic kernel for any supported shape and both
// storage types: one wave per (row, query head); lanes stride over the visible keys with a
// running softmax each and are merged at the end.  The tiled matrix-core kernel serves the
// Llama-shaped bf16 case; this one serves everything else (fp32 in particular).
#include "fr_internal.hpp"

namespace fr {

// inv[j] = row r of k_new/v_new that holds the recomputed entry of position j (q_index[r] == j), else -1.  The Q index is strictly ascending, so every position finds its own
// answer by a binary search (one launch, no fill-then-set ordering).
__global__ void inv_index_kernel(const int32_t* __restrict__ q_index, int R, int64_t L, int32_t* __restrict__ inv) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= L) return;
    int lo = 0, hi = R;   // first r with q_index[r] >= j
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (q_index[mid] < j) lo = mid + 1; else hi = mid;
    }
    inv[j] = (lo < R && q_index[lo] == j) ? lo : -1;
}

hipError_t launch_inv_index(const int32_t* q_index, int R, int64_t L, int32_t* inv, hipStream_t st) {
    if (L > 0) inv_index_kernel<<<dim3((unsigned)((L + 255) / 256)), dim3(256), 0, st>>>(q_index, R, L, inv);
    return hipGetLastError();
}

template <typename T, int D>
__global__ __launch_bounds__(64) void attn_simt_kernel(const T* __restrict__ q_rows, const int32_t* __restrict__ q_index,
                                                       const T* __restrict__ k_cache, const T* __restrict__ v_cache,
                                                       const T* __restrict__ k_new, const T* __restrict__ v_new,
                                                       const int32_t* __restrict__ inv, T* __restrict__ out,
                                                       float* __restrict__ lse, int Hq, int Hkv, float scale) {
    constexpr int N = 16 / sizeof(T);
    struct alignas(16) V16 { T v[N]; };
    const int r = blockIdx.x, h = blockIdx.y;
    const int g = h / (Hq / Hkv);
    const int lane = threadIdx.x;
    const int p = q_index[r];

    float qv[D];
    {
        const T* qp = q_rows + ((size_t)r * Hq + h) * D;
#pragma unroll
        for (int t = 0; t < D; t += N) {
            const V16 x = *reinterpret_cast<const V16*>(qp + t);
#pragma unroll
            for (int e = 0; e < N; ++e) qv[t + e] = Elem<T>::to_f32(x.v[e]);
        }
    }
    float acc[D];
#pragma unroll
    for (int t = 0; t < D; ++t) acc[t] = 0.f;
    float m = -INFINITY, l = 0.f;

    for (int j = lane; j <= p; j += 64) {
        const int row = (k_new != nullptr) ? inv[j] : -1;
        const T* kp = (row >= 0) ? k_new + ((size_t)row * Hkv + g) * D : k_cache + ((size_t)j * Hkv + g) * D;
        const T* vp = (row >= 0) ? v_new + ((size_t)row * Hkv + g) * D : v_cache + ((size_t)j * Hkv + g) * D;
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < D; t += N) {
            const V16 x = *reinterpret_cast<const V16*>(kp + t);
#pragma unroll
            for (int e = 0; e < N; ++e) s += qv[t + e] * Elem<T>::to_f32(x.v[e]);
        }
        s *= scale;
        const float mn = fmaxf(m, s);
        const float a = expf(m - mn);  // m = -inf on the first key: exp(-inf) = 0
        const float w = expf(s - mn);
        l = l * a + w;
#pragma unroll
        for (int t = 0; t < D; t += N) {
            const V16 x = *reinterpret_cast<const V16*>(vp + t);
#pragma unroll
            for (int e = 0; e < N; ++e) acc[t + e] = acc[t + e] * a + w * Elem<T>::to_f32(x.v[e]);
        }
        m = mn;
    }

    // merge the 64 lanes
    float M = m;
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float f = (m == -INFINITY) ? 0.f : expf(m - M);
    float lt = l * f;
    for (int o = 32; o > 0; o >>= 1) lt += __shfl_xor(lt, o);
    const float inv_l = 1.0f / lt;
    T* op = out + ((size_t)r * Hq + h) * D;
#pragma unroll
    for (int t = 0; t < D; ++t) {
        float v = acc[t] * f;
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == (t & 63)) op[t] = Elem<T>::from_f32(v * inv_l);
    }
    if (lse != nullptr && lane == 0) lse[(size_t)r * Hq + h] = M + logf(lt);
}

hipError_t launch_attn_simt(const Shape& s, const void* q_rows, const int32_t* q_index, int R, const void* k_cache,
                            const void* v_cache, int64_t L, const void* k_new, const void* v_new, const int32_t* inv,
                            void* out, float* lse, hipStream_t st) {
    (void)L;
    if (R == 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)s.d);
    dim3 grid(R, s.Hq), block(64);
#define FR_ATTN_LAUNCH(T, D)                                                                                   \
    attn_simt_kernel<T, D><<<grid, block, 0, st>>>((const T*)q_rows, q_index, (const T*)k_cache, (const T*)v_cache, \
                                                   (const T*)k_new, (const T*)v_new, inv, (T*)out, lse, s.Hq, s.Hkv, scale)
    if (s.dtype == FR_BF16) {
        if (s.d == 64) FR_ATTN_LAUNCH(__bf16, 64); else FR_ATTN_LAUNCH(__bf16, 128);
    } else {
        if (s.d == 64) FR_ATTN_LAUNCH(float, 64); else FR_ATTN_LAUNCH(float, 128);
    }
#undef FR_ATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace fr
