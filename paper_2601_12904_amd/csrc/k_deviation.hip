// KV deviation of one layer (eq. 7): per token, the sum over all head components of the squared
// difference between two versions of a K (or V) tensor.  With the top-k of fr_select_topk it is the
// CacheBlend selector (eq. 8), the comparison selector of Sec. 2.2.2.
//
// Pure streaming: both tensors are read once, 16 bytes per lane and load.  One wave owns a token row at a
// time (4 rows in flight); every lane adds its elements in index order and the 64 partial sums are combined
// by a fixed butterfly, so the result is reproducible bit for bit.
#include "fr_internal.hpp"

namespace fr {

namespace {

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ float sqdiff(const uint4& a, const uint4& b, float acc) {
        const float af[4] = {__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w)};
        const float bf[4] = {__uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float t = af[e] - bf[e];
            acc = __builtin_fmaf(t, t, acc);
        }
        return acc;
    }
};
template <>
struct Vec16<__bf16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ float sqdiff(const uint4& a, const uint4& b, float acc) {
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {   // a bf16 is the upper half of an fp32
            const float t0 = __uint_as_float(aw[e] << 16) - __uint_as_float(bw[e] << 16);
            acc = __builtin_fmaf(t0, t0, acc);
            const float t1 = __uint_as_float(aw[e] & 0xFFFF0000u) - __uint_as_float(bw[e] & 0xFFFF0000u);
            acc = __builtin_fmaf(t1, t1, acc);
        }
        return acc;
    }
};

constexpr int ROWS_IN_FLIGHT = 4;

// row_vecs = 16-byte vectors per token row.  Wave w of the grid takes rows w * ROWS_IN_FLIGHT + ..., stride = all waves.
template <typename T>
__global__ __launch_bounds__(256) void kv_deviation_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                           int64_t n_tokens, int row_vecs, float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    for (int64_t r0 = wave * ROWS_IN_FLIGHT; r0 < n_tokens; r0 += n_waves * ROWS_IN_FLIGHT) {
        float acc[ROWS_IN_FLIGHT];
#pragma unroll
        for (int i = 0; i < ROWS_IN_FLIGHT; ++i) acc[i] = 0.f;
        for (int v = lane; v < row_vecs; v += 64) {
            uint4 av[ROWS_IN_FLIGHT], bv[ROWS_IN_FLIGHT];
#pragma unroll
            for (int i = 0; i < ROWS_IN_FLIGHT; ++i) {   // rows past the end re-read the last row and are not stored
                const int64_t r = min(r0 + i, n_tokens - 1);
                av[i] = a[r * row_vecs + v];
                bv[i] = b[r * row_vecs + v];
            }
#pragma unroll
            for (int i = 0; i < ROWS_IN_FLIGHT; ++i) acc[i] = Vec16<T>::sqdiff(av[i], bv[i], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < ROWS_IN_FLIGHT; ++i) {
            float t = acc[i];
            for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
            if (lane == 0 && r0 + i < n_tokens) out[r0 + i] = t;
        }
    }
}

}  // namespace

hipError_t launch_kv_deviation(const Shape& s, const void* kv_a, const void* kv_b, int64_t n_tokens, float* out,
                               hipStream_t st) {
    if (n_tokens == 0) return hipSuccess;
    const int row_vecs = s.Hkv * s.d * s.esize / 16;
    const int64_t row_groups = (n_tokens + ROWS_IN_FLIGHT - 1) / ROWS_IN_FLIGHT;
    int64_t blocks = (row_groups + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;   // 8 workgroups per CU, grid-stride beyond that
    if (s.dtype == FR_BF16)
        kv_deviation_kernel<__bf16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((const uint4*)kv_a, (const uint4*)kv_b,
                                                                                  n_tokens, row_vecs, out);
    else
        kv_deviation_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((const uint4*)kv_a, (const uint4*)kv_b,
                                                                                 n_tokens, row_vecs, out);
    return hipGetLastError();
}

}  // namespace fr
