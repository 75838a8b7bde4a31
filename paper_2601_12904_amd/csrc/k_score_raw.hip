// Critical scores without the softmax (FR_NORM_RAW, the literal product of Sec. 3.2): the score of key j is
// sum over question tokens i and query heads h of q[i, h] . k[j, g(h)] / sqrt(d).  The sum over i and over the
// heads of a group commutes with the dot product, so the question is first reduced to one vector per KV head
// (qsum[g] = sum_i sum_{h in g} q[i, h]), after which every key row is read exactly once: a matrix-vector product
// that streams K from HBM (1 flop per byte) -- the HBM-bound special case of the scoring step.
// Fixed summation orders everywhere: results are reproducible bit for bit.
#include "fr_internal.hpp"

namespace fr {

namespace {

template <typename T>
struct Load16;
template <>
struct Load16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& w, float (&f)[4]) {
        f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y); f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
    }
};
template <>
struct Load16<__bf16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& w, float (&f)[8]) {
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(u[e] << 16);
            f[2 * e + 1] = __uint_as_float(u[e] & 0xFFFF0000u);
        }
    }
};

// qsum[g * d + e] = sum over question tokens of the sum over the G heads of group g, in two fixed-order stages:
// slice y of the tokens -> part[y][g * d + e] (one thread per (g, e), rows read coalesced along e), then the
// QSUM_SLICES partial sums in slice order.
constexpr int QSUM_SLICES = 128;   // a few question tokens per thread: the loads of a slice are all in flight at once

template <typename T>
__global__ __launch_bounds__(256) void question_sum_kernel(const T* __restrict__ q, int nq, int Hq, int G, int d,
                                                           float* __restrict__ part) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int Hkv = Hq / G;
    if (idx >= Hkv * d) return;
    const int g = idx / d, e = idx % d;
    const int per = (nq + QSUM_SLICES - 1) / QSUM_SLICES;
    const int i0 = blockIdx.y * per, i1 = min(nq, i0 + per);
    float acc = 0.f;
#pragma unroll 4
    for (int i = i0; i < i1; ++i) {
        float t = 0.f;
#pragma unroll 4
        for (int hh = 0; hh < G; ++hh) t += Elem<T>::to_f32(q[((size_t)i * Hq + g * G + hh) * d + e]);
        acc += t;
    }
    part[(size_t)blockIdx.y * Hkv * d + idx] = acc;
}

__global__ __launch_bounds__(256) void question_sum_finish_kernel(const float* __restrict__ part, int n,
                                                                  float* __restrict__ qsum) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    float acc = 0.f;
    for (int y = 0; y < QSUM_SLICES; ++y) acc += part[(size_t)y * n + idx];
    qsum[idx] = acc;
}

constexpr int ROWS_IN_FLIGHT = 4;
constexpr int MAX_VECS_PER_LANE = 4;   // row bytes <= 64 lanes x 4 x 16 B = 4 KB

// One wave per key row at a time, four rows in flight; lane l owns the 16-byte vectors l, l + 64, ... of the row
// and keeps the matching slice of qsum in registers.
template <typename T>
__global__ __launch_bounds__(256) void score_raw_kernel(const uint4* __restrict__ k, const float* __restrict__ qsum,
                                                        int64_t n_tokens, int row_vecs, float scale,
                                                        float* __restrict__ scores) {
    constexpr int N = Load16<T>::N;
    const int lane = threadIdx.x & 63;
    float w[MAX_VECS_PER_LANE][N];
#pragma unroll
    for (int j = 0; j < MAX_VECS_PER_LANE; ++j)
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const int v = lane + 64 * j;
            w[j][e] = (v < row_vecs) ? qsum[v * N + e] : 0.f;
        }
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    for (int64_t r0 = wave * ROWS_IN_FLIGHT; r0 < n_tokens; r0 += n_waves * ROWS_IN_FLIGHT) {
        float acc[ROWS_IN_FLIGHT];
#pragma unroll
        for (int i = 0; i < ROWS_IN_FLIGHT; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < MAX_VECS_PER_LANE; ++j) {
            const int v = lane + 64 * j;
            if (64 * j >= row_vecs) break;   // uniform
            uint4 kv[ROWS_IN_FLIGHT];
#pragma unroll
            for (int i = 0; i < ROWS_IN_FLIGHT; ++i) {   // rows past the end re-read the last row and are not stored
                const int64_t r = min(r0 + i, n_tokens - 1);
                kv[i] = k[r * row_vecs + min(v, row_vecs - 1)];
            }
#pragma unroll
            for (int i = 0; i < ROWS_IN_FLIGHT; ++i) {
                float f[N];
                Load16<T>::unpack(kv[i], f);
#pragma unroll
                for (int e = 0; e < N; ++e) acc[i] = __builtin_fmaf(f[e], w[j][e], acc[i]);   // w is 0 for v >= row_vecs
            }
        }
#pragma unroll
        for (int i = 0; i < ROWS_IN_FLIGHT; ++i) {
            float t = acc[i];
            for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o);
            if (lane == 0 && r0 + i < n_tokens) scores[r0 + i] = t * scale;
        }
    }
}

}  // namespace

bool score_raw_supported(const Shape& s) { return s.Hkv * s.d * s.esize <= 64 * MAX_VECS_PER_LANE * 16; }

size_t score_raw_workspace_bytes(const Shape& s) { return (size_t)(1 + QSUM_SLICES) * s.Hkv * s.d * sizeof(float); }

// qsum: score_raw_workspace_bytes() of workspace (the sums, then the partial sums).
hipError_t launch_score_raw(const Shape& s, const void* q, int nq, const void* k_ctx, int64_t L_ctx, float* qsum,
                            float* scores, hipStream_t st) {
    if (L_ctx == 0) return hipSuccess;
    const int row_vecs = s.Hkv * s.d * s.esize / 16;
    const float scale = 1.0f / sqrtf((float)s.d);
    const int64_t groups = (L_ctx + ROWS_IN_FLIGHT - 1) / ROWS_IN_FLIGHT;
    int64_t blocks = (groups + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;
    const int n = s.Hkv * s.d;
    float* part = qsum + n;
    const dim3 qgrid((n + 255) / 256, QSUM_SLICES);
    if (s.dtype == FR_BF16) {
        question_sum_kernel<__bf16><<<qgrid, dim3(256), 0, st>>>((const __bf16*)q, nq, s.Hq, s.G, s.d, part);
        question_sum_finish_kernel<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(part, n, qsum);
        score_raw_kernel<__bf16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((const uint4*)k_ctx, qsum, L_ctx, row_vecs, scale, scores);
    } else {
        question_sum_kernel<float><<<qgrid, dim3(256), 0, st>>>((const float*)q, nq, s.Hq, s.G, s.d, part);
        question_sum_finish_kernel<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(part, n, qsum);
        score_raw_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((const uint4*)k_ctx, qsum, L_ctx, row_vecs, scale, scores);
    }
    return hipGetLastError();
}

}  // namespace fr
