// Position recovery of cached chunk keys (Sec. 2.2.1 footnote, Appendix A): every key of chunk c is
// rotated by Delta_c positions.  HBM-bound streaming: one 16-byte load and one 16-byte store per
// lane per step; the chunk's cos/sin row is built once in fp64 and kept in LDS.
#include "fr_internal.hpp"

namespace fr {

// table[c][p] = (cos, sin)(Delta_c * theta_p), theta_p = base^(-2 (p + index_base) / d), in fp64,
// rounded once to fp32.  Delta reaches tens of thousands of positions, so the angle is formed and
// reduced in double precision.
__global__ void rope_table_kernel(ChunkDeltas deltas, int half_d, int d, double base, int index_base,
                                  float2* __restrict__ table) {
    const int c = blockIdx.x;
    for (int p = threadIdx.x; p < half_d; p += blockDim.x) {
        const double theta = pow(base, -2.0 * (double)(p + index_base) / (double)d);
        const double ang = (double)deltas.delta[c] * theta;
        double sn, cs;
        sincos(ang, &sn, &cs);
        table[(size_t)c * half_d + p] = make_float2((float)cs, (float)sn);
    }
}

template <typename T>
struct Vec16 {
    static constexpr int N = 16 / sizeof(T);
    T v[N];
};

// grid: x = token tiles inside a chunk, y = chunk, z = batch.  TOK tokens per block.
template <typename T, int LAYOUT, int TOK>
__global__ __launch_bounds__(256) void rope_shift_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                         ChunkTable ct, const float2* __restrict__ table,
                                                         int Hkv, int d, int64_t src_stride,
                                                         int64_t dst_stride, ChunkRows src_rows, int from_store) {
    constexpr int N = 16 / sizeof(T);  // elements per 16-byte vector
    __shared__ float2 cs[64];          // d/2 <= 64 (cos, sin) pairs of this chunk
    const int c = blockIdx.y;
    const int c0 = ct.off[c], c1 = ct.off[c + 1];
    const int tok0 = c0 + blockIdx.x * TOK;
    if (tok0 >= c1) return;
    const int half_d = d >> 1;
    if (threadIdx.x < half_d) cs[threadIdx.x] = table[(size_t)c * half_d + threadIdx.x];
    __syncthreads();

    const int ntok = min(TOK, c1 - tok0);
    const size_t row = (size_t)Hkv * d;  // elements per token
    // source row of the block's first token: its prompt position, or its row in a chunk store
    const size_t src_tok0 = from_store ? (size_t)src_rows.row0[c] + (size_t)(tok0 - c0) : (size_t)tok0;
    const T* s = src + (size_t)blockIdx.z * src_stride + src_tok0 * row;
    T* o = dst + (size_t)blockIdx.z * dst_stride + (size_t)tok0 * row;

    if (LAYOUT == FR_ROPE_INTERLEAVED) {
        const int vec_per_head = d / N;
        const int nvec = ntok * Hkv * vec_per_head;
        // vec_per_head divides 256 (d is 64 or 128), so a thread meets the same slice of the head row in every step:
        // its (cos, sin) values stay in registers
        const int p0 = (threadIdx.x % vec_per_head) * (N / 2);  // first rotary pair of this thread's vectors
        float2 tw[N / 2];
#pragma unroll
        for (int e = 0; e < N / 2; ++e) tw[e] = cs[p0 + e];
#pragma unroll 8
        for (int i = threadIdx.x; i < nvec; i += 256) {
            Vec16<T> x = *reinterpret_cast<const Vec16<T>*>(s + (size_t)i * N);
            Vec16<T> y;
#pragma unroll
            for (int e = 0; e < N / 2; ++e) {
                const float2 t = tw[e];
                const float a = Elem<T>::to_f32(x.v[2 * e]), b = Elem<T>::to_f32(x.v[2 * e + 1]);
                y.v[2 * e] = Elem<T>::from_f32(a * t.x - b * t.y);
                y.v[2 * e + 1] = Elem<T>::from_f32(b * t.x + a * t.y);
            }
            *reinterpret_cast<Vec16<T>*>(o + (size_t)i * N) = y;
        }
    } else {  // pairs (p, p + d/2): one lane moves the low and the high vector of a head together
        const int vec_per_half = half_d / N;
        const int nvec = ntok * Hkv * vec_per_half;
#pragma unroll 2
        for (int i = threadIdx.x; i < nvec; i += 256) {
            const int head_row = i / vec_per_half;  // (token, head) row
            const int p0 = (i % vec_per_half) * N;
            const size_t lo = (size_t)head_row * d + p0, hi = lo + half_d;
            Vec16<T> xa = *reinterpret_cast<const Vec16<T>*>(s + lo);
            Vec16<T> xb = *reinterpret_cast<const Vec16<T>*>(s + hi);
            Vec16<T> ya, yb;
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const float2 t = cs[p0 + e];
                const float a = Elem<T>::to_f32(xa.v[e]), b = Elem<T>::to_f32(xb.v[e]);
                ya.v[e] = Elem<T>::from_f32(a * t.x - b * t.y);
                yb.v[e] = Elem<T>::from_f32(b * t.x + a * t.y);
            }
            *reinterpret_cast<Vec16<T>*>(o + lo) = ya;
            *reinterpret_cast<Vec16<T>*>(o + hi) = yb;
        }
    }
}

hipError_t launch_rope_table(const Shape& s, const ChunkDeltas& deltas, int n_chunks, float2* table,
                             hipStream_t st) {
    if (n_chunks == 0) return hipSuccess;
    rope_table_kernel<<<dim3(n_chunks), dim3(64), 0, st>>>(deltas, s.d / 2, s.d, s.rope_base,
                                                            s.rope_index_base, table);
    return hipGetLastError();
}

hipError_t launch_rope_shift(const Shape& s, const void* src, void* dst, const ChunkTable& ct,
                             int max_chunk_len, const float2* table, int n_batch, int64_t src_stride,
                             int64_t dst_stride, const ChunkRows* src_rows, hipStream_t st) {
    if (ct.n == 0 || max_chunk_len == 0 || n_batch == 0) return hipSuccess;
    const ChunkRows none{};
    const ChunkRows& rows = src_rows ? *src_rows : none;
    const int from_store = src_rows ? 1 : 0;
    constexpr int TOK = 32;
    dim3 grid((max_chunk_len + TOK - 1) / TOK, ct.n, n_batch);
#define FR_ROPE_LAUNCH(T, LAY)                                                                      \
    rope_shift_kernel<T, LAY, TOK><<<grid, dim3(256), 0, st>>>((const T*)src, (T*)dst, ct, table, \
                                                               s.Hkv, s.d, src_stride, dst_stride, rows, from_store)
    if (s.dtype == FR_BF16) {
        if (s.rope_layout == FR_ROPE_INTERLEAVED)
            FR_ROPE_LAUNCH(__bf16, FR_ROPE_INTERLEAVED);
        else
            FR_ROPE_LAUNCH(__bf16, FR_ROPE_HALF);
    } else {
        if (s.rope_layout == FR_ROPE_INTERLEAVED)
            FR_ROPE_LAUNCH(float, FR_ROPE_INTERLEAVED);
        else
            FR_ROPE_LAUNCH(float, FR_ROPE_HALF);
    }
#undef FR_ROPE_LAUNCH
    return hipGetLastError();
}

}  // namespace fr
