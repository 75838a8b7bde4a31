// Query-Guided Selection, critical scores (Sec. 3.2) -- generic kernels for any supported shape
// and both storage types.  Two passes over the logits, as the definition needs: the normaliser
// of every (question token, head, scope) first, then the column sums of the normalised weights.
// Every sum runs in a fixed order, so the scores are reproducible bit for bit.
#include "fr_internal.hpp"

namespace fr {

template <typename T>
__device__ __forceinline__ float dot_row(const T* __restrict__ a, const T* __restrict__ b, int d) {
    float acc = 0.f;
    for (int t = 0; t < d; t += 4) {
        acc += Elem<T>::to_f32(a[t]) * Elem<T>::to_f32(b[t]);
        acc += Elem<T>::to_f32(a[t + 1]) * Elem<T>::to_f32(b[t + 1]);
        acc += Elem<T>::to_f32(a[t + 2]) * Elem<T>::to_f32(b[t + 2]);
        acc += Elem<T>::to_f32(a[t + 3]) * Elem<T>::to_f32(b[t + 3]);
    }
    return acc;
}

// Pass A.  grid (nq, Hq, n_chunks), one wave each: lse[(h * (C + 1) + c) * nq + i] = natural
// log-sum-exp of the scaled logits of question row (i, h) over the keys of chunk c.
template <typename T>
__global__ __launch_bounds__(64) void score_lse_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                       ChunkTable ct, int nq, int Hq, int Hkv, int d,
                                                       float scale, float* __restrict__ lse) {
    const int i = blockIdx.x, h = blockIdx.y, c = blockIdx.z;
    const int g = h / (Hq / Hkv);
    const int lane = threadIdx.x;
    const T* qv = q + ((size_t)i * Hq + h) * d;
    float m = -INFINITY, l = 0.f;
    for (int j = ct.off[c] + lane; j < ct.off[c + 1]; j += 64) {
        const float s = dot_row(qv, k + ((size_t)j * Hkv + g) * d, d) * scale;
        const float mn = fmaxf(m, s);
        l = l * expf(m - mn) + expf(s - mn);
        m = mn;
    }
    for (int o = 32; o > 0; o >>= 1) {
        const float m2 = __shfl_xor(m, o), l2 = __shfl_xor(l, o);
        const float mn = fmaxf(m, m2);
        const float a = (m == -INFINITY) ? 0.f : l * expf(m - mn);
        const float b = (m2 == -INFINITY) ? 0.f : l2 * expf(m2 - mn);
        l = a + b;
        m = mn;
    }
    if (lane == 0) lse[((size_t)h * (ct.n + 1) + c) * nq + i] = (l > 0.f) ? m + logf(l) : -INFINITY;
}

// Global scope: lse[h][C][i] = log-sum-exp over the chunk values.  grid (ceil(nq/256), Hq).
__global__ void score_lse_global_kernel(int n_chunks, int nq, float* __restrict__ lse) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int h = blockIdx.y;
    if (i >= nq) return;
    float* base = lse + (size_t)h * (n_chunks + 1) * nq;
    float m = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) m = fmaxf(m, base[(size_t)c * nq + i]);
    float l = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float v = base[(size_t)c * nq + i];
        if (v != -INFINITY) l += expf(v - m);
    }
    base[(size_t)n_chunks * nq + i] = m + logf(l);
}

// Pass B.  One thread per context key j: score[j] = sum_h sum_i w(h, i, j), heads outer, question
// tokens inner, sequentially.  norm: 0 per chunk, 1 global, 2 raw.
template <typename T>
__global__ __launch_bounds__(64) void score_colsum_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                          ChunkTable ct, int nq, int Hq, int Hkv, int d,
                                                          float scale, int norm, const float* __restrict__ lse,
                                                          float* __restrict__ scores) {
    const int L_ctx = ct.off[ct.n];
    const int j = blockIdx.x * 64 + threadIdx.x;
    if (j >= L_ctx) return;
    int c = 0;
    if (norm == FR_NORM_GLOBAL) {
        c = ct.n;
    } else if (norm == FR_NORM_PER_CHUNK) {
        int lo = 0, hi = ct.n - 1;  // last chunk whose offset is <= j (empty chunks are skipped)
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (ct.off[mid] <= j) lo = mid; else hi = mid - 1;
        }
        c = lo;
    }
    const int G = Hq / Hkv;
    float total = 0.f;
    for (int h = 0; h < Hq; ++h) {
        const T* kv = k + ((size_t)j * Hkv + h / G) * d;
        const float* lrow = lse + ((size_t)h * (ct.n + 1) + c) * nq;
        float acc = 0.f;
        for (int i = 0; i < nq; ++i) {
            const float s = dot_row(q + ((size_t)i * Hq + h) * d, kv, d) * scale;
            acc += (norm == FR_NORM_RAW) ? s : expf(s - lrow[i]);
        }
        total += acc;
    }
    scores[j] = total;
}

template <typename T>
static hipError_t run(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct, int norm,
                      const Workspace& ws, float* scores, hipStream_t st) {
    const int L_ctx = ct.off[ct.n];
    if (L_ctx == 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)s.d);
    if (norm != FR_NORM_RAW && nq > 0) {
        score_lse_kernel<T><<<dim3(nq, s.Hq, ct.n), dim3(64), 0, st>>>((const T*)q, (const T*)k_ctx, ct, nq, s.Hq,
                                                                      s.Hkv, s.d, scale, ws.lse);
        if (norm == FR_NORM_GLOBAL)
            score_lse_global_kernel<<<dim3((nq + 255) / 256, s.Hq), dim3(256), 0, st>>>(ct.n, nq, ws.lse);
    }
    score_colsum_kernel<T><<<dim3((L_ctx + 63) / 64), dim3(64), 0, st>>>((const T*)q, (const T*)k_ctx, ct, nq, s.Hq,
                                                                       s.Hkv, s.d, scale, norm, ws.lse, scores);
    return hipGetLastError();
}

hipError_t launch_score_simt(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct,
                             int norm, const Workspace& ws, float* scores, hipStream_t st) {
    return s.dtype == FR_BF16 ? run<__bf16>(s, q, nq, k_ctx, ct, norm, ws, scores, st)
                              : run<float>(s, q, nq, k_ctx, ct, norm, ws, scores, st);
}

}  // namespace fr
