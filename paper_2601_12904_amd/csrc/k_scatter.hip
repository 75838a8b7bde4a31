// Write-back of the recomputed K/V rows (Sec. 4.3): cache[q_index[r]] = new[r], bit-exact.
// Pure data movement: 16-byte vectors, K and V in the same launch.  A call moves 24 MB on the headline layer, so the
// kernel is sized by latency, not by bandwidth: every thread has four independent vectors in flight and the grid holds
// a thread for every four vectors (about 750 workgroups), rather than a few workgroups that loop.
#include "fr_internal.hpp"

namespace fr {

// grid: x = blocks of 1024 vectors, y = 0 (K) / 1 (V).  row_vecs = 16-byte vectors per token row (a power of two
// or not: rows are found by division).
__global__ __launch_bounds__(256) void kv_scatter_kernel(const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
                                                         const int32_t* __restrict__ q_index, int R,
                                                         uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                         int64_t L, int row_vecs) {
    constexpr int U = 4;
    const uint4* src = blockIdx.y ? v_new : k_new;
    uint4* dst = blockIdx.y ? v_cache : k_cache;
    const int64_t n_vec = (int64_t)R * row_vecs;
    const int64_t base = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    uint4 val[U];
    int64_t pos[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {   // all loads first: the four vectors and their rows' positions travel together
        const int64_t i = min(base + 256 * u, n_vec - 1);
        pos[u] = q_index[i / row_vecs];
        val[u] = src[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = base + 256 * u;
        // (an entry outside the cache breaks the caller's contract; its row is dropped rather than written out of bounds)
        if (i < n_vec && pos[u] >= 0 && pos[u] < L) dst[(size_t)pos[u] * row_vecs + (i % row_vecs)] = val[u];
    }
}

hipError_t launch_kv_scatter(const Shape& s, const void* k_new, const void* v_new, const int32_t* q_index,
                             int R, void* k_cache, void* v_cache, int64_t L, hipStream_t st) {
    if (R == 0) return hipSuccess;
    const int row_vecs = s.Hkv * s.d * s.esize / 16;
    const int64_t n_vec = (int64_t)R * row_vecs;
    dim3 grid((unsigned)((n_vec + 1023) / 1024), 2);
    kv_scatter_kernel<<<grid, dim3(256), 0, st>>>((const uint4*)k_new, (const uint4*)v_new, q_index, R,
                                                  (uint4*)k_cache, (uint4*)v_cache, L, row_vecs);
    return hipGetLastError();
}

}  // namespace fr
