// Write-back of the recomputed K/V rows (Sec. 4.3): cache[q_index[r]] = new[r], bit-exact.
// Pure data movement: 16-byte vectors, one block per few rows, K and V in the same launch.
#include "fr_internal.hpp"

namespace fr {

// grid: x = row tiles, y = 0 (K) / 1 (V).  row_vecs = 16-byte vectors per token row.
__global__ __launch_bounds__(256) void kv_scatter_kernel(const uint4* __restrict__ k_new,
                                                         const uint4* __restrict__ v_new,
                                                         const int32_t* __restrict__ q_index, int R,
                                                         uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                         int64_t L, int row_vecs, int rows_per_block) {
    const uint4* src = blockIdx.y ? v_new : k_new;
    uint4* dst = blockIdx.y ? v_cache : k_cache;
    const int r0 = blockIdx.x * rows_per_block;
    const int nrows = min(rows_per_block, R - r0);
    const int nvec = nrows * row_vecs;
    for (int i = threadIdx.x; i < nvec; i += 256) {
        const int r = r0 + i / row_vecs;
        const int v = i % row_vecs;
        const int64_t pos = q_index[r];
        // (an entry outside the cache breaks the caller's contract; its row is dropped rather than written out of bounds)
        if (pos >= 0 && pos < L) dst[(size_t)pos * row_vecs + v] = src[(size_t)r * row_vecs + v];
    }
}

hipError_t launch_kv_scatter(const Shape& s, const void* k_new, const void* v_new, const int32_t* q_index,
                             int R, void* k_cache, void* v_cache, int64_t L, hipStream_t st) {
    if (R == 0) return hipSuccess;
    const int row_vecs = s.Hkv * s.d * s.esize / 16;
    // about 2048 vectors (32 KB) per block
    int rows_per_block = 2048 / row_vecs;
    if (rows_per_block < 1) rows_per_block = 1;
    dim3 grid((R + rows_per_block - 1) / rows_per_block, 2);
    kv_scatter_kernel<<<grid, dim3(256), 0, st>>>((const uint4*)k_new, (const uint4*)v_new, q_index, R,
                                                  (uint4*)k_cache, (uint4*)v_cache, L, row_vecs, rows_per_block);
    return hipGetLastError();
}

}  // namespace fr
