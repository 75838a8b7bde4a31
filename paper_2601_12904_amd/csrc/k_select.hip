// Selection half of Query-Guided Selection: argTopk of the critical scores (Table 1, Sec. 3.2)
// and the Q index of Sec. 4.3 (ascending critical tokens, then the question tokens).
//
// Integer work only.  Scores are mapped to order-preserving 32-bit keys; a most-significant-digit
// radix select (4 passes of 8 bits, LDS histograms) finds the key of the k-th largest score; an
// ordered compaction then emits, in index order, every token above that key plus the first
// (lowest-index) tokens equal to it that are still needed.  The result is unique, so it does not
// depend on scheduling.
#include "fr_internal.hpp"

namespace fr {

__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger score <=> larger key
}

constexpr int SEL_THREADS = 1024;

// exclusive prefix sum of one value per thread over the block; *total = block sum
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    if (wave == 0) {
        uint32_t w = (lane < SEL_THREADS / 64) ? wave_sums[lane] : 0u;
        uint32_t winc = w;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_up(winc, o);
            if (lane >= o) winc += t;
        }
        if (lane < SEL_THREADS / 64) wave_sums[lane] = winc - w;  // exclusive wave offsets
        if (lane == SEL_THREADS / 64 - 1) wave_sums[SEL_THREADS / 64] = winc;
    }
    __syncthreads();
    const uint32_t res = wave_sums[wave] + inc - v;
    *total = wave_sums[SEL_THREADS / 64];
    __syncthreads();
    return res;
}

__global__ __launch_bounds__(SEL_THREADS) void select_topk_kernel(const float* __restrict__ scores, int64_t n,
                                                                  int64_t k, int nq, int32_t* __restrict__ out) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_sums[SEL_THREADS / 64 + 1];
    __shared__ uint32_t s_prefix, s_remaining;
    const int tid = threadIdx.x;

    // question tokens: positions n .. n + nq - 1
    for (int i = tid; i < nq; i += SEL_THREADS) out[k + i] = (int32_t)(n + i);
    if (k <= 0 || n <= 0) return;

    uint32_t thr_key = 0u;     // key of the k-th largest score
    uint32_t need_eq = 0u;     // how many tokens equal to it are taken
    if (k < n) {
        if (tid == 0) { s_prefix = 0u; s_remaining = (uint32_t)k; }
        uint32_t mask = 0u;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            for (int64_t i = tid; i < n; i += SEL_THREADS) {
                const uint32_t key = score_key(scores[i]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t remaining = s_remaining, cum = 0u;
                int dg = 255;
                for (; dg > 0; --dg) {
                    if (cum + hist[dg] >= remaining) break;
                    cum += hist[dg];
                }
                s_remaining = remaining - cum;  // still to take among keys with this digit
                s_prefix = prefix | ((uint32_t)dg << shift);
            }
            mask |= 0xFFu << shift;
            __syncthreads();
        }
        thr_key = s_prefix;
        need_eq = s_remaining;
    } else {
        thr_key = 0u;  // every key is >= 0x00000000: take everything
        need_eq = 0u;
    }

    // ordered compaction: thread t owns the contiguous index range [lo, hi)
    const int64_t per = (n + SEL_THREADS - 1) / SEL_THREADS;
    const int64_t lo = min(n, (int64_t)tid * per), hi = min(n, lo + per);
    uint32_t cnt_gt = 0u, cnt_eq = 0u;
    const bool take_all = (k >= n);
    for (int64_t i = lo; i < hi; ++i) {
        const uint32_t key = score_key(scores[i]);
        cnt_gt += (take_all || key > thr_key) ? 1u : 0u;
        cnt_eq += (!take_all && key == thr_key) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t eq_before = block_exclusive_scan(cnt_eq, wave_sums, &total);
    uint32_t eq_take = 0u;
    if (need_eq > eq_before) eq_take = min(cnt_eq, need_eq - eq_before);
    const uint32_t out_before = block_exclusive_scan(cnt_gt + eq_take, wave_sums, &total);
    uint32_t pos = out_before, eq_left = eq_take;
    for (int64_t i = lo; i < hi; ++i) {
        const uint32_t key = score_key(scores[i]);
        bool sel = take_all || key > thr_key;
        if (!take_all && key == thr_key && eq_left > 0u) { sel = true; --eq_left; }
        if (sel) out[pos++] = (int32_t)i;
    }
}

hipError_t launch_select(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* tmp,
                         hipStream_t st) {
    (void)tmp;
    if (k + nq == 0) return hipSuccess;
    select_topk_kernel<<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    return hipGetLastError();
}

}  // namespace fr
