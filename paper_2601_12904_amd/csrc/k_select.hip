// Selection half of Query-Guided Selection: argTopk of the critical scores (Table 1, Sec. 3.2)
// and the Q index of Sec. 4.3 (ascending critical tokens, then the question tokens).
//
// Integer work only.  Scores are mapped to order-preserving 32-bit keys; a most-significant-digit
// radix select (4 passes of 8 bits, LDS histograms) finds the key of the k-th largest score; an
// ordered compaction then emits, in index order, every token above that key plus the first
// (lowest-index) tokens equal to it that are still needed.  The result is unique, so it does not
// depend on scheduling.  One workgroup: the 64 KB of scores of a 17k-token prompt fit its registers, and the
// whole selection is latency- rather than bandwidth-sized.
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

// Among the candidates of this pass (keys that share the digits fixed so far), the digit of the k-th largest
// key is the largest d whose suffix count S[d] = sum_{b >= d} hist[b] still reaches `remaining`.  One thread
// per bin: suffix sums by wave shuffles, then the single thread that satisfies the condition publishes it.
__device__ __forceinline__ void pick_digit(const uint32_t* hist, uint32_t* wave_tot, uint32_t* s_prefix,
                                           uint32_t* s_remaining, int shift) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t suf = 0u, own = 0u;
    if (tid < 256) {
        own = hist[tid];
        suf = own;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_down(suf, o);
            if (lane + o < 64) suf += t;
        }
        if (lane == 0) wave_tot[wave] = suf;   // total of bins 64 wave .. 64 wave + 63
    }
    __syncthreads();
    if (tid < 256) {
        for (int w2 = wave + 1; w2 < 4; ++w2) suf += wave_tot[w2];
        const uint32_t remaining = *s_remaining;
        const uint32_t above = suf - own;      // candidates with a larger digit
        if (suf >= remaining && above < remaining) {
            *s_remaining = remaining - above;  // still to take among keys with this digit
            *s_prefix |= (uint32_t)tid << shift;
        }
    }
    __syncthreads();
}

// PER > 0: every thread keeps its PER consecutive keys in registers (n <= SEL_THREADS * PER);
// PER == 0: any n, the scores are re-read from memory in every pass.
template <int PER>
__global__ __launch_bounds__(SEL_THREADS) void select_topk_kernel(const float* __restrict__ scores, int64_t n,
                                                                  int64_t k, int nq, int32_t* __restrict__ out) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_sums[SEL_THREADS / 64 + 1];
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t s_prefix, s_remaining;
    const int tid = threadIdx.x;

    // question tokens: positions n .. n + nq - 1
    for (int i = tid; i < nq; i += SEL_THREADS) out[k + i] = (int32_t)(n + i);
    if (k <= 0 || n <= 0) return;

    // thread t owns the contiguous index range [lo, hi)
    const int64_t per = (PER > 0) ? PER : (n + SEL_THREADS - 1) / SEL_THREADS;
    const int64_t lo = min(n, (int64_t)tid * per), hi = min(n, lo + per);
    const int cnt = (int)(hi - lo);
    uint32_t keys[PER > 0 ? PER : 1];
    if (PER > 0) {
#pragma unroll
        for (int i = 0; i < PER; ++i) keys[i] = (i < cnt) ? score_key(scores[lo + i]) : 0u;
    }
    auto key_at = [&](int i) -> uint32_t { return (PER > 0) ? keys[i] : score_key(scores[lo + i]); };

    uint32_t thr_key = 0u;     // key of the k-th largest score
    uint32_t need_eq = 0u;     // how many tokens equal to it are taken
    const bool take_all = (k >= n);
    if (!take_all) {
        if (tid == 0) { s_prefix = 0u; s_remaining = (uint32_t)k; }
        uint32_t mask = 0u;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            if (PER > 0) {
#pragma unroll
                for (int i = 0; i < PER; ++i)
                    if (i < cnt && (keys[i] & mask) == prefix) atomicAdd(&hist[(keys[i] >> shift) & 255u], 1u);
            } else {
                for (int i = 0; i < cnt; ++i) {
                    const uint32_t key = key_at(i);
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                }
            }
            __syncthreads();
            pick_digit(hist, wave_tot, &s_prefix, &s_remaining, shift);
            mask |= 0xFFu << shift;
        }
        thr_key = s_prefix;
        need_eq = s_remaining;
    }

    // ordered compaction
    uint32_t cnt_gt = 0u, cnt_eq = 0u;
    if (PER > 0) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            cnt_gt += (i < cnt && (take_all || keys[i] > thr_key)) ? 1u : 0u;
            cnt_eq += (i < cnt && !take_all && keys[i] == thr_key) ? 1u : 0u;
        }
    } else {
        for (int i = 0; i < cnt; ++i) {
            const uint32_t key = key_at(i);
            cnt_gt += (take_all || key > thr_key) ? 1u : 0u;
            cnt_eq += (!take_all && key == thr_key) ? 1u : 0u;
        }
    }
    uint32_t total;
    const uint32_t eq_before = block_exclusive_scan(cnt_eq, wave_sums, &total);
    uint32_t eq_take = 0u;
    if (need_eq > eq_before) eq_take = min(cnt_eq, need_eq - eq_before);
    const uint32_t out_before = block_exclusive_scan(cnt_gt + eq_take, wave_sums, &total);
    uint32_t pos = out_before, eq_left = eq_take;
    if (PER > 0) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (i < cnt) {
                bool sel = take_all || keys[i] > thr_key;
                if (!take_all && keys[i] == thr_key && eq_left > 0u) { sel = true; --eq_left; }
                if (sel) out[pos++] = (int32_t)(lo + i);
            }
        }
    } else {
        for (int i = 0; i < cnt; ++i) {
            const uint32_t key = key_at(i);
            bool sel = take_all || key > thr_key;
            if (!take_all && key == thr_key && eq_left > 0u) { sel = true; --eq_left; }
            if (sel) out[pos++] = (int32_t)(lo + i);
        }
    }
}

hipError_t launch_select(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* tmp,
                         hipStream_t st) {
    (void)tmp;
    if (k + nq == 0) return hipSuccess;
    if (n <= (int64_t)SEL_THREADS * 8)
        select_topk_kernel<8><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    else if (n <= (int64_t)SEL_THREADS * 32)
        select_topk_kernel<32><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    else
        select_topk_kernel<0><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    return hipGetLastError();
}

}  // namespace fr
