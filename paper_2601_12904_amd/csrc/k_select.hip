// Selection half of Query-Guided Selection: argTopk of the critical scores (Table 1, Sec. 3.2)
// and the Q index of Sec. 4.3 (ascending critical tokens, then the question tokens).
//
// Integer work only.  Scores are mapped to order-preserving 32-bit keys; a most-significant-digit
// radix select (at most 4 passes of 8 bits, LDS histograms) finds the key of the k-th largest score; an
// ordered compaction then emits, in index order, every token above that key plus the first
// (lowest-index) tokens equal to it that are still needed.  The result is unique, so it does not
// depend on scheduling.  One workgroup: the 64 KB of scores of a 17k-token prompt fit its registers, and the
// whole selection is latency- rather than bandwidth-sized (longer score vectors: k_select_large.hip).  Scores of one prompt are clustered (their sign and
// most exponent bits agree), which would pile a plain histogram onto one or two bins; the digits are therefore
// taken from key - min(key), starting at the highest bit in which the largest and the smallest key differ.
#include "fr_internal.hpp"

namespace fr {

__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger score <=> larger key
}

constexpr int SEL_THREADS = 1024;

// Among the candidates of this pass (keys that share the digits fixed so far), the digit of the k-th largest
// key is the largest d whose suffix count S[d] = sum_{b >= d} hist[b] still reaches `remaining`.  One thread
// per bin: suffix sums by wave shuffles, then the single thread that satisfies the condition publishes it.
// `remaining` is read before the first barrier: between the two barriers the matching thread overwrites it, and the
// four bin waves do not run in lockstep, so a read behind the first barrier could see the reduced value and let a
// second bin match.  (The caller's barrier after the histogram orders this read behind the previous pass's write.)
__device__ __forceinline__ void pick_digit(const uint32_t* hist, uint32_t* wave_tot, uint32_t* s_prefix,
                                           uint32_t* s_remaining, int shift) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t remaining = *s_remaining;
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
        const uint32_t above = suf - own;      // candidates with a larger digit
        if (suf >= remaining && above < remaining) {
            *s_remaining = remaining - above;  // still to take among keys with this digit
            *s_prefix |= (uint32_t)tid << shift;
        }
    }
    __syncthreads();
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {   // set bits of lanes lower than this one
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

// Wave w owns the contiguous index range [w * 64 * per, (w + 1) * 64 * per); its i-th load covers the 64
// consecutive tokens base + 64 i + lane, so loads and stores are coalesced and (i, lane) order is index order.
// Every thread keeps its PER keys in registers (n <= SEL_THREADS * PER).
template <int PER>
__global__ __launch_bounds__(SEL_THREADS) void select_topk_kernel(const float* __restrict__ scores, int64_t n,
                                                                  int64_t k, int nq, int32_t* __restrict__ out) {
    constexpr int WAVES = SEL_THREADS / 64;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_a[WAVES], wave_b[WAVES];
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t s_prefix, s_remaining;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // question tokens: positions n .. n + nq - 1
    for (int i = tid; i < nq; i += SEL_THREADS) out[k + i] = (int32_t)(n + i);
    if (k <= 0 || n <= 0) return;

    const int64_t first = (int64_t)wave * 64 * PER + lane;     // this lane's tokens: first + 64 i
    const int cnt = (int)max((int64_t)0, min((int64_t)PER, (n - first + 63) / 64));
    uint32_t keys[PER];
    {
        // branch-free: every load is issued (index clamped into the array) before the first one is waited for
        float raw[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) raw[i] = scores[min(first + 64 * i, n - 1)];
#pragma unroll
        for (int i = 0; i < PER; ++i) keys[i] = (i < cnt) ? score_key(raw[i]) : 0u;
    }

    uint32_t thr_key = 0u;     // key of the k-th largest score
    uint32_t need_eq = 0u;     // how many tokens equal to it are taken
    const bool take_all = (k >= n);
    if (!take_all) {
        // range of the keys: block-wide minimum and maximum
        uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (i < cnt) { kmin = min(kmin, keys[i]); kmax = max(kmax, keys[i]); }
        for (int o = 32; o > 0; o >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
        }
        if (lane == 0) { wave_a[wave] = kmin; wave_b[wave] = kmax; }
        if (tid == 0) { s_prefix = 0u; s_remaining = (uint32_t)k; }
        __syncthreads();
        kmin = wave_a[0];
        kmax = wave_b[0];
        for (int w2 = 1; w2 < WAVES; ++w2) { kmin = min(kmin, wave_a[w2]); kmax = max(kmax, wave_b[w2]); }
        // relative keys rk = key - kmin lie in [0, kmax - kmin]; digits of 8 bits (the last one narrower) are taken
        // from the highest bit in which the two extremes differ downwards
        const uint32_t span = kmax - kmin;
        int hi_bit = (span == 0u) ? 1 : 32 - __clz((int)span);   // number of significant bits of the relative keys
        uint32_t mask = 0u;
        while (hi_bit > 0) {
            const int width = min(8, hi_bit), shift = hi_bit - width;
            const uint32_t digit_mask = (1u << width) - 1u;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t prefix = s_prefix;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const uint32_t rk = keys[i] - kmin;
                if (i < cnt && (rk & mask) == prefix) atomicAdd(&hist[(rk >> shift) & digit_mask], 1u);
            }
            __syncthreads();
            pick_digit(hist, wave_tot, &s_prefix, &s_remaining, shift);
            mask |= digit_mask << shift;
            hi_bit = shift;
        }
        thr_key = s_prefix + kmin;
        need_eq = s_remaining;
    }

    // ordered compaction: per-wave counts by ballots, one exchange of the 16 wave totals, then every wave
    // writes its tokens in (i, lane) order
    auto is_gt = [&](int i, uint32_t key) { return i < cnt && (take_all || key > thr_key); };
    auto is_eq = [&](int i, uint32_t key) { return i < cnt && !take_all && key == thr_key; };
    uint32_t w_gt = 0u, w_eq = 0u;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        w_gt += (uint32_t)__popcll(__ballot(is_gt(i, keys[i])));
        w_eq += (uint32_t)__popcll(__ballot(is_eq(i, keys[i])));
    }
    __syncthreads();   // wave_a / wave_b are free again
    if (lane == 0) { wave_a[wave] = w_gt; wave_b[wave] = w_eq; }
    __syncthreads();
    uint32_t eq_seen = 0u, pos = 0u;   // equal keys and outputs of the waves before this one
    for (int w2 = 0; w2 < wave; ++w2) {
        const uint32_t e = wave_b[w2];
        pos += wave_a[w2] + ((need_eq > eq_seen) ? min(e, need_eq - eq_seen) : 0u);
        eq_seen += e;
    }
    auto emit = [&](int i, uint32_t key) {
        const bool gt = is_gt(i, key), eq = is_eq(i, key);
        const uint64_t beq = __ballot(eq);
        const bool sel = gt || (eq && eq_seen + lanes_below(beq) < need_eq);
        const uint64_t bsel = __ballot(sel);
        if (sel) out[pos + lanes_below(bsel)] = (int32_t)(first + 64 * (int64_t)i);
        pos += (uint32_t)__popcll(bsel);
        eq_seen += (uint32_t)__popcll(beq);
    };
#pragma unroll
    for (int i = 0; i < PER; ++i) emit(i, keys[i]);
}

static_assert(SELECT_ONE_WORKGROUP_MAX == (int64_t)SEL_THREADS * 32, "largest score vector of the one-workgroup kernel");

hipError_t launch_select(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* tmp,
                         size_t tmp_bytes, hipStream_t st) {
    if (k + nq == 0) return hipSuccess;
    if (n <= (int64_t)SEL_THREADS * 8)
        select_topk_kernel<8><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    else if (n <= (int64_t)SEL_THREADS * 16)
        select_topk_kernel<16><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    else if (n <= (int64_t)SEL_THREADS * 32)
        select_topk_kernel<32><<<dim3(1), dim3(SEL_THREADS), 0, st>>>(scores, n, k, nq, q_index);
    else
        return launch_select_large(scores, n, k, nq, q_index, tmp, tmp_bytes, st);
    return hipGetLastError();
}

}  // namespace fr
