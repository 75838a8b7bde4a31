// argTopk + Q index (Table 1, Sec. 3.2; Sec. 4.3) for score vectors that no longer fit one workgroup's registers:
// the same definition as k_select.hip (the k largest scores, ties to the lowest index, emitted in ascending index
// order, then the question positions), spread over the chip.  At these sizes the selection is bound by reading the
// scores, so the aim is few passes over them:
//   1. minimum and maximum key                                                    (one read)
//   2. 4096-bin histogram of the top 12 bits of key - min, pick the bin of the k-th largest   (one read)
//   3. the same for the next 12 bits among the keys of that bin; these candidates (about n / 4096 of them for spread
//      data) are also listed, and the last 8 bits are settled on the list alone   (one read)
//   4. per wave: how many of its keys lie above the threshold key / equal it, then a scan over the waves  (one read)
//   5. every wave emits its selected indices at its offset, in index order        (one read)
// Integer work only: the result is unique and equal to the single-workgroup kernel's.
#include "fr_internal.hpp"

#include <algorithm>

namespace fr {

namespace {

__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger score <=> larger key
}

constexpr int BINS = 4096, DIGIT = 12;
constexpr int MAX_UNITS = 8192;          // waves of the counting / emitting passes
constexpr int CAND_CAP = 1 << 18;        // listed candidates; more than that and the last level re-reads the scores
constexpr int WG_LIST = 2048;            // candidates one workgroup collects in LDS before it appends them

struct State {
    uint32_t kmin, kmax;
    uint32_t prefix, mask;   // digits of (key - kmin) fixed so far
    uint32_t remaining;      // how many keys are still to be taken among those that match the prefix
    uint32_t cand_count;     // candidates seen by level 1 (listed up to CAND_CAP)
    uint32_t thr_key, need_eq;
    uint32_t pad[8];
};
// workspace, in 32-bit words
constexpr size_t W_STATE = 0, W_HIST = 16, W_GT = W_HIST + BINS, W_EQ = W_GT + MAX_UNITS, W_POS = W_EQ + MAX_UNITS,
                 W_SEEN = W_POS + MAX_UNITS, W_CAND = W_SEEN + MAX_UNITS, W_END = W_CAND + CAND_CAP;

__device__ __forceinline__ int bits_of(uint32_t span) { return span == 0u ? 1 : 32 - __clz((int)span); }
// digit position of a level: hi = bits not yet fixed before it; width = 0 means the level has nothing to do
__device__ __forceinline__ void level_digit(const State& s, int level, int& width, int& shift) {
    const int hi = bits_of(s.kmax - s.kmin) - DIGIT * level;
    width = hi <= 0 ? 0 : (hi < DIGIT ? hi : DIGIT);
    shift = hi - width;
}

__global__ __launch_bounds__(1024) void select_init_kernel(uint32_t* __restrict__ ws, int64_t n, int64_t k, int nq,
                                                           int32_t* __restrict__ out) {
    State* s = reinterpret_cast<State*>(ws + W_STATE);
    const int tid = threadIdx.x;
    if (tid == 0) {
        s->kmin = 0xFFFFFFFFu; s->kmax = 0u; s->prefix = 0u; s->mask = 0u;
        s->remaining = (uint32_t)k; s->cand_count = 0u; s->thr_key = 0u; s->need_eq = 0u;
    }
    for (int i = tid; i < BINS; i += 1024) ws[W_HIST + i] = 0u;
    for (int i = tid; i < nq; i += 1024) out[k + i] = (int32_t)(n + i);   // question tokens: positions n .. n + nq - 1
}

// Streams all n scores through f(index, key, valid): 16-byte loads, eight per thread in flight, every load issued
// before the first is used.  Every thread of the grid makes the same number of calls per round (invalid ones past
// the end carry valid = false), so f may use wave-wide votes.  The few scores before the first and after the last
// aligned 16 bytes go through block 0.
constexpr int STREAM_U = 8;
constexpr int STREAM_BLOCKS = 512;   // few workgroups: each ends with atomics on shared words (min / max, histogram bins)
template <class F>
__device__ __forceinline__ void stream_scores(const float* __restrict__ scores, int64_t n, F&& f) {
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const int64_t head = min(n, (int64_t)((4 - ((reinterpret_cast<uintptr_t>(scores) >> 2) & 3)) & 3));
    const int64_t nv = (n - head) >> 2;                       // aligned 16-byte groups
    const f32x4* v = reinterpret_cast<const f32x4*>(scores + head);
    const int64_t per_round = (int64_t)gridDim.x * 256 * STREAM_U;
    for (int64_t base = 0; base < nv; base += per_round) {
        f32x4 x[STREAM_U];
        int64_t vi[STREAM_U];
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) {
            vi[u] = base + ((int64_t)blockIdx.x * STREAM_U + u) * 256 + threadIdx.x;
            x[u] = v[min(vi[u], nv - 1)];
        }
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) f(head + 4 * vi[u] + e, score_key(x[u][e]), vi[u] < nv);
    }
    if (blockIdx.x == 0) {   // at most 3 + 3 scores
        const int64_t tail0 = head + 4 * nv, rest = head + (n - tail0);
        const int64_t i = (int64_t)threadIdx.x < head ? (int64_t)threadIdx.x : tail0 + ((int64_t)threadIdx.x - head);
        const bool valid = (int64_t)threadIdx.x < rest;
        f(i, valid ? score_key(scores[i]) : 0u, valid);
    }
}

__global__ __launch_bounds__(256) void select_minmax_kernel(const float* __restrict__ scores, int64_t n,
                                                            uint32_t* __restrict__ ws) {
    __shared__ uint32_t w_min[4], w_max[4];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    stream_scores(scores, n, [&](int64_t, uint32_t key, bool valid) {
        if (valid) { kmin = min(kmin, key); kmax = max(kmax, key); }
    });
    for (int o = 32; o > 0; o >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
    }
    if ((threadIdx.x & 63) == 0) { w_min[threadIdx.x >> 6] = kmin; w_max[threadIdx.x >> 6] = kmax; }
    __syncthreads();
    if (threadIdx.x == 0) {
        State* s = reinterpret_cast<State*>(ws + W_STATE);
        atomicMin(&s->kmin, min(min(w_min[0], w_min[1]), min(w_min[2], w_min[3])));
        atomicMax(&s->kmax, max(max(w_max[0], w_max[1]), max(w_max[2], w_max[3])));
    }
}

// Histogram of this level's digit over the keys that match the digits fixed so far.  LEVEL 1 also lists those
// keys' indices; LEVEL 2 walks that list when it is complete, else all scores.
template <int LEVEL>
__global__ __launch_bounds__(256) void select_hist_kernel(const float* __restrict__ scores, int64_t n,
                                                          uint32_t* __restrict__ ws) {
    __shared__ uint32_t hist[BINS];
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    const State s = *sp;
    int width, shift;
    level_digit(s, LEVEL, width, shift);
    if (width == 0) return;
    const uint32_t dm = (1u << width) - 1u;
    for (int i = threadIdx.x; i < BINS; i += 256) hist[i] = 0u;
    __syncthreads();
    // LEVEL 1 lists its candidates: first in LDS, then one reservation in the global list per workgroup (an atomic
    // per candidate on one global word would serialise: about 8 ns each)
    __shared__ uint32_t wg_list[WG_LIST];
    __shared__ uint32_t wg_count, wg_base;
    if (threadIdx.x == 0) wg_count = 0u;
    __syncthreads();
    auto visit = [&](int64_t idx, uint32_t key, bool valid) {
        const uint32_t rk = key - s.kmin;
        if (valid && (rk & s.mask) == s.prefix) {
            atomicAdd(&hist[(rk >> shift) & dm], 1u);
            if (LEVEL == 1) {
                const uint32_t slot = atomicAdd(&wg_count, 1u);
                if (slot < (uint32_t)WG_LIST) wg_list[slot] = (uint32_t)idx;
            }
        }
    };
    if (LEVEL == 2 && s.cand_count <= (uint32_t)CAND_CAP) {
        for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < (int64_t)s.cand_count; j += (int64_t)gridDim.x * 256)
            visit(0, score_key(scores[ws[W_CAND + j]]), true);
    } else {
        stream_scores(scores, n, visit);
    }
    __syncthreads();
    if (LEVEL == 1) {
        // a workgroup with more candidates than its LDS list holds makes the global count overflow on purpose:
        // the last level then re-reads the scores instead of the list
        if (threadIdx.x == 0) wg_base = atomicAdd(&sp->cand_count, wg_count <= (uint32_t)WG_LIST ? wg_count : (uint32_t)CAND_CAP + 1u);
        __syncthreads();
        if (wg_count <= (uint32_t)WG_LIST)
            for (uint32_t i = threadIdx.x; i < wg_count; i += 256)
                if (wg_base + i < (uint32_t)CAND_CAP) ws[W_CAND + wg_base + i] = wg_list[i];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < BINS; i += 256) {
        const uint32_t c = hist[i];
        if (c != 0u) atomicAdd(&ws[W_HIST + i], c);
    }
}

// One workgroup: the digit of the k-th largest key is the largest d whose suffix count reaches `remaining`.
template <int LEVEL>
__global__ __launch_bounds__(1024) void select_pick_kernel(uint32_t* __restrict__ ws) {
    __shared__ uint32_t wave_tot[16];
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    const State s = *sp;
    int width, shift;
    level_digit(s, LEVEL, width, shift);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (width != 0) {
        // thread t owns bins 4t .. 4t+3; suffix sums run from the last bin down
        uint32_t c[4], own = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) { c[e] = ws[W_HIST + 4 * tid + e]; own += c[e]; }
        uint32_t suf = own;   // sum over threads >= t of this wave
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = (uint32_t)__shfl_down((int)suf, o);
            if (lane + o < 64) suf += t;
        }
        if (lane == 0) wave_tot[wave] = suf;
        __syncthreads();
        for (int w2 = wave + 1; w2 < 16; ++w2) suf += wave_tot[w2];
        uint32_t above = suf - own;   // keys with a digit beyond this thread's bins
        if (suf >= s.remaining && above < s.remaining) {
#pragma unroll
            for (int e = 3; e >= 0; --e) {
                if (above + c[e] >= s.remaining) {
                    sp->prefix = s.prefix | ((uint32_t)(4 * tid + e) << shift);
                    sp->mask = s.mask | (((1u << width) - 1u) << shift);
                    sp->remaining = s.remaining - above;
                    break;
                }
                above += c[e];
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) ws[W_HIST + 4 * tid + e] = 0u;
    }
    if (LEVEL == 2) {
        __syncthreads();
        if (tid == 0) {
            sp->thr_key = sp->prefix + s.kmin;
            sp->need_eq = sp->remaining;
        }
    }
}

// Unit u (one wave) owns the contiguous range [u * per_unit, (u + 1) * per_unit), per_unit a multiple of 64.
__global__ __launch_bounds__(256) void select_count_kernel(const float* __restrict__ scores, int64_t n, int64_t per_unit,
                                                           uint32_t* __restrict__ ws) {
    const State* sp = reinterpret_cast<const State*>(ws + W_STATE);
    const uint32_t thr = sp->thr_key;
    const int lane = threadIdx.x & 63;
    const int64_t u = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t begin = u * per_unit, end = min(n, begin + per_unit);
    uint32_t gt = 0u, eq = 0u;
    for (int64_t i = begin + lane; i < end; i += 64) {
        const uint32_t key = score_key(scores[i]);
        gt += key > thr;
        eq += key == thr;
    }
    for (int o = 32; o > 0; o >>= 1) {
        gt += (uint32_t)__shfl_xor((int)gt, o);
        eq += (uint32_t)__shfl_xor((int)eq, o);
    }
    if (lane == 0) { ws[W_GT + u] = gt; ws[W_EQ + u] = eq; }
}

// Exclusive scans over the units: equal keys seen before each unit, then output offsets (keys above the threshold
// plus the share of the equal keys that is still needed, lowest index first).
__global__ __launch_bounds__(1024) void select_scan_kernel(uint32_t* __restrict__ ws, int n_units) {
    __shared__ uint32_t wave_tot[16];
    const State* sp = reinterpret_cast<const State*>(ws + W_STATE);
    const uint32_t need_eq = sp->need_eq;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int PER = MAX_UNITS / 1024;
    auto block_exclusive = [&](uint32_t own) -> uint32_t {   // sum of `own` over the threads before this one
        uint32_t inc = own;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = (uint32_t)__shfl_up((int)inc, o);
            if (lane >= o) inc += t;
        }
        __syncthreads();
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t before = 0u;
        for (int w2 = 0; w2 < wave; ++w2) before += wave_tot[w2];
        return before + inc - own;
    };
    uint32_t gt[PER], eq[PER], own = 0u;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int u = PER * tid + e;
        gt[e] = u < n_units ? ws[W_GT + u] : 0u;
        eq[e] = u < n_units ? ws[W_EQ + u] : 0u;
        own += eq[e];
    }
    uint32_t seen = block_exclusive(own);
    uint32_t out_own = 0u, seen_at[PER], take[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        seen_at[e] = seen;
        take[e] = gt[e] + (need_eq > seen ? min(eq[e], need_eq - seen) : 0u);
        out_own += take[e];
        seen += eq[e];
    }
    uint32_t pos = block_exclusive(out_own);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int u = PER * tid + e;
        if (u < n_units) { ws[W_POS + u] = pos; ws[W_SEEN + u] = seen_at[e]; }
        pos += take[e];
    }
}

__global__ __launch_bounds__(256) void select_emit_kernel(const float* __restrict__ scores, int64_t n, int64_t per_unit,
                                                          const uint32_t* __restrict__ ws, int32_t* __restrict__ out) {
    const State* sp = reinterpret_cast<const State*>(ws + W_STATE);
    const uint32_t thr = sp->thr_key, need_eq = sp->need_eq;
    const int lane = threadIdx.x & 63;
    const int64_t u = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t begin = u * per_unit, end = min(n, begin + per_unit);
    if (begin >= end) return;
    uint32_t pos = ws[W_POS + u], eq_seen = ws[W_SEEN + u];
    const uint64_t below = (1ull << lane) - 1ull;
    for (int64_t base = begin; base < end; base += 64) {   // wave-uniform trip count
        const int64_t i = base + lane;
        const uint32_t key = i < end ? score_key(scores[i]) : 0u;
        const bool gt = i < end && key > thr, eq = i < end && key == thr;
        const uint64_t beq = __ballot(eq);
        const bool sel = gt || (eq && eq_seen + (uint32_t)__popcll(beq & below) < need_eq);
        const uint64_t bsel = __ballot(sel);
        if (sel) out[pos + (uint32_t)__popcll(bsel & below)] = (int32_t)i;
        pos += (uint32_t)__popcll(bsel);
        eq_seen += (uint32_t)__popcll(beq);
    }
}

}  // namespace

size_t select_workspace_bytes() { return W_END * sizeof(uint32_t); }

hipError_t launch_select_large(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* ws,
                               hipStream_t st) {
    select_init_kernel<<<dim3(1), dim3(1024), 0, st>>>(ws, n, k, nq, q_index);
    if (k <= 0 || n <= 0) return hipGetLastError();
    // (k == n needs no special case: the threshold is then the smallest key, and every key equal to it is needed)
    const int grid = (int)std::min<int64_t>(STREAM_BLOCKS, (n + 2047) / 2048);
    select_minmax_kernel<<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws);
    select_hist_kernel<0><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws);
    select_pick_kernel<0><<<dim3(1), dim3(1024), 0, st>>>(ws);
    select_hist_kernel<1><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws);
    select_pick_kernel<1><<<dim3(1), dim3(1024), 0, st>>>(ws);
    select_hist_kernel<2><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws);
    select_pick_kernel<2><<<dim3(1), dim3(1024), 0, st>>>(ws);
    // units of at least 1024 scores, at most MAX_UNITS of them
    int64_t per_unit = std::max<int64_t>(1024, (n + MAX_UNITS - 1) / MAX_UNITS);
    per_unit = (per_unit + 63) / 64 * 64;
    const int n_units = (int)((n + per_unit - 1) / per_unit);
    const int blocks = (n_units + 3) / 4;
    select_count_kernel<<<dim3(blocks), dim3(256), 0, st>>>(scores, n, per_unit, ws);
    select_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(ws, n_units);
    select_emit_kernel<<<dim3(blocks), dim3(256), 0, st>>>(scores, n, per_unit, ws, q_index);
    return hipGetLastError();
}

}  // namespace fr
