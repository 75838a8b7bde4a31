// argTopk + Q index (Table 1, Sec. 3.2; Sec. 4.3) for score vectors that no longer fit one workgroup's registers:
// the same definition as k_select.hip (the k largest scores, ties to the lowest index, emitted in ascending index
// order, then the question positions), spread over the chip.  At these sizes the selection is bound by reading the
// scores, so the aim is few passes over them.  Three reads:
//   1. histogram of the top 14 bits of the order-preserving key (sign, exponent, 5 mantissa bits); the bin that holds
//      the k-th largest key follows from its suffix sums                                              (one read)
//   2. histogram of the next 14 bits among the keys of that bin, whose indices are also listed; the last 4 bits are
//      settled on the list alone (on all scores only if the list overflowed)                           (one read)
//   3. one kernel counts, scans and emits: a workgroup keeps its 32768 keys in registers, counts those above / equal
//      to the threshold, publishes the counts, obtains the counts of all tiles before it by a decoupled look-back
//      over the tiles' status words, and writes its selected indices at their final places          (one read)
// No minimum / maximum pass: the digits are those of the raw key.  Integer work only: the result is unique and equal
// to the single-workgroup kernel's.
#include "fr_internal.hpp"

#include <algorithm>

namespace fr {

namespace {

__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger score <=> larger key
}

// digit positions of the three levels
constexpr int BITS0 = 14, BITS1 = 14, BITS2 = 4;
constexpr int SHIFT0 = 18, SHIFT1 = 4, SHIFT2 = 0;
constexpr int BINS = 1 << 14;            // bins of levels 0 and 1 (level 2: 16)
static_assert(BITS0 + BITS1 + BITS2 == 32 && SHIFT0 == BITS1 + BITS2 && SHIFT1 == BITS2, "digits");
constexpr int WG_LIST = 2048;            // candidates one workgroup collects in LDS before it appends them
constexpr int TILE = (int)SELECT_TILE;    // scores per workgroup of the emitting pass (1024 threads x 32 keys)
constexpr int64_t MAX_TILES = 65536;     // 2^31 scores

struct State {
    uint32_t prefix, mask;   // digits of the key fixed so far
    uint32_t remaining;      // how many keys are still to be taken among those that match the prefix
    uint32_t cand_count;     // candidates seen by level 1 (listed up to the list's capacity)
    uint32_t ticket;         // tiles of the emitting pass are numbered in the order in which their workgroups start
    uint32_t pad[11];
};
// workspace, in 32-bit words: state, three histograms, the tiles' status words (64 bits each), candidate list
constexpr size_t W_STATE = 0, W_HIST0 = 16, W_HIST1 = W_HIST0 + BINS, W_HIST2 = W_HIST1 + BINS, W_STATUS = W_HIST2 + 16;
static_assert(W_STATUS % 2 == 0, "status words are 8-byte aligned");
static_assert(W_STATUS == SELECT_FIXED_WORDS, "layout as announced to the callers that size the scratch");
constexpr size_t CAND_MIN = 1 << 16;     // smallest candidate list worth having

struct Layout {
    int64_t n_tiles;
    size_t w_cand;        // first word of the candidate list
    uint32_t cand_cap;    // its capacity
};
// false: the workspace cannot hold the status words of n scores plus a minimal candidate list
bool make_layout(int64_t n, size_t ws_words, Layout* l) {
    l->n_tiles = (n + TILE - 1) / TILE;
    l->w_cand = W_STATUS + 2 * (size_t)l->n_tiles;
    if (l->n_tiles > MAX_TILES || l->w_cand + CAND_MIN > ws_words) return false;
    const size_t cap = ws_words - l->w_cand;
    l->cand_cap = (uint32_t)std::min<size_t>(cap, (size_t)1 << 30);
    return true;
}

__global__ __launch_bounds__(256) void select_init_kernel(uint32_t* __restrict__ ws, int64_t n, int64_t k, int nq,
                                                          int64_t n_tiles, int32_t* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x, stride = (int64_t)gridDim.x * 256;
    if (t == 0) {
        State* s = reinterpret_cast<State*>(ws + W_STATE);
        s->prefix = 0u; s->mask = 0u; s->remaining = (uint32_t)k; s->cand_count = 0u; s->ticket = 0u;
    }
    const int64_t n_clear = (int64_t)(W_STATUS - W_HIST0) + 2 * n_tiles;   // histograms and status words
    for (int64_t i = t; i < n_clear; i += stride) ws[W_HIST0 + i] = 0u;
    for (int64_t i = t; i < nq; i += stride) out[k + i] = (int32_t)(n + i);   // question tokens: positions n .. n + nq - 1
}

// Streams all n scores through f(index, key, valid): 16-byte loads, eight per thread in flight, every load issued
// before the first is used.  Every thread of the grid makes the same number of calls per round (invalid ones past
// the end carry valid = false), so f may use wave-wide votes.  The few scores before the first and after the last
// aligned 16 bytes go through block 0.
constexpr int STREAM_U = 8;
constexpr int STREAM_BLOCKS = 512;   // few workgroups: each ends with atomics on shared words (histogram bins)
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

// Histogram of this level's digit over the keys that match the digits fixed so far.  LEVEL 1 also lists those
// keys' indices; LEVEL 2 walks that list when it is complete, else all scores.
template <int LEVEL>
__global__ __launch_bounds__(256) void select_hist_kernel(const float* __restrict__ scores, int64_t n,
                                                          uint32_t* __restrict__ ws, size_t w_cand, uint32_t cand_cap) {
    constexpr int NB = LEVEL == 2 ? 16 : BINS;
    constexpr int SHIFT = LEVEL == 0 ? SHIFT0 : (LEVEL == 1 ? SHIFT1 : SHIFT2);
    constexpr size_t W_HIST = LEVEL == 0 ? W_HIST0 : (LEVEL == 1 ? W_HIST1 : W_HIST2);
    __shared__ uint32_t hist[NB];
    __shared__ uint32_t wg_list[LEVEL == 1 ? WG_LIST : 1];
    __shared__ uint32_t wg_count, wg_base;
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    const uint32_t prefix = sp->prefix, mask = sp->mask, cand_count = sp->cand_count;
    for (int i = threadIdx.x; i < NB; i += 256) hist[i] = 0u;
    if (threadIdx.x == 0) wg_count = 0u;
    __syncthreads();
    // LEVEL 1 lists its candidates: first in LDS, then one reservation in the global list per workgroup (an atomic
    // per candidate on one global word would serialise: about 8 ns each)
    auto visit = [&](int64_t idx, uint32_t key, bool valid) {
        if (valid && (key & mask) == prefix) {
            atomicAdd(&hist[(key >> SHIFT) & (uint32_t)(NB - 1)], 1u);
            if (LEVEL == 1) {
                const uint32_t slot = atomicAdd(&wg_count, 1u);
                if (slot < (uint32_t)WG_LIST) wg_list[slot] = (uint32_t)idx;
            }
        }
    };
    if (LEVEL == 2 && cand_count <= cand_cap) {
        for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < (int64_t)cand_count; j += (int64_t)gridDim.x * 256)
            visit(0, score_key(scores[ws[w_cand + j]]), true);
    } else {
        stream_scores(scores, n, visit);
    }
    __syncthreads();
    if (LEVEL == 1) {
        // a workgroup with more candidates than its LDS list holds makes the global count overflow on purpose:
        // the last level then re-reads the scores instead of the list
        if (threadIdx.x == 0) wg_base = atomicAdd(&sp->cand_count, wg_count <= (uint32_t)WG_LIST ? wg_count : cand_cap + 1u);
        __syncthreads();
        if (wg_count <= (uint32_t)WG_LIST)
            for (uint32_t i = threadIdx.x; i < wg_count; i += 256)
                if (wg_base + i < cand_cap) ws[w_cand + wg_base + i] = wg_list[i];
    }
    for (int i = threadIdx.x; i < NB; i += 256) {
        const uint32_t c = hist[i];
        if (c != 0u) atomicAdd(&ws[W_HIST + i], c);
    }
}

// One workgroup: the digit of the k-th largest key is the largest d whose suffix count reaches `remaining`.
// Thread t owns PER consecutive bins; suffix sums run from the last bin down.  Afterwards `remaining` counts the keys
// still to take among those with the chosen digits; after LEVEL 2 the prefix is the threshold key itself.
template <int LEVEL>
__global__ __launch_bounds__(1024) void select_pick_kernel(uint32_t* __restrict__ ws) {
    constexpr int NB = LEVEL == 2 ? 16 : BINS;
    constexpr int PER = LEVEL == 2 ? 1 : BINS / 1024;
    constexpr int SHIFT = LEVEL == 0 ? SHIFT0 : (LEVEL == 1 ? SHIFT1 : SHIFT2);
    constexpr size_t W_HIST = LEVEL == 0 ? W_HIST0 : (LEVEL == 1 ? W_HIST1 : W_HIST2);
    __shared__ uint32_t wave_tot[16];
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    const uint32_t prefix = sp->prefix, mask = sp->mask, remaining = sp->remaining;   // read before any thread writes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t c[PER], own = 0u;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        c[e] = (PER * tid + e < NB) ? ws[W_HIST + PER * tid + e] : 0u;
        own += c[e];
    }
    uint32_t suf = own;   // sum over threads >= t of this wave
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = (uint32_t)__shfl_down((int)suf, o);
        if (lane + o < 64) suf += t;
    }
    if (lane == 0) wave_tot[wave] = suf;
    __syncthreads();
    for (int w2 = wave + 1; w2 < 16; ++w2) suf += wave_tot[w2];
    uint32_t above = suf - own;   // keys with a digit beyond this thread's bins
    if (suf >= remaining && above < remaining) {   // exactly one thread
#pragma unroll
        for (int e = PER - 1; e >= 0; --e) {
            if (above + c[e] >= remaining) {
                sp->prefix = prefix | ((uint32_t)(PER * tid + e) << SHIFT);
                sp->mask = mask | ((uint32_t)(NB - 1) << SHIFT);
                sp->remaining = remaining - above;
                break;
            }
            above += c[e];
        }
    }
}

// ---- pass 3: count, scan over the tiles (decoupled look-back) and emit, in one kernel ---------------------------
// A tile's status word: bits 62..63 = 0 nothing yet / 1 the tile's own counts / 2 the counts of all tiles up to and
// including it; bits 31..61 = keys equal to the threshold; bits 0..30 = keys above it.  The word is the whole
// message (no other memory is exchanged between workgroups), so relaxed device-scope accesses suffice.  Tiles are
// numbered by a ticket taken when a workgroup starts: every tile with a lower number has then started too and
// publishes without waiting for anything but lower-numbered tiles, so every wait below ends.
constexpr uint64_t ST_OWN = 1ull << 62, ST_INCL = 2ull << 62;
__device__ __forceinline__ uint64_t st_pack(uint64_t flag, uint32_t gt, uint32_t eq) { return flag | ((uint64_t)eq << 31) | gt; }

__global__ __launch_bounds__(1024, 8) void select_emit_kernel(const float* __restrict__ scores, int64_t n,
                                                           uint32_t* __restrict__ ws, int32_t* __restrict__ out) {
    constexpr int SLOTS = 32;   // keys per thread; wave w owns keys [2048 w, 2048 (w + 1)) of the tile, slot j = 64 of them
    __shared__ uint32_t s_tile, s_gt[16], s_eq[16], s_base_gt, s_base_eq;
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    uint64_t* status = reinterpret_cast<uint64_t*>(ws + W_STATUS);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_tile = atomicAdd(&sp->ticket, 1u);
    const uint32_t thr = sp->prefix, need_eq = sp->remaining;   // (level 2 left the threshold key and the equal keys to take)
    __syncthreads();
    const int64_t tile = s_tile;
    const int64_t first = tile * TILE + wave * (64 * SLOTS) + lane;   // this lane's keys: first + 64 j
    // all loads in flight together, addressed as (tile base: uniform) + (32-bit offset in the tile); offsets clamped
    // to the last score
    const float* __restrict__ tile_scores = scores + tile * TILE;
    const uint32_t off0 = (uint32_t)(wave * (64 * SLOTS) + lane);
    const uint32_t last = (uint32_t)min((int64_t)TILE - 1, n - 1 - tile * TILE);
    float raw[SLOTS];
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) raw[j] = tile_scores[min(off0 + 64u * j, last)];
    uint32_t gt_bits = 0u, eq_bits = 0u;   // bit j: this lane's key of slot j lies above / equals the threshold
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
        const uint32_t key = score_key(raw[j]);
        const bool valid = off0 + 64u * j <= last;
        gt_bits |= (uint32_t)(valid && key > thr) << j;
        eq_bits |= (uint32_t)(valid && key == thr) << j;
    }
    uint32_t w_cnt = (uint32_t)__popc(gt_bits) | ((uint32_t)__popc(eq_bits) << 16);   // wave totals, packed (<= 2048 each)
    for (int o = 32; o > 0; o >>= 1) w_cnt += (uint32_t)__shfl_xor((int)w_cnt, o);
    const uint32_t w_gt = w_cnt & 0xFFFFu, w_eq = w_cnt >> 16;
    if (lane == 0) { s_gt[wave] = w_gt; s_eq[wave] = w_eq; }
    __syncthreads();
    if (wave == 0) {
        uint32_t t_gt = 0u, t_eq = 0u;   // the tile's own counts
#pragma unroll
        for (int w2 = 0; w2 < 16; ++w2) { t_gt += s_gt[w2]; t_eq += s_eq[w2]; }
        if (lane == 0 && tile > 0)
            __hip_atomic_store(&status[tile], st_pack(ST_OWN, t_gt, t_eq), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // look back: lane l examines tile (tile - 1 - l - 64 r); tiles below 0 count as "all before: nothing"
        uint32_t b_gt = 0u, b_eq = 0u;
        for (int64_t hi = tile - 1; ; hi -= 64) {
            const int64_t t = hi - lane;
            uint64_t st = ST_INCL;
            if (t >= 0) {
                do {
                    st = __hip_atomic_load(&status[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((st >> 62) == 0ull) __builtin_amdgcn_s_sleep(1);
                } while ((st >> 62) == 0ull);
            }
            const uint64_t incl = __ballot((st >> 62) == 2ull);
            // the nearest tile that knows its inclusive counts ends the walk: lanes up to it contribute
            const int stop = incl ? (int)__builtin_ctzll(incl) : 63;
            uint32_t g = lane <= stop ? (uint32_t)(st & 0x7FFFFFFFull) : 0u;
            uint32_t e = lane <= stop ? (uint32_t)((st >> 31) & 0x7FFFFFFFull) : 0u;
            for (int o = 32; o > 0; o >>= 1) {
                g += (uint32_t)__shfl_xor((int)g, o);
                e += (uint32_t)__shfl_xor((int)e, o);
            }
            b_gt += g;
            b_eq += e;
            if (incl) break;
        }
        if (lane == 0) {
            __hip_atomic_store(&status[tile], st_pack(ST_INCL, b_gt + t_gt, b_eq + t_eq), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            s_base_gt = b_gt;
            s_base_eq = b_eq;
        }
    }
    __syncthreads();
    uint32_t gt_seen = s_base_gt, eq_seen = s_base_eq;   // keys above / equal to the threshold before this wave's first key
    for (int w2 = 0; w2 < wave; ++w2) { gt_seen += s_gt[w2]; eq_seen += s_eq[w2]; }
    // key i is chosen if it lies above the threshold, or equals it and fewer than need_eq equal keys precede it; its
    // place is (keys above the threshold before i) + min(equal keys before i, need_eq)
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
        const bool gt = (gt_bits >> j) & 1u, eq = (eq_bits >> j) & 1u;
        const uint64_t bg = __ballot(gt), be = __ballot(eq);
        const uint32_t g_before = gt_seen + __builtin_amdgcn_mbcnt_hi((uint32_t)(bg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bg, 0u));
        const uint32_t e_before = eq_seen + __builtin_amdgcn_mbcnt_hi((uint32_t)(be >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)be, 0u));
        if (gt || (eq && e_before < need_eq)) out[g_before + min(e_before, need_eq)] = (int32_t)(first + 64 * j);
        gt_seen += (uint32_t)__popcll(bg);
        eq_seen += (uint32_t)__popcll(be);
    }
}

}  // namespace

size_t select_workspace_bytes() { return select_workspace_words((int64_t)MAX_TILES * TILE) * sizeof(uint32_t); }

hipError_t launch_select_large(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* ws,
                               size_t ws_bytes, hipStream_t st) {
    Layout lay;
    if (!make_layout(n, ws_bytes / sizeof(uint32_t), &lay)) return hipErrorInvalidValue;
    const int64_t n_clear = (int64_t)(W_STATUS - W_HIST0) + 2 * lay.n_tiles + nq;
    select_init_kernel<<<dim3((unsigned)std::min<int64_t>(256, (n_clear + 255) / 256)), dim3(256), 0, st>>>(ws, n, k, nq, lay.n_tiles, q_index);
    if (k <= 0 || n <= 0) return hipGetLastError();
    // (k == n needs no special case: the threshold is then the smallest key, and every key equal to it is needed)
    const int grid = (int)std::min<int64_t>(STREAM_BLOCKS, (n + 2047) / 2048);
    select_hist_kernel<0><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws, lay.w_cand, lay.cand_cap);
    select_pick_kernel<0><<<dim3(1), dim3(1024), 0, st>>>(ws);
    select_hist_kernel<1><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws, lay.w_cand, lay.cand_cap);
    select_pick_kernel<1><<<dim3(1), dim3(1024), 0, st>>>(ws);
    select_hist_kernel<2><<<dim3(grid), dim3(256), 0, st>>>(scores, n, ws, lay.w_cand, lay.cand_cap);
    select_pick_kernel<2><<<dim3(1), dim3(1024), 0, st>>>(ws);
    select_emit_kernel<<<dim3((unsigned)lay.n_tiles), dim3(1024), 0, st>>>(scores, n, ws, q_index);
    return hipGetLastError();
}

}  // namespace fr
