// argTopk + Q index (Table 1, Sec. 3.2; Sec. 4.3) for score vectors that no longer fit one workgroup's registers:
// the same definition as k_select.hip (the k largest scores, ties to the lowest index, emitted in ascending index
// order, then the question positions), spread over the chip.  At these sizes the selection is bound by reading the
// scores and by the launches, so the aim is few passes and few kernels.  Four kernels, three reads:
//   1. histogram of the top 14 bits of the order-preserving key (sign, exponent, 5 mantissa bits)   (one read)
//   2. every workgroup derives from that histogram the bin that holds the k-th largest key (the largest digit whose
//      suffix count still reaches k); histogram of the next 14 bits among the keys of that bin, whose indices are
//      also listed                                                                                     (one read)
//   3. the same step for the last 4 bits, on the list alone (on all scores only if the list overflowed)
//   4. one kernel derives the threshold key, then counts, scans and emits: a workgroup keeps its 32768 keys in
//      registers, counts those above / equal to the threshold, publishes the counts, obtains the counts of all tiles
//      before it by a decoupled look-back over the tiles' status words, and writes its selected indices at their
//      final places                                                                                    (one read)
// No minimum / maximum pass: the digits are those of the raw key.  Integer work only: the result is unique and equal
// to the single-workgroup kernel's.
// The first kernel clears what the later ones need at zero (state, the other histograms, status words).  Its own
// histogram must be zero when a call starts: it is zero when the scratch is handed over, and every call leaves it zero
// (the third kernel clears it; after a failed launch the host does).
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
constexpr int THREADS = 1024;            // per workgroup, all kernels
constexpr int WG_LIST = 2048;            // candidates one workgroup collects in LDS before it appends them
constexpr int TILE = (int)SELECT_TILE;    // scores per workgroup of the emitting pass (1024 threads x 32 keys)
constexpr int64_t MAX_TILES = 65536;     // 2^31 scores

// What the levels so far have settled: digits of the threshold key, and how many keys are still to be taken among
// those that match them.
struct Pick {
    uint32_t prefix, mask, remaining;
};
struct State {
    Pick pick0, pick1;       // after levels 0 and 1 (recorded by workgroup 0 of the kernel that derives them)
    uint32_t cand_count;     // candidates seen by level 1 (listed up to the list's capacity)
    uint32_t ticket;         // tiles of the emitting pass are numbered in the order in which their workgroups start
    uint32_t pad[8];
};
static_assert(sizeof(State) == 64, "16 words");
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

// k = 0: only the question tokens, positions n .. n + nq - 1
__global__ __launch_bounds__(256) void select_questions_kernel(int64_t n, int64_t k, int nq, int32_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nq) out[k + i] = (int32_t)(n + i);
}

__global__ __launch_bounds__(256) void select_clear_kernel(uint32_t* __restrict__ ws, int64_t n_words) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * 256) ws[i] = 0u;
}

// Streams all n scores through f(index, key, valid): 16-byte loads, STREAM_U per thread; the loads of the next round
// are issued before the keys of this round are visited.  Every thread of the grid makes the same number of calls per
// round (invalid ones past the end carry valid = false), so f may use wave-wide votes.  The few scores before the
// first and after the last aligned 16 bytes go through workgroup 0.
constexpr int STREAM_U = 4;
constexpr int STREAM_BLOCKS = 512;   // two workgroups per compute unit (a histogram fills under half its LDS)
template <class F>
__device__ __forceinline__ void stream_scores(const float* __restrict__ scores, int64_t n, F&& f) {
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const int64_t head = min(n, (int64_t)((4 - ((reinterpret_cast<uintptr_t>(scores) >> 2) & 3)) & 3));
    const int64_t nv = (n - head) >> 2;                       // aligned 16-byte groups
    const f32x4* v = reinterpret_cast<const f32x4*>(scores + head);
    const int64_t per_round = (int64_t)gridDim.x * THREADS * STREAM_U;
    const int64_t mine = (int64_t)blockIdx.x * STREAM_U * THREADS + threadIdx.x;   // + u THREADS + round per_round
    f32x4 x[STREAM_U], nx[STREAM_U];
    if (nv > 0) {
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) x[u] = v[min(mine + u * THREADS, nv - 1)];
    }
    for (int64_t base = 0; base < nv; base += per_round) {
        if (base + per_round < nv) {
#pragma unroll
            for (int u = 0; u < STREAM_U; ++u) nx[u] = v[min(base + per_round + mine + u * THREADS, nv - 1)];
        }
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) {
            const int64_t vi = base + mine + u * THREADS;
#pragma unroll
            for (int e = 0; e < 4; ++e) f(head + 4 * vi + e, score_key(x[u][e]), vi < nv);
        }
#pragma unroll
        for (int u = 0; u < STREAM_U; ++u) x[u] = nx[u];
    }
    if (blockIdx.x == 0) {   // at most 3 + 3 scores
        const int64_t tail0 = head + 4 * nv, rest = head + (n - tail0);
        const int64_t i = (int64_t)threadIdx.x < head ? (int64_t)threadIdx.x : tail0 + ((int64_t)threadIdx.x - head);
        const bool valid = (int64_t)threadIdx.x < rest;
        f(i, valid ? score_key(scores[i]) : 0u, valid);
    }
}

// The next digit of the k-th largest key: the largest d whose suffix count over `hist` (the digit's histogram among
// the keys that match `before`) reaches before.remaining.  All THREADS threads of the workgroup call it and get the
// result; `lds` holds 20 words.  Thread t owns PER consecutive bins; suffix sums run from the last bin down.
template <int NB, int SHIFT>
__device__ __forceinline__ Pick pick_digit(const uint32_t* __restrict__ hist, Pick before, uint32_t* lds) {
    constexpr int PER = NB >= THREADS ? NB / THREADS : 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t c[PER], own = 0u;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        c[e] = (PER * tid + e < NB) ? hist[PER * tid + e] : 0u;
        own += c[e];
    }
    uint32_t suf = own;   // sum over threads >= t of this wave
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = (uint32_t)__shfl_down((int)suf, o);
        if (lane + o < 64) suf += t;
    }
    if (lane == 0) lds[wave] = suf;
    if (tid == 0) {   // (kept if no digit qualifies, which k <= n excludes)
        lds[16] = before.prefix;
        lds[17] = before.mask;
        lds[18] = before.remaining;
    }
    __syncthreads();
    for (int w2 = wave + 1; w2 < THREADS / 64; ++w2) suf += lds[w2];
    uint32_t above = suf - own;   // keys with a digit beyond this thread's bins
    if (suf >= before.remaining && above < before.remaining) {   // exactly one thread
#pragma unroll
        for (int e = PER - 1; e >= 0; --e) {
            if (above + c[e] >= before.remaining) {
                lds[16] = before.prefix | ((uint32_t)(PER * tid + e) << SHIFT);
                lds[17] = before.mask | ((uint32_t)(NB - 1) << SHIFT);
                lds[18] = before.remaining - above;
                break;
            }
            above += c[e];
        }
    }
    __syncthreads();
    return Pick{lds[16], lds[17], lds[18]};
}

// Histogram of this level's digit over the keys that match the digits fixed so far (which every workgroup derives
// from the histogram of the level before; workgroup 0 also records them).  LEVEL 1 also lists those keys' indices;
// LEVEL 2 walks that list when it is complete, else all scores, and clears the level-0 histogram for the next call.
// LEVEL 0 clears everything else the call uses (state, the other histograms, the status words up to w_cand).
template <int LEVEL>
__global__ __launch_bounds__(THREADS, 8) void select_hist_kernel(const float* __restrict__ scores, int64_t n, uint32_t k,
                                                                 uint32_t* __restrict__ ws, size_t w_cand, uint32_t cand_cap) {
    constexpr int NB = LEVEL == 2 ? 16 : BINS;
    constexpr int SHIFT = LEVEL == 0 ? SHIFT0 : (LEVEL == 1 ? SHIFT1 : SHIFT2);
    constexpr size_t W_HIST = LEVEL == 0 ? W_HIST0 : (LEVEL == 1 ? W_HIST1 : W_HIST2);
    __shared__ uint32_t hist[NB];
    __shared__ uint32_t wg_list[LEVEL == 1 ? WG_LIST : 1];
    __shared__ uint32_t wg_count, wg_base;
    __shared__ uint32_t pick_lds[20];
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    Pick fixed{0u, 0u, k};
    if (LEVEL == 1) fixed = pick_digit<BINS, SHIFT0>(ws + W_HIST0, fixed, pick_lds);
    if (LEVEL == 2) fixed = pick_digit<BINS, SHIFT1>(ws + W_HIST1, sp->pick0, pick_lds);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (LEVEL == 1) sp->pick0 = fixed;
        if (LEVEL == 2) sp->pick1 = fixed;
    }
    if (LEVEL == 2)   // every workgroup has read the level-0 histogram in the kernel before
        for (int i = blockIdx.x * THREADS + threadIdx.x; i < BINS; i += gridDim.x * THREADS) ws[W_HIST0 + i] = 0u;
    if (LEVEL == 0) {
        for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < w_cand; i += (size_t)gridDim.x * THREADS)
            if (i < W_HIST0 || i >= W_HIST1) ws[i] = 0u;
    }
    const uint32_t prefix = fixed.prefix, mask = fixed.mask;
    const uint32_t cand_count = LEVEL == 2 ? sp->cand_count : 0u;
    for (int i = threadIdx.x; i < NB; i += THREADS) hist[i] = 0u;
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
        for (int64_t j = (int64_t)blockIdx.x * THREADS + threadIdx.x; j < (int64_t)cand_count; j += (int64_t)gridDim.x * THREADS)
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
            for (uint32_t i = threadIdx.x; i < wg_count; i += THREADS)
                if (wg_base + i < cand_cap) ws[w_cand + wg_base + i] = wg_list[i];
    }
    for (int i = threadIdx.x; i < NB; i += THREADS) {
        const uint32_t c = hist[i];
        if (c != 0u) atomicAdd(&ws[W_HIST + i], c);
    }
}

// ---- last pass: threshold, count, scan over the tiles (decoupled look-back) and emit, in one kernel ----------------
// A tile's status word: bits 62..63 = 0 nothing yet / 1 the tile's own counts / 2 the counts of all tiles up to and
// including it; bits 31..61 = keys equal to the threshold; bits 0..30 = keys above it.  The word is the whole
// message (no other memory is exchanged between workgroups), so relaxed device-scope accesses suffice.  Tiles are
// numbered by a ticket taken when a workgroup starts: every tile with a lower number has then started too and
// publishes its own counts without waiting for anything, so every wait below ends.
constexpr uint64_t ST_OWN = 1ull << 62, ST_INCL = 2ull << 62;
__device__ __forceinline__ uint64_t st_pack(uint64_t flag, uint32_t gt, uint32_t eq) { return flag | ((uint64_t)eq << 31) | gt; }
__device__ __forceinline__ uint32_t st_gt(uint64_t st) { return (uint32_t)(st & 0x7FFFFFFFull); }
__device__ __forceinline__ uint32_t st_eq(uint64_t st) { return (uint32_t)((st >> 31) & 0x7FFFFFFFull); }
__device__ __forceinline__ uint64_t ld_status(const uint64_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_status(uint64_t* p, uint64_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

constexpr int LOOK_THREADS = 256;
// (Register budget of four waves per SIMD, i.e. one workgroup per CU: workgroups that all start together also all
// finish loading together and then all wait on each other's counts; with half of them resident at a time the second
// half loads while the first scans and writes: 37.5 -> 33.9 us at 2^24 scores.)
__global__ __launch_bounds__(THREADS, 4) void select_emit_kernel(const float* __restrict__ scores, int64_t n, int64_t k,
                                                                 int nq, uint32_t* __restrict__ ws,
                                                                 int32_t* __restrict__ out) {
    constexpr int SLOTS = 32;   // keys per thread; wave w owns keys [2048 w, 2048 (w + 1)) of the tile, slot j = 64 of them
    __shared__ uint32_t s_tile, s_gt[16], s_eq[16], s_lb_gt[16], s_lb_eq[16], s_lb_incl[16];
    __shared__ uint32_t pick_lds[20];
    State* sp = reinterpret_cast<State*>(ws + W_STATE);
    uint64_t* tile_word = reinterpret_cast<uint64_t*>(ws + W_STATUS);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_tile = atomicAdd(&sp->ticket, 1u);
    // the last digit completes the threshold key; `remaining` = keys equal to it that are still to be taken
    const Pick fin = pick_digit<16, SHIFT2>(ws + W_HIST2, sp->pick1, pick_lds);   // (its barriers also publish s_tile)
    const uint32_t thr = fin.prefix, need_eq = fin.remaining;
    const int64_t tile = s_tile;
    if (tile == 0)   // question tokens: positions n .. n + nq - 1 behind the k chosen ones
        for (int i = tid; i < nq; i += THREADS) out[k + i] = (int32_t)(n + i);
    // all loads in flight together, addressed as (tile base: uniform) + (32-bit offset in the tile); offsets clamped
    // to the last score
    const float* __restrict__ tile_scores = scores + tile * TILE;
    const uint32_t off0 = (uint32_t)(wave * (64 * SLOTS) + lane);
    const uint32_t last = (uint32_t)min((int64_t)TILE - 1, n - 1 - tile * TILE);
    const uint32_t tile_first = (uint32_t)(tile * TILE);   // this lane's keys: tile_first + off0 + 64 j
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
    uint32_t t_gt = 0u, t_eq = 0u;   // the tile's own counts
#pragma unroll
    for (int w2 = 0; w2 < 16; ++w2) { t_gt += s_gt[w2]; t_eq += s_eq[w2]; }
    if (tid == 0 && tile > 0) st_status(&tile_word[tile], st_pack(ST_OWN, t_gt, t_eq));
    // Look back, LOOK_THREADS tiles per step in one memory round trip: thread i examines tile hi - i (tiles below 0
    // count as "all before: nothing") and waits until that tile has published at least its own counts; each wave sums
    // its 64 tiles from the nearest up to its nearest tile that already knows its inclusive counts; the waves' sums are
    // then added from the nearest wave on, up to the first that met such a tile.  (The workgroups of a launch start
    // together, so mostly all words hold own counts at the first fetch.)
    uint32_t b_gt = 0u, b_eq = 0u;   // keys above / equal to the threshold in all tiles before this one
    for (int64_t hi = tile - 1; ; hi -= LOOK_THREADS) {
        if (tid < LOOK_THREADS) {
            const int64_t t = hi - tid;
            uint64_t st = ST_INCL;
            if (t >= 0) {
                st = ld_status(&tile_word[t]);
                while ((st >> 62) == 0ull) {
                    __builtin_amdgcn_s_sleep(1);
                    st = ld_status(&tile_word[t]);
                }
            }
            const uint64_t incl = __ballot((st >> 62) == 2ull);
            const int stop = incl ? (int)__builtin_ctzll(incl) : 63;   // lanes up to it contribute
            uint32_t g = lane <= stop ? st_gt(st) : 0u, e = lane <= stop ? st_eq(st) : 0u;
            for (int o = 32; o > 0; o >>= 1) {
                g += (uint32_t)__shfl_xor((int)g, o);
                e += (uint32_t)__shfl_xor((int)e, o);
            }
            if (lane == 0) { s_lb_gt[wave] = g; s_lb_eq[wave] = e; s_lb_incl[wave] = incl != 0ull ? 1u : 0u; }
        }
        __syncthreads();
        bool found = false;
        for (int w2 = 0; w2 < LOOK_THREADS / 64 && !found; ++w2) {
            b_gt += s_lb_gt[w2];
            b_eq += s_lb_eq[w2];
            found = s_lb_incl[w2] != 0u;
        }
        __syncthreads();   // (the next step writes these words again)
        if (found) break;
    }
    if (tid == 0) st_status(&tile_word[tile], st_pack(ST_INCL, b_gt + t_gt, b_eq + t_eq));
    uint32_t gt_seen = b_gt, eq_seen = b_eq;   // keys above / equal to the threshold before this wave's first key
    for (int w2 = 0; w2 < wave; ++w2) { gt_seen += s_gt[w2]; eq_seen += s_eq[w2]; }
    // key i is chosen if it lies above the threshold, or equals it and fewer than need_eq equal keys precede it; its
    // place is (keys above the threshold before i) + min(equal keys before i, need_eq)
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
        const bool gt = (gt_bits >> j) & 1u, eq = (eq_bits >> j) & 1u;
        const uint64_t bg = __ballot(gt), be = __ballot(eq);
        const uint32_t g_before = gt_seen + __builtin_amdgcn_mbcnt_hi((uint32_t)(bg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bg, 0u));
        const uint32_t e_before = eq_seen + __builtin_amdgcn_mbcnt_hi((uint32_t)(be >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)be, 0u));
        if (gt || (eq && e_before < need_eq)) out[g_before + min(e_before, need_eq)] = (int32_t)(tile_first + off0 + 64u * j);
        gt_seen += (uint32_t)__popcll(bg);
        eq_seen += (uint32_t)__popcll(be);
    }
}

}  // namespace

size_t select_workspace_bytes() { return select_workspace_words((int64_t)MAX_TILES * TILE) * sizeof(uint32_t); }
size_t select_zeroed_bytes() { return W_HIST1 * sizeof(uint32_t); }   // state and the first histogram

hipError_t launch_select_large(const float* scores, int64_t n, int64_t k, int nq, int32_t* q_index, uint32_t* ws,
                               size_t ws_bytes, hipStream_t st) {
    if (k <= 0 || n <= 0) {
        if (nq > 0) select_questions_kernel<<<dim3((nq + 255) / 256), dim3(256), 0, st>>>(n, k, nq, q_index);
        return hipGetLastError();
    }
    Layout lay;
    if (!make_layout(n, ws_bytes / sizeof(uint32_t), &lay)) return hipErrorInvalidValue;
    // (k == n needs no special case: the threshold is then the smallest key, and every key equal to it is needed)
    const int grid = (int)std::min<int64_t>(STREAM_BLOCKS, (n + 4 * THREADS - 1) / (4 * THREADS));
    const int grid2 = std::min(grid, 128);   // the last level normally walks a short list
    hipError_t e = hipSuccess;
    auto ok = [&]() { return e == hipSuccess && (e = hipGetLastError()) == hipSuccess; };
    select_hist_kernel<0><<<dim3(grid), dim3(THREADS), 0, st>>>(scores, n, (uint32_t)k, ws, lay.w_cand, lay.cand_cap);
    if (ok()) select_hist_kernel<1><<<dim3(grid), dim3(THREADS), 0, st>>>(scores, n, (uint32_t)k, ws, lay.w_cand, lay.cand_cap);
    if (ok()) select_hist_kernel<2><<<dim3(grid2), dim3(THREADS), 0, st>>>(scores, n, (uint32_t)k, ws, lay.w_cand, lay.cand_cap);
    if (ok()) select_emit_kernel<<<dim3((unsigned)lay.n_tiles), dim3(THREADS), 0, st>>>(scores, n, k, nq, ws, q_index);
    if (!ok()) {   // some kernel did not start: leave the scratch as a call expects it
        select_clear_kernel<<<dim3(64), dim3(256), 0, st>>>(ws, (int64_t)lay.w_cand);
        (void)hipGetLastError();
    }
    return e;
}

}  // namespace fr
