// Query-Guided Selection, critical scores (Sec. 3.2) on the gfx950 matrix cores: bf16, head_dim 128.
//
// The score of context token j is the column sum, over all question rows and query heads, of the
// softmax-normalised attention weights.  A column sum needs every row's normaliser first, so the
// logits are formed twice (recomputing a 128-deep bf16 product is far cheaper than storing and
// re-reading nq x Hq x L_ctx fp32 values):
//   pass A  per (KV head, chunk, 256 query columns): S^T = K Q^T tile by tile, running max / sum per
//           query column -> base-2 log-sum-exp of the scaled logits, lse2[g][chunk][column] (rows padded to a
//           multiple of 64 columns, the padding +inf: pass B copies whole 64-column tiles and their weights are 0)
//   pass B  per (KV head, 256 keys of one chunk): S = Q K^T over all query columns of the group,
//           p = exp2(s * c - lse2), summed down the rows -> col_partial[g][key]
//   reduce  scores[j] = sum over KV heads g of col_partial[g][j], in a fixed order.
// A "query column" n of KV head g is the pair (question token i = n / G, query head g*G + n % G).
// Orientation is chosen so that each reduction runs inside a lane: pass A puts keys on the
// accumulator's register dimension and query columns on lanes; pass B the other way round.
// All sums run in a fixed order: the scores are reproducible bit for bit.
//
// Key source (template parameter SRC).  SRC_PROMPT: k holds the context keys at their prompt positions.  SRC_STORE_*:
// k is a chunk store shared between queries (Sec. 4.3); chunk c of the prompt occupies store rows row0[c] .., and its
// keys are moved to their prompt positions on the way into the kernel (Appendix A: rotation by the chunk's row of
// `table`, interleaved or half-split pairs), so the selection needs no per-query copy of the keys either.
#include "fr_internal.hpp"
#include "k_rotate.hpp"

#include <type_traits>

namespace fr {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int D = 128;
constexpr float NEG_BIG = -1.0e30f;
enum { SRC_PROMPT = 0, SRC_STORE_INTERLEAVED = 1, SRC_STORE_HALF = 2 };

// Row of `k` that holds prompt position j of chunk c (c0 = the chunk's first position).
template <int SRC>
__device__ __forceinline__ int64_t key_row(const ChunkRows& rows, int c, int c0, int j) {
    return SRC == SRC_PROMPT ? (int64_t)j : (int64_t)rows.row0[c] + (j - c0);
}
// 16-byte vector `vec` (8 elements) of one key row, moved to its prompt position where the source is a store.
template <int SRC>
__device__ __forceinline__ u32x4 load_key_vector(const __bf16* row, int vec, const float2* trow) {
    const u32x4 own = *reinterpret_cast<const u32x4*>(row + 8 * vec);
    if (SRC == SRC_PROMPT) return own;
    if (SRC == SRC_STORE_INTERLEAVED) return rotate_key_vector<FR_ROPE_INTERLEAVED>(own, own, trow, vec);
    const u32x4 partner = *reinterpret_cast<const u32x4*>(row + 8 * (vec ^ 8));
    return rotate_key_vector<FR_ROPE_HALF>(own, partner, trow, vec);
}

__device__ __forceinline__ bf16x8 zero8() {
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.0f;
    return z;
}

// Asks the scheduler to alternate matrix and transcendental instructions in the enclosing block, so that the
// products of one half tile are issued between the exponentials of the half before it.
__device__ __forceinline__ void interleave_hint() {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);   // two transcendental
    }
}

// ---- streamed tiles, copied global -> LDS directly -------------------------------------------------------------
// A streamed tile is 64 rows of 256 bytes, unpadded: row r at byte 256 r, its 16-byte chunk c in slot
// c ^ row_key(r).  The fragment reads (lane = row x of a 32-row half, chunk 2 ks + h) then hit 16 different slots in
// any 16 lanes that the LDS serves together, whether those are 16 rows of one h or 8 rows of both.
constexpr int TILE_BYTES = 64 * D * 2;
constexpr int NW = 4;                 // waves per workgroup: they share every streamed tile (8 was measured: half the
                                      // copies per wave and half the L2 traffic, same time; 4 wastes less on short chunks)
constexpr int COPIES = 16 / NW;       // 1 KB copies per wave and tile
__device__ __forceinline__ int row_key(int r) { return ((r & 7) << 1) | ((r >> 3) & 1); }

// Byte offsets, inside a 32-row half, of this lane's eight A fragments.
__device__ __forceinline__ void frag_offsets(int x, int h, uint32_t (&a_off)[8]) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) a_off[ks] = (uint32_t)(x * 256 + (((2 * ks + h) ^ row_key(x)) << 4));
}
__device__ __forceinline__ void load_frags(const unsigned char* tile, int mb, const uint32_t (&a_off)[8], bf16x8 (&a)[8]) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(tile + mb * (32 * 256) + a_off[ks]);
}
__device__ __forceinline__ void mfma_half(const bf16x8 (&a)[8], const bf16x8 (&bf)[2][8], f32x16 (&s)[2]) {
    f32x16 zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
            s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bf[nb][ks], ks == 0 ? zero : s[nb], 0, 0, 0);
}
// Which LDS row this lane fills in copy j of its wave (each copy: 1 KB = 4 rows, lane = (row, slot)), and which
// chunk of the source row belongs there.
__device__ __forceinline__ int copy_row(int j, int wave, int lane) { return 4 * (NW * j + wave) + (lane >> 4); }
__device__ __forceinline__ int copy_chunk(int j, int wave, int lane) { return (lane & 15) ^ row_key(copy_row(j, wave, lane)); }
// A workgroup-uniform address, pinned to scalar registers (the copies take their base address from there; without
// this the compiler may keep a pointer it also uses for vector loads in vector registers).
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}
// One tile, global -> LDS without passing through registers (global_load_lds_dwordx4: lane i of a wave deposits its
// 16 bytes at the LDS address in M0 + 16 i).  The source is a workgroup-uniform base in scalar registers plus a
// 32-bit per-lane offset, so a copy costs the vector ALU nothing.  Written out rather than left to the builtin: with
// it the compiler takes the pending copy for an access that may complete out of order with the LDS reads and waits
// for all outstanding fragment reads before every matrix instruction.  Completion: the issuing wave's vmcnt, then
// a workgroup barrier.
__device__ __forceinline__ void dma_tile(const unsigned char* src, const uint32_t (&lane_off)[COPIES], uint32_t lds_tile, int wave_u) {
    src = uniform_ptr(src);
#pragma unroll
    for (int j = 0; j < COPIES; ++j) {
        const uint32_t l = lds_tile + (uint32_t)(NW * j + wave_u) * 1024u;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off[j]), "s"(src), "s"(l) : "memory");
    }
}
// 64 floats (one per lane) global -> LDS the same way.
__device__ __forceinline__ void dma_floats(const float* src, uint32_t lane_off, uint32_t lds_dst) {
    src = uniform_ptr(src);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" : : "v"(lane_off), "s"(src), "s"(lds_dst) : "memory");
}
// Top of a step: this wave's copies have landed and its LDS reads have returned (vmcnt(0), lgkmcnt(0)); after the
// barrier that follows, the slot that is overwritten next has no reader left anywhere in the workgroup.  (The reads
// still outstanding here are the fragments requested at the end of the step before, which the first matrix
// instruction after the barrier needs at once: waiting for them here costs nothing measurable.)
__device__ __forceinline__ void wait_copies_and_reads() { __builtin_amdgcn_s_waitcnt(0x0070); }
// Workgroup barrier without the fences of __syncthreads() (which add nothing here: the waits are explicit); the
// empty asm statements keep the compiler from moving LDS accesses across it.
__device__ __forceinline__ void plain_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p);
}

// ---- pass A -------------------------------------------------------------------------------------
// One workgroup = (KV head, chunk, 256 query columns).  1-D grid with the KV head as the fastest index:
// consecutive workgroups land on different XCDs, so all query-column tiles of one (head, chunk) share one L2.
// A wave keeps its 64 query columns in registers (B operand); the chunk's key tiles stream past them through a
// ring of three LDS slots.  Step t (one workgroup barrier) multiplies keys 32..63 of tile t while the exponentials
// of keys 0..31 run, then keys 0..31 of tile t + 1 against the exponentials of keys 32..63, and fills the slot
// tile t - 1 has left with tile t + 2: copied global -> LDS directly where the keys are used as stored
// (SRC_PROMPT), through registers where they are rotated on the way (chunk store).  Every lane keeps a running
// maximum and sum over the keys it sees itself (one of the two 4-row groups in every 8 keys); the two lanes of a
// query column are merged once at the end.
template <int G, int SRC>
__global__ __launch_bounds__(64 * NW, 8 / NW) void score_lse_mfma_kernel(const __bf16* __restrict__ q,
                                                                const __bf16* __restrict__ k, ChunkTable ct, int nq,
                                                                int Hq, int Hkv, int n_qtiles, float scale_log2e,
                                                                float* __restrict__ lse2, ChunkRows rows,
                                                                const float2* __restrict__ table) {
    constexpr bool DIRECT = (SRC == SRC_PROMPT);
    __shared__ __attribute__((aligned(1024))) unsigned char k_lds[3 * TILE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x % Hkv;
    const int qtile = (blockIdx.x / Hkv) % n_qtiles;
    const int c = blockIdx.x / (Hkv * n_qtiles);
    const int c0 = ct.off[c], c1 = ct.off[c + 1];
    const int NQG = nq * G, NQG_pad = (NQG + 63) & ~63;
    const int n_base = (qtile * NW + wave) * 64;
    const float2* trow = SRC == SRC_PROMPT ? nullptr : table + (size_t)c * (D / 2);

    bf16x8 qf[2][8];
    int col_n[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int n = n_base + 32 * nb + x;
        col_n[nb] = n;
        const int nc = min(n, NQG - 1);   // columns past the end copy the last one and are never stored
        const __bf16* qp = q + ((size_t)(nc / G) * Hq + g * G + (nc % G)) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }
    float m2[2] = {NEG_BIG, NEG_BIG}, lsum[2] = {0.f, 0.f};
    const int n_kt = (c1 - c0 + 63) / 64;
    if (n_kt == 0) {   // an empty chunk: no key, the log-sum-exp of nothing
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
            if (h == 0 && col_n[nb] < NQG_pad)
                lse2[((size_t)g * (ct.n + 1) + c) * NQG_pad + col_n[nb]] = col_n[nb] >= NQG ? INFINITY : -INFINITY;
        return;
    }
    uint32_t a_off[8];
    frag_offsets(x, h, a_off);
    // DIRECT: key row j of the chunk starts at byte j Hkv 256 of the head's slice; the per-lane part of a copy's
    // address is the same for every tile but the last, whose rows past the chunk's end repeat its last key.
    const unsigned char* k_head = reinterpret_cast<const unsigned char*>(k + ((size_t)c0 * Hkv + g) * D);
    const size_t tile_stride = (size_t)64 * Hkv * D * 2;
    uint32_t off_full[COPIES], off_last[COPIES];
#pragma unroll
    for (int j = 0; j < COPIES; ++j) {
        const int r = copy_row(j, wave, lane), ch = copy_chunk(j, wave, lane);
        const int rl = min(64 * (n_kt - 1) + r, c1 - c0 - 1) - 64 * (n_kt - 1);
        off_full[j] = (uint32_t)(r * Hkv * (D * 2) + 16 * ch);
        off_last[j] = (uint32_t)(rl * Hkv * (D * 2) + 16 * ch);
    }
    const uint32_t lds_k = lds_address(k_lds);
    auto copy_tile = [&](int t, int slot) {
        uint32_t off[COPIES];
#pragma unroll
        for (int j = 0; j < COPIES; ++j) off[j] = (t == n_kt - 1) ? off_last[j] : off_full[j];
        dma_tile(k_head + (size_t)t * tile_stride, off, lds_k + (uint32_t)slot * TILE_BYTES, wave);
    };
    // chunk store: a tile waits in registers for one step (its rows rotated as they arrive), then goes to its slot
    const int st_vec = tid & 15, st_key = tid >> 4;   // 4 NW rows per round of the workgroup
    u32x4 kreg[COPIES];
    auto load_tile = [&](int t) {   // tiles past the last one re-read it; keys past the chunk's end are clamped
        t = min(t, n_kt - 1);
#pragma unroll
        for (int i = 0; i < COPIES; ++i) {
            const int j = min(c0 + t * 64 + st_key + 4 * NW * i, c1 - 1);
            kreg[i] = load_key_vector<SRC>(k + ((size_t)key_row<SRC>(rows, c, c0, j) * Hkv + g) * D, st_vec, trow);
        }
    };
    auto write_tile = [&](int slot) {
#pragma unroll
        for (int i = 0; i < COPIES; ++i) {
            const int r = st_key + 4 * NW * i;
            *reinterpret_cast<u32x4*>(k_lds + slot * TILE_BYTES + r * 256 + ((st_vec ^ row_key(r)) << 4)) = kreg[i];
        }
    };
    // running log-sum-exp of one half: rows (keys) key_lo + 8 (v / 4) + 4 h + v % 4 of the accumulator
    auto fold_half = [&](auto ragged, f32x16 (&s)[2], int key_lo) {
        if constexpr (decltype(ragged)::value) {   // last tile of the chunk: keys past its end do not count
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (key_lo + 8 * (v >> 2) + 4 * h + (v & 3) >= c1) s[nb][v] = -INFINITY;
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            float mx = NEG_BIG;
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[nb][v]);
            const float m_new = fmaxf(m2[nb], mx * scale_log2e);
            float psum = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[nb][v], scale_log2e, -m_new));
            lsum[nb] = lsum[nb] * __builtin_amdgcn_exp2f(m2[nb] - m_new) + psum;
            m2[nb] = m_new;
        }
    };
    f32x16 s_a[2], s_b[2];
    bf16x8 fa[8];   // fragments of keys 32..63 of the step's tile; DIRECT: requested a step ahead
    auto step = [&](auto slot_c, auto ragged, int t) {
        constexpr int b = decltype(slot_c)::value, b1 = (b + 1) % 3, b2 = (b + 2) % 3;   // slots of tiles t, t + 1, t + 2
        wait_copies_and_reads();
        plain_barrier();   // tile t + 1 is complete; every wave is done with tile t - 1
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (DIRECT) {
            copy_tile(min(t + 2, n_kt - 1), b2);   // past the last tile: once more the last one, into a slot nobody reads
        } else {
            write_tile(b2);      // tile t + 2, loaded a step ago
            load_tile(t + 3);
            load_frags(k_lds + b * TILE_BYTES, 1, a_off, fa);   // (no registers to spare for requesting these a step ahead)
        }
        mfma_half(fa, qf, s_b);
        fold_half(ragged, s_a, c0 + 64 * t);
        interleave_hint();
        bf16x8 fb[8];
        load_frags(k_lds + b1 * TILE_BYTES, 0, a_off, fb);   // past the last tile: a stale slot, the products are dropped
        mfma_half(fb, qf, s_a);
        fold_half(ragged, s_b, c0 + 64 * t + 32);
        interleave_hint();
        if constexpr (DIRECT) load_frags(k_lds + b1 * TILE_BYTES, 1, a_off, fa);
    };
    if constexpr (DIRECT) {
        copy_tile(0, 0);
        copy_tile(min(1, n_kt - 1), 1);
    } else {
        load_tile(0);
        write_tile(0);
        load_tile(1);
        write_tile(1);
        load_tile(2);
    }
    __builtin_amdgcn_s_waitcnt(DIRECT ? 0x0f70 : 0xc07f);   // the copies (vmcnt(0)) or the LDS writes (lgkmcnt(0)) are done
    plain_barrier();
    {
        bf16x8 fb[8];
        load_frags(k_lds, 0, a_off, fb);
        mfma_half(fb, qf, s_a);
        if constexpr (DIRECT) load_frags(k_lds, 1, a_off, fa);
    }
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    int t = 0;
    for (; t + 3 < n_kt; t += 3) {   // whole tiles only: at least one step is left for the ragged end
        step(S0{}, std::false_type{}, t);
        step(S1{}, std::false_type{}, t + 1);
        step(S2{}, std::false_type{}, t + 2);
    }
    const int left = n_kt - t;   // 1, 2 or 3 steps; the last one masks the keys past the chunk's end
    if (left == 1) {
        step(S0{}, std::true_type{}, t);
    } else if (left == 2) {
        step(S0{}, std::false_type{}, t);
        step(S1{}, std::true_type{}, t + 1);
    } else {
        step(S0{}, std::false_type{}, t);
        step(S1{}, std::false_type{}, t + 1);
        step(S2{}, std::true_type{}, t + 2);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {   // merge the two lanes of a query column
        const float m_o = __shfl_xor(m2[nb], 32), l_o = __shfl_xor(lsum[nb], 32);
        const float m = fmaxf(m2[nb], m_o);
        const float l = lsum[nb] * __builtin_amdgcn_exp2f(m2[nb] - m) + l_o * __builtin_amdgcn_exp2f(m_o - m);
        // columns NQG .. NQG_pad - 1 hold +inf: pass B copies whole 64-column tiles and their weights must be 0
        if (h == 0 && col_n[nb] < NQG_pad)
            lse2[((size_t)g * (ct.n + 1) + c) * NQG_pad + col_n[nb]] =
                col_n[nb] >= NQG ? INFINITY : (l > 0.f) ? m + __builtin_amdgcn_logf(l) : -INFINITY;
    }
}

// Global scope: lse2[g][C][n] = base-2 log-sum-exp over the chunks.  grid (NQG_pad / 256 rounded up, Hkv); rows of
// NQG_pad columns, the padding +inf.
__global__ void score_lse2_global_kernel(int n_chunks, int NQG, int NQG_pad, float* __restrict__ lse2) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= NQG_pad) return;
    float* base = lse2 + (size_t)blockIdx.y * (n_chunks + 1) * NQG_pad;
    if (n >= NQG) {
        base[(size_t)n_chunks * NQG_pad + n] = INFINITY;
        return;
    }
    float m = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) m = fmaxf(m, base[(size_t)c * NQG_pad + n]);
    float l = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float v = base[(size_t)c * NQG_pad + n];
        if (v != -INFINITY) l += exp2f(v - m);
    }
    base[(size_t)n_chunks * NQG_pad + n] = m + log2f(l);
}

// ---- pass B -------------------------------------------------------------------------------------
// One workgroup = (KV head, chunk, 256 keys of the chunk), KV head fastest in the 1-D grid (see pass A); a wave
// keeps its 64 keys in registers (B operand) and all query columns of the group stream past them.
// scope_global: use lse2[g][C].  The query-column tiles (64 columns with their normalisers) go global -> LDS
// directly into a ring of three; step t (one workgroup barrier) multiplies rows 32..63 of tile t while the
// weights of rows 0..31 are formed, then rows 0..31 of tile t + 1 against the weights of rows 32..63, and copies
// tile t + 2 into the slot tile t - 1 has left.  A tile lands a whole step before it is read; the fragments of the
// next step's first half are requested at the end of a step, so that they arrive while the wave waits at the barrier.
template <int G, int SRC>
__global__ __launch_bounds__(64 * NW, 8 / NW) void score_colsum_mfma_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                                                                ChunkTable ct, int nq, int Hq, int Hkv, int n_ktiles,
                                                                float scale_log2e, int scope_global,
                                                                const float* __restrict__ lse2,
                                                                float* __restrict__ col_partial, ChunkRows rows,
                                                                const float2* __restrict__ table) {
    __shared__ __attribute__((aligned(1024))) unsigned char q_lds[3 * TILE_BYTES];
    __shared__ __attribute__((aligned(256))) float lse_lds[3][64];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = blockIdx.x % Hkv;
    const int ktile = (blockIdx.x / Hkv) % n_ktiles;
    const int c = blockIdx.x / (Hkv * n_ktiles);
    const int c0 = ct.off[c], c1 = ct.off[c + 1];
    const int kbase = c0 + ktile * (64 * NW);
    if (kbase >= c1) return;
    const int NQG = nq * G, NQG_pad = (NQG + 63) & ~63;
    const int L_ctx = ct.off[ct.n];
    const float* lrow = lse2 + ((size_t)g * (ct.n + 1) + (scope_global ? ct.n : c)) * NQG_pad;

    bf16x8 kf[2][8];   // B operand: this wave's 64 keys
    int col_key[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int j = kbase + 64 * wave + 32 * nb + x;
        col_key[nb] = j;
        // keys past the end: copy, never stored
        const __bf16* kp = k + ((size_t)key_row<SRC>(rows, c, c0, min(j, c1 - 1)) * Hkv + g) * D;
        const float2* trow = SRC == SRC_PROMPT ? nullptr : table + (size_t)c * (D / 2);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            kf[nb][ks] = __builtin_bit_cast(bf16x8, load_key_vector<SRC>(kp, 2 * ks + h, trow));
    }
    float csum[2] = {0.f, 0.f};
    const int n_qt = NQG_pad / 64;
    // Query column n of the group = (question token n / G, head g G + n % G): tile t starts at token 64 t / G, and
    // the per-lane part of a copy's address is the same for every tile but the last, whose rows past the end
    // repeat the last column (finite numbers; their normaliser is +inf).
    const unsigned char* q_head = reinterpret_cast<const unsigned char*>(q + (size_t)g * G * D);
    const size_t tile_stride = (size_t)(64 / G) * Hq * D * 2;
    uint32_t off_full[COPIES], off_last[COPIES], a_off[8];
#pragma unroll
    for (int j = 0; j < COPIES; ++j) {
        const int r = copy_row(j, wave, lane), ch = copy_chunk(j, wave, lane);
        const int rl = min(64 * (n_qt - 1) + r, NQG - 1) - 64 * (n_qt - 1);
        off_full[j] = (uint32_t)(((r / G) * Hq + (r % G)) * (D * 2) + 16 * ch);
        off_last[j] = (uint32_t)(((rl / G) * Hq + (rl % G)) * (D * 2) + 16 * ch);
    }
    frag_offsets(x, h, a_off);
    const uint32_t lds_q = lds_address(q_lds), lds_l = lds_address(lse_lds);
    auto copy_tile = [&](int t, int slot) {
        uint32_t off[COPIES];
#pragma unroll
        for (int j = 0; j < COPIES; ++j) off[j] = (t == n_qt - 1) ? off_last[j] : off_full[j];
        dma_tile(q_head + (size_t)t * tile_stride, off, lds_q + (uint32_t)slot * TILE_BYTES, wave);
        // (every wave copies the tile's 64 normalisers, the same values to the same place: no branch in the step)
        dma_floats(lrow + 64 * t, (uint32_t)lane * 4u, lds_l + (uint32_t)slot * 256u);
    };
    // weights of one half (32 query rows), summed down the rows into the lane's key columns
    auto fold_half = [&](const f32x16 (&s)[2], int slot, int mb) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 lz = *reinterpret_cast<const f32x4*>(&lse_lds[slot][32 * mb + 8 * q4 + 4 * h]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    csum[nb] += __builtin_amdgcn_exp2f(__builtin_fmaf(s[nb][4 * q4 + e], scale_log2e, -lz[e]));
        }
    };
    f32x16 s_a[2], s_b[2];
    bf16x8 fa[8];   // fragments of rows 32..63 of the step's tile, requested a step ahead
    auto step = [&](auto slot_c, int t) {
        constexpr int b = decltype(slot_c)::value, b1 = (b + 1) % 3, b2 = (b + 2) % 3;   // slots of tiles t, t + 1, t + 2
        wait_copies_and_reads();
        plain_barrier();   // tile t + 1 is complete; every wave is done with tile t - 1
        __builtin_amdgcn_sched_barrier(0);
        copy_tile(min(t + 2, n_qt - 1), b2);   // past the last tile: once more the last one, into a slot nobody reads
        mfma_half(fa, kf, s_b);
        fold_half(s_a, b, 0);
        interleave_hint();
        bf16x8 fb[8];
        load_frags(q_lds + b1 * TILE_BYTES, 0, a_off, fb);   // past the last tile: a stale slot, the products are dropped
        mfma_half(fb, kf, s_a);
        fold_half(s_b, b, 1);
        interleave_hint();
        load_frags(q_lds + b1 * TILE_BYTES, 1, a_off, fa);
    };
    copy_tile(0, 0);
    if (n_qt > 1) copy_tile(1, 1);
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
    plain_barrier();
    {
        bf16x8 fb[8];
        load_frags(q_lds, 0, a_off, fb);
        mfma_half(fb, kf, s_a);
        load_frags(q_lds, 1, a_off, fa);
    }
    int t = 0;
    for (; t + 3 <= n_qt; t += 3) {
        step(std::integral_constant<int, 0>{}, t);
        step(std::integral_constant<int, 1>{}, t + 1);
        step(std::integral_constant<int, 2>{}, t + 2);
    }
    if (t < n_qt) step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < n_qt) step(std::integral_constant<int, 1>{}, t + 1);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float tot = csum[nb] + __shfl_xor(csum[nb], 32);
        if (h == 0 && col_key[nb] < c1) col_partial[(size_t)g * L_ctx + col_key[nb]] = tot;
    }
}

__global__ void score_reduce_heads_kernel(const float* __restrict__ col_partial, int L_ctx, int Hkv,
                                          float* __restrict__ scores) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= L_ctx) return;
    float t = 0.f;
    for (int g = 0; g < Hkv; ++g) t += col_partial[(size_t)g * L_ctx + j];
    scores[j] = t;
}

template <int G, int SRC>
hipError_t run(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct, int norm,
               const Workspace& ws, float* scores, const ChunkRows& rows, const float2* table, hipStream_t st) {
    const int L_ctx = ct.off[ct.n];
    const float c = (1.0f / sqrtf((float)s.d)) * 1.4426950408889634f;
    const int NQG = nq * G;
    int max_len = 0;
    for (int i = 0; i < ct.n; ++i) max_len = ct.off[i + 1] - ct.off[i] > max_len ? ct.off[i + 1] - ct.off[i] : max_len;
    const int n_qtiles = (NQG + 64 * NW - 1) / (64 * NW), n_ktiles = (max_len + 64 * NW - 1) / (64 * NW);
    score_lse_mfma_kernel<G, SRC><<<dim3(n_qtiles * ct.n * s.Hkv), dim3(64 * NW), 0, st>>>(
        (const __bf16*)q, (const __bf16*)k_ctx, ct, nq, s.Hq, s.Hkv, n_qtiles, c, ws.lse, rows, table);
    if (norm == FR_NORM_GLOBAL)
        score_lse2_global_kernel<<<dim3((NQG + 255) / 256, s.Hkv), dim3(256), 0, st>>>(ct.n, NQG, (NQG + 63) & ~63, ws.lse);
    score_colsum_mfma_kernel<G, SRC><<<dim3(n_ktiles * ct.n * s.Hkv), dim3(64 * NW), 0, st>>>(
        (const __bf16*)q, (const __bf16*)k_ctx, ct, nq, s.Hq, s.Hkv, n_ktiles, c, norm == FR_NORM_GLOBAL ? 1 : 0,
        ws.lse, ws.col_partial, rows, table);
    score_reduce_heads_kernel<<<dim3((L_ctx + 255) / 256), dim3(256), 0, st>>>(ws.col_partial, L_ctx, s.Hkv, scores);
    return hipGetLastError();
}

template <int SRC>
hipError_t dispatch(const Shape& s, const void* q, int nq, const void* k, const ChunkTable& ct, int norm,
                    const Workspace& ws, float* scores, const ChunkRows& rows, const float2* table, hipStream_t st) {
    if (ct.off[ct.n] == 0 || nq == 0) return hipSuccess;
    switch (s.G) {
        case 1: return run<1, SRC>(s, q, nq, k, ct, norm, ws, scores, rows, table, st);
        case 2: return run<2, SRC>(s, q, nq, k, ct, norm, ws, scores, rows, table, st);
        case 4: return run<4, SRC>(s, q, nq, k, ct, norm, ws, scores, rows, table, st);
        default: return run<8, SRC>(s, q, nq, k, ct, norm, ws, scores, rows, table, st);
    }
}

}  // namespace

bool score_mfma_supported(const Shape& s) {
    return s.dtype == FR_BF16 && s.d == 128 && (s.G == 1 || s.G == 2 || s.G == 4 || s.G == 8);
}

// Softmax scopes only; the caller routes FR_NORM_RAW to the generic kernels.
hipError_t launch_score_mfma(const Shape& s, const void* q, int nq, const void* k_ctx, const ChunkTable& ct, int norm,
                             const Workspace& ws, float* scores, hipStream_t st) {
    const ChunkRows none{};
    return dispatch<SRC_PROMPT>(s, q, nq, k_ctx, ct, norm, ws, scores, none, nullptr, st);
}

// The same over a shared chunk store: store_row0 (host) gives every chunk's first store row, `table` (device,
// [chunks][d / 2]) the (cos, sin) of every chunk's position shift.
hipError_t launch_score_mfma_shared(const Shape& s, const void* q, int nq, const void* k_store, const ChunkTable& ct,
                                    const int32_t* store_row0, const float2* table, int norm, const Workspace& ws,
                                    float* scores, hipStream_t st) {
    ChunkRows rows{};
    for (int c = 0; c < ct.n; ++c) rows.row0[c] = store_row0[c];
    if (s.rope_layout == FR_ROPE_INTERLEAVED)
        return dispatch<SRC_STORE_INTERLEAVED>(s, q, nq, k_store, ct, norm, ws, scores, rows, table, st);
    return dispatch<SRC_STORE_HALF>(s, q, nq, k_store, ct, norm, ws, scores, rows, table, st);
}

}  // namespace fr
