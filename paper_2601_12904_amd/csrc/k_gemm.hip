// The model steps around the selective-prefill path for the recomputed rows (the per-layer work of the
// full-stack configuration): y = x W^T on the gfx950 matrix cores with fused epilogues, RMSNorm, and the
// rotary table of the rows' positions.
//
// GEMM.  out[M, N] = a[M, K] . w[N, K]^T, bf16 in, fp32 accumulate.  Both operands are K-contiguous, so the
// kernel computes the transposed tile C^T = W A^T with v_mfma_f32_32x32x16_bf16: output features run along the
// accumulator's register dimension and activation rows along lanes, which puts four consecutive features of one
// row into one lane -- rotary pairs and (gate, up) pairs are then combined without any lane exchange.
// One workgroup computes (64 WF) features x 128 rows with WF x 2 waves of 64 x 64 each: WF = 4 (8 waves, two per
// SIMD, so one wave's LDS reads and barriers hide behind the other's matrix instructions; 48 KB per K tile, ring
// of 3) where the feature count allows, else WF = 2 (4 waves, 32 KB per K tile, ring of 4).  K is walked in tiles
// of 64: both operand tiles (rows of 128 bytes) are copied straight into an LDS ring with direct-to-LDS loads
// (no staging registers); each lane chooses which 16-byte chunk of its row it fetches so that chunk c of row r
// lands at chunk position c ^ swz(r), swz(r) = (r ^ (r >> 3)) & 7: the 16-byte fragment reads (one lane per row)
// of any 16 consecutive rows then fall into 16 distinct bank groups.
#include "fr_internal.hpp"

#include <type_traits>

#include <algorithm>

namespace fr {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int BR = 128;   // activation rows per workgroup (MFMA N side)
constexpr int BK = 64;    // K elements per tile: 128 bytes per row
constexpr int EPI_PITCH = 64 + 4;                   // fp32 elements per row of a wave's epilogue staging

template <int WF>
struct Tiling {
    static constexpr int NW = 2 * WF;                    // waves per workgroup
    static constexpr int BF = 64 * WF;                   // output features per workgroup (MFMA M side)
    static constexpr int W_TILE_BYTES = BF * BK * 2;     // 16 or 32 KB
    static constexpr int A_TILE_BYTES = BR * BK * 2;     // 16 KB
    static constexpr int STAGE_BYTES = W_TILE_BYTES + A_TILE_BYTES;
    static constexpr int N_STAGE = (WF == 4) ? 3 : 4;
    static constexpr int W_ROUNDS = BF * 8 / (NW * 64);  // direct-to-LDS instructions per lane and W tile
    static constexpr int A_ROUNDS = BR * 8 / (NW * 64);
    static constexpr int LDS_BYTES = N_STAGE * STAGE_BYTES;
    static_assert(NW * 64 * EPI_PITCH * 4 <= LDS_BYTES, "epilogue staging must fit into the ring");
};

__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }

// Copy one operand tile (rows of 128 bytes) into LDS.  Chunk u (16 bytes) of the tile sits at byte 16 u; every wave
// moves 1 KB per round.  The per-lane part of a copy's source address does not change from K tile to K tile (which
// row, which 16-byte chunk of its 128 bytes: `lane_off`, set up once by dma_offsets; rows past the end of the operand
// are clamped and never stored), the rest is the same for the whole workgroup and travels in scalar registers, as
// does the LDS address: a copy costs the vector ALU nothing.
// (The copies are written out rather than left to the builtin: with it the compiler takes the pending copy for an
// access that may complete out of order with the LDS reads, and waits for all outstanding fragment reads before
// every matrix instruction.)
template <int ROUNDS, int NW>
__device__ __forceinline__ void dma_offsets(int64_t ld, int row0, int rows, int wave, int lane, uint32_t (&lane_off)[ROUNDS]) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        const int u = (j * NW + wave) * 64 + lane;
        const int r = u >> 3, cpos = u & 7;
        const int c = cpos ^ swz(r);
        // relative to the operand's row row0 and the current K tile; fits 32 bits: at most 256 rows of at most 2^22
        // elements (checked by the caller)
        lane_off[j] = (uint32_t)(((int64_t)(min(row0 + r, rows - 1) - row0) * ld + 8 * c) * 2);
    }
}
template <int ROUNDS, int NW>
__device__ __forceinline__ void dma_tile(const unsigned char* tile_src /* uniform: row row0, current K tile */,
                                         const uint32_t (&lane_off)[ROUNDS], uint32_t lds_tile /* uniform */, int wave_u) {
#pragma unroll
    for (int j = 0; j < ROUNDS; ++j) {
        const uint32_t l = lds_tile + (uint32_t)(j * NW + wave_u) * 1024u;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off[j]), "s"(tile_src), "s"(l) : "memory");
    }
}

// Workgroup barrier without the fences of __syncthreads(): those make the compiler wait for *all* outstanding
// memory operations (vmcnt(0)), which would drain the direct-to-LDS copies and register prefetches that are meant
// to stay in flight across the barrier.  The callers wait by hand for exactly the copies the next phase needs; the
// empty asm statements keep the compiler from moving LDS accesses across the barrier.
__device__ __forceinline__ void barrier_keep_loads_in_flight() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

enum { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_QKV_ROPE = 2, EPI_SWIGLU = 3 };

struct GemmArgs {
    const __bf16* a;        // [M, K]
    const __bf16* w;        // [N, K]
    int M, N, K;
    __bf16* out;            // EPI_STORE / EPI_RESIDUAL: [M, N];  EPI_SWIGLU: [M, N / 2]
    const __bf16* residual; // EPI_RESIDUAL: [M, N]
    // EPI_QKV_ROPE: features [0, Hq d) -> q_out[M, Hq, d] rotated, [Hq d, (Hq + Hkv) d) -> k_out rotated, rest -> v_out
    __bf16 *q_out, *k_out, *v_out;
    const float2* rope;     // [M][d / 2] (cos, sin) of each row's position
    int Hq, Hkv, d;
    // Tail split.  Tiles [0, n_whole) are computed by one workgroup each; every later tile by n_parts workgroups that
    // walk 1 / n_parts of K each and leave their fp32 accumulators in `partials` (gemm_fixup_kernel adds them and
    // runs the epilogue).  n_parts = 1: no tile is split.
    int n_whole, n_parts;
    float* partials;        // [(tile - n_whole) * n_parts + part][wave][64 registers][64 lanes]
    size_t partials_bytes;  // (host side: what the buffer holds)
};
constexpr int PARTIAL_FLOATS_PER_WAVE = 64 * 64;
constexpr int MIN_K_TILES_PER_PART = 16;

// Epilogue shared by the kernels: this wave's fp32 64 x 64 tile goes through LDS ([row][feature]), then every lane
// handles 8 consecutive features of a row.  fw0 / rw0 = first feature / row of the wave's tile.
template <int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, f32x16 (&acc)[2][2], unsigned char* smem, int wave, int lane,
                                              int fw0, int rw0) {
    const int x = lane & 31, h = lane >> 5;
    // ---- epilogue: fp32 tile through LDS ([row][feature] per wave), then 8 consecutive features per lane ----
    __syncthreads();
    float* ep = reinterpret_cast<float*>(smem) + wave * 64 * EPI_PITCH;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 t;
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = acc[mb][nb][4 * q4 + e];
                *reinterpret_cast<f32x4*>(&ep[(32 * nb + x) * EPI_PITCH + 32 * mb + 8 * q4 + 4 * h]) = t;
            }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rl = 8 * i + (lane >> 3), seg = lane & 7;     // local row, group of 8 features
        const int r = rw0 + rl;
        const int f = fw0 + 8 * seg;
        if (r >= g.M || f >= g.N) continue;
        float v[8];
        {
            const f32x4 lo = *reinterpret_cast<const f32x4*>(&ep[rl * EPI_PITCH + 8 * seg]);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(&ep[rl * EPI_PITCH + 8 * seg + 4]);
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
        }
        if (EPI == EPI_STORE || EPI == EPI_RESIDUAL) {
            if (EPI == EPI_RESIDUAL) {
                const bf16x8 res = *reinterpret_cast<const bf16x8*>(g.residual + (int64_t)r * g.N + f);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += (float)res[e];
            }
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
            *reinterpret_cast<bf16x8*>(g.out + (int64_t)r * g.N + f) = o;
        } else if (EPI == EPI_SWIGLU) {   // features interleaved (gate_j, up_j): out_j = silu(gate_j) * up_j
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float gt = v[2 * e], up = v[2 * e + 1];
                o[e] = (__bf16)(gt / (1.0f + __expf(-gt)) * up);
            }
            *reinterpret_cast<bf16x4*>(g.out + (int64_t)r * (g.N / 2) + f / 2) = o;
        } else {                          // EPI_QKV_ROPE
            const int qf_end = g.Hq * g.d, kf_end = qf_end + g.Hkv * g.d;
            __bf16* dst;
            bool rotate = true;
            if (f < qf_end) dst = g.q_out + (int64_t)r * qf_end + f;
            else if (f < kf_end) dst = g.k_out + (int64_t)r * (g.Hkv * g.d) + (f - qf_end);
            else { dst = g.v_out + (int64_t)r * (g.Hkv * g.d) + (f - kf_end); rotate = false; }
            if (rotate) {
                const int p0 = (f % g.d) >> 1;   // first rotary pair of this group (interleaved pairs)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float2 cs = g.rope[(int64_t)r * (g.d / 2) + p0 + e];
                    const float a = v[2 * e], b = v[2 * e + 1];
                    v[2 * e] = a * cs.x - b * cs.y;
                    v[2 * e + 1] = b * cs.x + a * cs.y;
                }
            }
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
            *reinterpret_cast<bf16x8*>(dst) = o;
        }
    }
}

template <int EPI, int WF>
__global__ __launch_bounds__(128 * WF) void gemm_bf16_kernel(GemmArgs g) {
    using TL = Tiling<WF>;
    constexpr int NW = TL::NW, BF = TL::BF, STAGE_BYTES = TL::STAGE_BYTES, N_STAGE = TL::N_STAGE;
    constexpr int DMA_PER_TILE = TL::W_ROUNDS + TL::A_ROUNDS;   // outstanding copies per lane and K tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wf = wave % WF, wr = wave / WF;          // wave position: features x rows
    // tile order: feature tiles fastest, so that workgroups that share an activation tile are neighbours
    const int n_ftiles = (g.N + BF - 1) / BF;
    int tile = (int)blockIdx.x, part = 0;
    if (tile >= g.n_whole) {
        const int j = tile - g.n_whole;
        tile = g.n_whole + j / g.n_parts;
        part = j % g.n_parts;
    }
    const bool split_tile = (int)blockIdx.x >= g.n_whole && g.n_parts > 1;
    const int f0 = (tile % n_ftiles) * BF, r0 = (tile / n_ftiles) * BR;
    const int n_kt_all = g.K / BK;
    const int kt_begin = split_tile ? (int)((int64_t)n_kt_all * part / g.n_parts) : 0;
    const int kt_end = split_tile ? (int)((int64_t)n_kt_all * (part + 1) / g.n_parts) : n_kt_all;
    const int n_kt = kt_end - kt_begin;   // K tiles of this workgroup: kt below counts from kt_begin

    // fragment byte offsets inside a tile: row (32 blk + x) of this wave's half, k step ks -> chunk (2 ks + h)
    int frag[4][2];   // [ks][blk & 1]
    {
        const int keyx = (x ^ (x >> 3)) & 7;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int par = 0; par < 2; ++par) frag[ks][par] = x * 128 + (((2 * ks + h) ^ keyx ^ (4 * par)) << 4);
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    uint32_t w_off[TL::W_ROUNDS], a_off[TL::A_ROUNDS];
    dma_offsets<TL::W_ROUNDS, NW>(g.K, f0, g.N, wave, lane, w_off);
    dma_offsets<TL::A_ROUNDS, NW>(g.K, r0, g.M, wave, lane, a_off);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem);
    const unsigned char* w_row0 = reinterpret_cast<const unsigned char*>(g.w + (int64_t)f0 * g.K);
    const unsigned char* a_row0 = reinterpret_cast<const unsigned char*>(g.a + (int64_t)r0 * g.K);
    auto issue = [&](int kt) {
        const uint32_t st = lds0 + (uint32_t)(kt % N_STAGE) * STAGE_BYTES;
        const int64_t k_bytes = (int64_t)(kt_begin + kt) * BK * 2;
        dma_tile<TL::W_ROUNDS, NW>(w_row0 + k_bytes, w_off, st, wave_u);
        dma_tile<TL::A_ROUNDS, NW>(a_row0 + k_bytes, a_off, st + TL::W_TILE_BYTES, wave_u);
    };
#pragma unroll
    for (int p = 0; p < N_STAGE - 1; ++p)
        if (p < n_kt) issue(p);

    // One K tile.  The ring slot is a compile-time constant (the loop below is unrolled by the ring's length) and the
    // LDS address of every fragment read sits in a register of its own, set up once (the ring is larger than the 64 KB
    // an instruction's offset field reaches, and the compiler, left to itself, adds the slot's offset before every
    // read): no address arithmetic between the matrix instructions.
    uint32_t rd_w[N_STAGE][4][2], rd_a[N_STAGE][4][2];   // [slot][k step][row block parity]
    {
        const uint32_t lds_v = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
#pragma unroll
        for (int sl = 0; sl < N_STAGE; ++sl)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int par = 0; par < 2; ++par) {
                    rd_w[sl][ks][par] = lds_v + sl * STAGE_BYTES + (64 * wf) * 128 + frag[ks][par];
                    rd_a[sl][ks][par] = lds_v + sl * STAGE_BYTES + TL::W_TILE_BYTES + (64 * wr) * 128 + frag[ks][par];
                    asm volatile("" : "+v"(rd_w[sl][ks][par]), "+v"(rd_a[sl][ks][par]));   // keep them: no re-derivation in the loop
                }
    }
    auto step = [&](auto slot_c, int kt) {
        constexpr int slot = decltype(slot_c)::value;
        // own copies of tile kt are the oldest outstanding: wait until at most the (N_STAGE - 2) newer tiles remain
        if (kt + N_STAGE - 2 < n_kt) {
            constexpr int newer = DMA_PER_TILE * (N_STAGE - 2);
            __builtin_amdgcn_s_waitcnt(0x0f70 | (newer & 15) | ((newer >> 4) << 14));
        } else {
            __builtin_amdgcn_s_waitcnt(0x0f70);
        }
        barrier_keep_loads_in_flight();   // tile kt complete and visible; everyone is done with tile kt-1, whose stage is refilled next
        // fragments of K step ks + 1 are requested before the matrix instructions of step ks are issued
        typedef const bf16x8 __attribute__((address_space(3))) * lds_frag_ptr;
        bf16x8 wfrag[2][2], afrag[2][2];
        auto request = [&](int ks, int buf) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                wfrag[buf][b] = *reinterpret_cast<lds_frag_ptr>((uintptr_t)(rd_w[slot][ks][b] + b * (32 * 128)));
                afrag[buf][b] = *reinterpret_cast<lds_frag_ptr>((uintptr_t)(rd_a[slot][ks][b] + b * (32 * 128)));
            }
        };
        request(0, 0);
        // the refill of the freed stage is issued behind the first fragment requests: its issue time passes while they
        // are on their way, instead of in front of them
        if (kt + N_STAGE - 1 < n_kt) issue(kt + N_STAGE - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + 1 < 4) request(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag[ks & 1][mb], afrag[ks & 1][nb], acc[mb][nb], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);   // LDS reads of step 0
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + 1 < 4) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);   // matrix
        }
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;
    int kt = 0;
    for (; kt + N_STAGE <= n_kt; kt += N_STAGE) {
        step(S0{}, kt);
        step(S1{}, kt + 1);
        step(S2{}, kt + 2);
        if constexpr (N_STAGE == 4) step(S3{}, kt + 3);
    }
    if (kt < n_kt) step(S0{}, kt);
    if (kt + 1 < n_kt) step(S1{}, kt + 1);
    if constexpr (N_STAGE == 4) {
        if (kt + 2 < n_kt) step(S2{}, kt + 2);
    }

    if (split_tile) {   // leave the partial sums: register-major, one coalesced 256-byte line per wave and register
        float* dst = g.partials + ((size_t)(((int)blockIdx.x - g.n_whole) * NW + wave)) * PARTIAL_FLOATS_PER_WAVE + lane;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[((2 * mb + nb) * 16 + v) * 64] = acc[mb][nb][v];
        return;
    }
    gemm_epilogue<EPI>(g, acc, smem, wave, lane, f0 + 64 * wf, r0 + 64 * wr);
}

// Adds the n_parts partial sums of every split tile and runs the epilogue on the result.  One wave per workgroup and
// grid.x = split tiles * NW: the work is a stream of partial sums, and with a 17 KB staging area instead of the
// ring's LDS many of these small workgroups share a CU and keep enough loads in flight.
template <int EPI, int WF>
__global__ __launch_bounds__(64) void gemm_fixup_kernel(GemmArgs g) {
    using TL = Tiling<WF>;
    constexpr int NW = TL::NW, BF = TL::BF;
    __shared__ __attribute__((aligned(16))) unsigned char smem[64 * EPI_PITCH * 4];
    const int lane = threadIdx.x;
    const int split = (int)blockIdx.x / NW, wave = (int)blockIdx.x % NW;
    const int wf = wave % WF, wr = wave / WF;
    const int n_ftiles = (g.N + BF - 1) / BF;
    const int tile = g.n_whole + split;
    const int f0 = (tile % n_ftiles) * BF, r0 = (tile / n_ftiles) * BR;
    f32x16 acc[2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    for (int p = 0; p < g.n_parts; ++p) {
        const float* src = g.partials + ((size_t)((split * g.n_parts + p) * NW + wave)) * PARTIAL_FLOATS_PER_WAVE + lane;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][nb][v] += src[((2 * mb + nb) * 16 + v) * 64];
    }
    gemm_epilogue<EPI>(g, acc, smem, /*staging slot*/ 0, lane, f0 + 64 * wf, r0 + 64 * wr);
}

// y = x * rsqrt(mean(x^2) + eps) * gain, one wave per row, fp32 statistics.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __bf16* __restrict__ x, const __bf16* __restrict__ gain, int R,
                                                      int hidden, float eps, __bf16* __restrict__ out) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= R) return;
    const __bf16* xr = x + (int64_t)row * hidden;
    float ss = 0.f;
    for (int c = lane * 8; c < hidden; c += 512) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += (float)v[e] * (float)v[e];
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float inv = 1.0f / sqrtf(ss / (float)hidden + eps);
    __bf16* orow = out + (int64_t)row * hidden;
    for (int c = lane * 8; c < hidden; c += 512) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
        const bf16x8 gn = *reinterpret_cast<const bf16x8*>(gain + c);
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)v[e] * inv * (float)gn[e]);
        *reinterpret_cast<bf16x8*>(orow + c) = o;
    }
}

// rope[r][p] = (cos, sin)(positions[r] * theta_p) in fp64, rounded once.
__global__ void rope_rows_table_kernel(const int32_t* __restrict__ positions, int R, int half_d, int d, double base,
                                       int index_base, float2* __restrict__ table) {
    const int r = blockIdx.x, p = threadIdx.x;
    if (r >= R || p >= half_d) return;
    const double theta = pow(base, -2.0 * (double)(p + index_base) / (double)d);
    double sn, cs;
    sincos((double)positions[r] * theta, &sn, &cs);
    table[(size_t)r * half_d + p] = make_float2((float)cs, (float)sn);
}

template <int EPI, int WF>
hipError_t launch_gemm_wf(GemmArgs g, const GemmTuning& tune, hipStream_t st) {
    using TL = Tiling<WF>;
    // once per process (a function-local static is initialised exactly once, also under concurrent first calls)
    struct Setup { hipError_t err; int n_cu; };
    static const Setup setup = [] {
        Setup r{hipSuccess, 0};
        r.err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<EPI, WF>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
        if (r.err != hipSuccess) return r;
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&r.n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || r.n_cu <= 0)
            r.err = hipErrorInvalidDevice;
        return r;
    }();
    if (setup.err != hipSuccess) return setup.err;
    const int n_cu = setup.n_cu;
    // One workgroup per CU at a time (the LDS ring fills it), so a launch runs in rounds of n_cu tiles and a last round
    // of `rest` tiles leaves CUs idle.  The tiles of that round are split along K over n_cu / rest workgroups each: the
    // round then takes 1 / n_parts of a tile's time, and the launch rest / n_cu rounds less.
    const int n_tiles = ((g.N + TL::BF - 1) / TL::BF) * ((g.M + BR - 1) / BR);
    const int rest = n_tiles % n_cu;
    int n_parts = (rest == 0 || tune.tail_split == 0) ? 1 : std::min(n_cu / rest, 8);
    // A part pays its own pipeline fill, a 128 KB dump of partial sums and its share of the second kernel (13 us for 128
    // tiles in two parts).  Measured at 2970 rows: K = 14336, 384 tiles, two parts of 112 K tiles: 9 % less time;
    // K = 4096, 576 tiles, four parts of 16: 8 % less; K = 4096, 384 tiles, two parts of 32: 4 % less; K = 4096,
    // 2688 tiles (a tenth of them in the last round): no change.
    n_parts = std::min(n_parts, (g.K / BK) / MIN_K_TILES_PER_PART);
    if (n_parts > 1 &&
        (g.partials == nullptr || (size_t)rest * n_parts * TL::NW * PARTIAL_FLOATS_PER_WAVE * sizeof(float) > g.partials_bytes))
        n_parts = 1;
    g.n_parts = std::max(n_parts, 1);
    g.n_whole = g.n_parts > 1 ? n_tiles - rest : n_tiles;
    const int grid = g.n_whole + (n_tiles - g.n_whole) * g.n_parts;
    gemm_bf16_kernel<EPI, WF><<<dim3(grid), dim3(64 * TL::NW), TL::LDS_BYTES, st>>>(g);
    if (g.n_parts > 1)
        gemm_fixup_kernel<EPI, WF><<<dim3((n_tiles - g.n_whole) * TL::NW), dim3(64), 0, st>>>(g);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_gemm(const GemmArgs& g, const GemmTuning& tune, hipStream_t st) {
    // (Feeding the weight fragments from memory straight into registers, to halve the LDS traffic, was tried: 16-byte
    // pieces of 32 rows per load instruction cost far more in the memory pipeline than they save: 400-500 TFLOP/s.)
    const bool wide = (tune.tile == 256) || (tune.tile == 0 && g.N % 256 == 0);
    return wide ? launch_gemm_wf<EPI, 4>(g, tune, st) : launch_gemm_wf<EPI, 2>(g, tune, st);
}

}  // namespace

size_t gemm_partials_bytes() { return (size_t)256 * 8 * PARTIAL_FLOATS_PER_WAVE * sizeof(float); }   // 256 parts of 8 waves

hipError_t launch_linear(const void* a, const void* w, int M, int N, int K, const void* residual, void* out,
                         float* partials, size_t partials_bytes, const GemmTuning& tune, hipStream_t st) {
    GemmArgs g{};
    g.partials = partials; g.partials_bytes = partials_bytes;
    g.a = (const __bf16*)a; g.w = (const __bf16*)w; g.M = M; g.N = N; g.K = K;
    g.out = (__bf16*)out; g.residual = (const __bf16*)residual;
    return residual ? launch_gemm<EPI_RESIDUAL>(g, tune, st) : launch_gemm<EPI_STORE>(g, tune, st);
}

hipError_t launch_linear_swiglu(const void* a, const void* w_gate_up, int M, int F, int K, void* out, float* partials,
                                size_t partials_bytes, const GemmTuning& tune, hipStream_t st) {
    GemmArgs g{};
    g.partials = partials; g.partials_bytes = partials_bytes;
    g.a = (const __bf16*)a; g.w = (const __bf16*)w_gate_up; g.M = M; g.N = 2 * F; g.K = K; g.out = (__bf16*)out;
    return launch_gemm<EPI_SWIGLU>(g, tune, st);
}

hipError_t launch_qkv_rope(const Shape& s, const void* a, const void* w_qkv, int M, int K, const int32_t* positions,
                           float2* rope_rows, void* q_out, void* k_out, void* v_out, float* partials,
                           size_t partials_bytes, const GemmTuning& tune, hipStream_t st) {
    rope_rows_table_kernel<<<dim3(M), dim3(64), 0, st>>>(positions, M, s.d / 2, s.d, s.rope_base, s.rope_index_base,
                                                          rope_rows);
    GemmArgs g{};
    g.partials = partials; g.partials_bytes = partials_bytes;
    g.a = (const __bf16*)a; g.w = (const __bf16*)w_qkv; g.M = M; g.N = (s.Hq + 2 * s.Hkv) * s.d; g.K = K;
    g.q_out = (__bf16*)q_out; g.k_out = (__bf16*)k_out; g.v_out = (__bf16*)v_out; g.rope = rope_rows;
    g.Hq = s.Hq; g.Hkv = s.Hkv; g.d = s.d;
    return launch_gemm<EPI_QKV_ROPE>(g, tune, st);
}

hipError_t launch_rmsnorm(const void* x, const void* gain, int R, int hidden, float eps, void* out, hipStream_t st) {
    if (R == 0) return hipSuccess;
    rmsnorm_kernel<<<dim3((R + 3) / 4), dim3(256), 0, st>>>((const __bf16*)x, (const __bf16*)gain, R, hidden, eps,
                                                           (__bf16*)out);
    return hipGetLastError();
}

}  // namespace fr
