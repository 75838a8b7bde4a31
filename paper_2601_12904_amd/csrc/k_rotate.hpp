// Position shift of Appendix A applied to one 16-byte vector of a bf16 key on its way from a shared chunk store
// into a kernel (the store itself is never written): rotation of every (even, odd) or (p, p + d/2) pair by the
// chunk's angle, fp32 arithmetic, rounded to bf16 -- the same arithmetic as the stand-alone shift.  head_dim 128.
#pragma once

#include "fr_internal.hpp"

namespace fr {

typedef __attribute__((ext_vector_type(4))) uint32_t rot_u32x4;

template <int LAYOUT>
__device__ __forceinline__ rot_u32x4 rotate_key_vector(rot_u32x4 own, rot_u32x4 partner, const float2* __restrict__ trow, int st_vec) {
    // own = elements 8 st_vec .. + 7 of the head row.  Interleaved pairs: (2p, 2p + 1) inside the vector.
    // Half-split pairs: (p, p + 64): `partner` is the vector 64 elements away.
    rot_u32x4 outv;
    if (LAYOUT == FR_ROPE_INTERLEAVED) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = trow[4 * st_vec + e];
            const float a = __uint_as_float(own[e] << 16), b = __uint_as_float(own[e] & 0xFFFF0000u);
            const __bf16 ya = (__bf16)(a * t.x - b * t.y), yb = (__bf16)(b * t.x + a * t.y);
            outv[e] = (uint32_t)__builtin_bit_cast(unsigned short, ya) | ((uint32_t)__builtin_bit_cast(unsigned short, yb) << 16);
        }
    } else {
        const bool low = st_vec < 8;   // this vector holds the first elements of its pairs
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsigned short r2[2];
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const float2 t = trow[(8 * st_vec + 2 * e + hlf) & 63];
                const float mine = hlf ? __uint_as_float(own[e] & 0xFFFF0000u) : __uint_as_float(own[e] << 16);
                const float other = hlf ? __uint_as_float(partner[e] & 0xFFFF0000u) : __uint_as_float(partner[e] << 16);
                const float a = low ? mine : other, b = low ? other : mine;
                const __bf16 y = low ? (__bf16)(a * t.x - b * t.y) : (__bf16)(b * t.x + a * t.y);
                r2[hlf] = __builtin_bit_cast(unsigned short, y);
            }
            outv[e] = (uint32_t)r2[0] | ((uint32_t)r2[1] << 16);
        }
    }
    return outv;
}


}  // namespace fr
