// Cross-lane helpers shared by the packing, backward and fused kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbmm {

constexpr int kDppQuadSwap1 = 0xB1;    // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;    // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each group of 8
constexpr int kDppRowMirror = 0x140;   // lane i <-> 15-i inside each group of 16

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over `LANES` consecutive lanes (a power of two, aligned); every lane gets the result.  The
// order of the additions is fixed (pairwise, nearest partner first), so every kernel that uses it
// produces the same fp32 value for the same inputs.
template <int LANES>
__device__ __forceinline__ float segment_sum(float v)
{
    if (LANES >= 2) v += dpp_f32<kDppQuadSwap1>(v);
    if (LANES >= 4) v += dpp_f32<kDppQuadSwap2>(v);
    if (LANES >= 8) v += dpp_f32<kDppHalfMirror>(v);
    if (LANES >= 16) v += dpp_f32<kDppRowMirror>(v);
    if (LANES >= 32) v += __shfl_xor(v, 16);
    if (LANES >= 64) v += __shfl_xor(v, 32);
    return v;
}

// The 4 sign bits of a lane's four elements, placed at nibble (lane mod 8) and OR-ed over the 8
// lanes that make up one 32-bit packed word; every one of those lanes gets the word.
__device__ __forceinline__ uint32_t pack_word_from_nibbles(uint32_t nib, int lane)
{
    uint32_t t = nib << (4 * (lane & 7));
    t |= dpp_u32<kDppQuadSwap1>(t);
    t |= dpp_u32<kDppQuadSwap2>(t);
    t |= dpp_u32<kDppHalfMirror>(t);
    return t;
}

}  // namespace hbmm
