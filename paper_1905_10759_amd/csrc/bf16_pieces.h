// An fp32 value as three bf16 pieces, the form in which the matrix-core kernels multiply fp32 operands
// exactly (shared by gemm_mfma_split.hip and conv_direct.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbmm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Exact split of an fp32 value into three bf16 patterns (each returned in the HIGH half of a word):
// hi = the top half of the fp32 pattern, mid = the top half of (v - hi), lo = v - hi - mid; 8 + 8 + 8
// significant bits, so hi + mid + lo == v.
__device__ __forceinline__ void split3(float v, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    hi = __builtin_bit_cast(uint32_t, v) & 0xffff0000u;
    const float r1 = v - __builtin_bit_cast(float, hi);
    mid = __builtin_bit_cast(uint32_t, r1) & 0xffff0000u;
    const float r2 = r1 - __builtin_bit_cast(float, mid);
    lo = __builtin_bit_cast(uint32_t, r2) & 0xffff0000u;
}
// Two high-half patterns -> one dword holding element a in the low half and element b in the high half.
__device__ __forceinline__ uint32_t pair16(uint32_t a_hi, uint32_t b_hi) { return (a_hi >> 16) | b_hi; }

// The six piece pairs (x piece, y piece) whose products are added when both operands are pieces, smallest
// contributions first: (hi,lo) (lo,hi) (mid,mid) (hi,mid) (mid,hi) (hi,hi).  The three that are dropped
// are below 2^-24 of a term.
constexpr int kPiecePairs[6][2] = {{0, 2}, {2, 0}, {1, 1}, {0, 1}, {1, 0}, {0, 0}};

}  // namespace hbmm
