// Binary-weight HBMM (beta_a = 1, the paper's HBWN): activations stay fp32, weights are
// delta_w (.) Sign(W).   C[m, n] = sum_j sB[n, j] * sum_{k in segment j} A[m, k] * (+-1)_B[n, k].
//
// Vector-ALU formulation.  A lane owns one weight row n (its packed word in a VGPR); a wave owns
// kRowsA activation rows whose values arrive through scalar loads and are used as the SGPR operand
// of v_fma_f32.  Per (lane, k) the sign bit is expanded once into +-1.0f (3 instructions) and
// shared by the kRowsA FMAs, so the cost is (1 + 3/kRowsA) instructions per multiply-add.  A
// product a * (+-1) is exact, so each segment sum is a plain fp32 running sum in ascending k; the
// first product of a segment starts the sum (no reset instruction) and the segment's scale is
// applied once, with one FMA, when the segment ends.
#include "kernels.h"

namespace hbmm {
namespace {

constexpr int kRowsA = 16;                  // activation rows per wave
constexpr int kWavesBW = 4;
constexpr int kTileM = kRowsA * kWavesBW;   // 64
constexpr int kTileN = 64;

typedef const float __attribute__((address_space(4))) *const_f32_ptr;

__global__ __launch_bounds__(64 * kWavesBW) void binary_weight_gemm_kernel(
    const float *__restrict__ A, int64_t lda, const uint32_t *__restrict__ b_bits,
    const float *__restrict__ b_scales, int64_t ldw_b, int64_t lds_b, int log2_words_per_seg, int M,
    int N, int K, float *__restrict__ C, int64_t ldc)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = blockIdx.x * kTileN + lane;
    const int m0 = blockIdx.y * kTileM + wave * kRowsA;
    const int nc = min(n, N - 1);
    const uint32_t *brow = b_bits + (int64_t)nc * ldw_b;
    const float *srow = b_scales + (int64_t)nc * lds_b;

    const_f32_ptr arow[kRowsA];
#pragma unroll
    for (int r = 0; r < kRowsA; ++r) arow[r] = (const_f32_ptr)(A + (int64_t)min(m0 + r, M - 1) * lda);

    float seg[kRowsA], res[kRowsA];
#pragma unroll
    for (int r = 0; r < kRowsA; ++r) { seg[r] = 0.f; res[r] = 0.f; }

    const int words = K >> 5;
    const int seg_mask = (1 << log2_words_per_seg) - 1;
    for (int w = 0; w < words; ++w) {
        const uint32_t inv = ~brow[w];
        const bool seg_start = (w & seg_mask) == 0;
        const bool seg_end = ((w + 1) & seg_mask) == 0;
#pragma unroll 4
        for (int b = 0; b < 32; ++b) {
            // bit 1 -> +1.0f, bit 0 -> -1.0f
            const float sgn = __builtin_bit_cast(float, 0x3f800000u | ((inv << (31 - b)) & 0x80000000u));
            const int k = w * 32 + b;
            if (seg_start && b == 0) {
#pragma unroll
                for (int r = 0; r < kRowsA; ++r) seg[r] = arow[r][k] * sgn;
            } else {
#pragma unroll
                for (int r = 0; r < kRowsA; ++r) seg[r] = __builtin_fmaf(arow[r][k], sgn, seg[r]);
            }
        }
        if (seg_end) {
            const float s = srow[w >> log2_words_per_seg];
#pragma unroll
            for (int r = 0; r < kRowsA; ++r) res[r] = __builtin_fmaf(s, seg[r], res[r]);
        }
    }
    if (n < N) {
#pragma unroll
        for (int r = 0; r < kRowsA; ++r)
            if (m0 + r < M) C[(int64_t)(m0 + r) * ldc + n] = res[r];
    }
}

}  // namespace

hipError_t launch_binary_weight_gemm(const float *A, int64_t lda, const uint32_t *b_bits,
                                     const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                     int64_t M, int64_t N, int64_t K, float *C, int64_t ldc,
                                     hipStream_t s)
{
    int lg = 0;
    while ((32 << lg) < beta_w) ++lg;
    dim3 grid((unsigned)((N + kTileN - 1) / kTileN), (unsigned)((M + kTileM - 1) / kTileM));
    if (grid.y > 65535u) return hipErrorInvalidConfiguration;
    binary_weight_gemm_kernel<<<grid, dim3(64 * kWavesBW), 0, s>>>(A, lda, b_bits, b_scales, ldw_b, lds_b, lg,
                                                                  (int)M, (int)N, (int)K, C, ldc);
    return hipGetLastError();
}

}  // namespace hbmm
