// Dense comparison GEMM on unquantised operands: C = A . B^T, A M x K, B N x K, both K contiguous,
// fp32 accumulate and fp32 C.  It plays the role of the full-precision matrix multiply that section
// 4.2 times its kernel against; it is not part of the HBMM path.
//
// Matrix-core kernel for gfx950.  A workgroup of 4 waves owns a 128 x 128 tile of C; K is walked in
// stages of 128 bytes per operand row, staged through LDS (row stride padded by 16 bytes so that
// the 16-byte fragment reads of 8 consecutive rows fall on distinct banks).  Each wave owns a
// 64 x 64 quadrant = 2 x 2 MFMA tiles of 32 x 32:
//   bf16:  v_mfma_f32_32x32x16_bf16, lane l feeds row (l mod 32), 8 consecutive k at 8 * (l div 32);
//   fp32:  v_mfma_f32_32x32x2_f32,   lane l feeds row (l mod 32), k = l div 32.
// Both operands use the same lane -> k map, so the products pair up whatever order the hardware
// walks k in.  Accumulator element v of lane l is C[8 * (v div 4) + 4 * (l div 32) + v mod 4][l mod 32]
// of the 32 x 32 tile.  The next stage is fetched from global memory into registers while the
// current one is multiplied, then parked in the other LDS buffer (one barrier per stage).
#include "kernels.h"

namespace hbmm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 128, kBN = 128;
constexpr int kStageBytes = 128;                 // per operand row per stage
constexpr int kRowStride = kStageBytes + 16;     // LDS row stride in bytes
constexpr int kThreadsD = 256;

template <typename T>
struct Traits;
template <>
struct Traits<__bf16> {
    static constexpr int kBK = 64;               // elements per stage
};
template <>
struct Traits<float> {
    static constexpr int kBK = 32;
};

template <typename T>
__global__ __launch_bounds__(kThreadsD) void dense_gemm_kernel(const T *__restrict__ A, int64_t lda,
                                                              const T *__restrict__ B, int64_t ldb, int M,
                                                              int N, int K, float *__restrict__ C,
                                                              int64_t ldc, int tiles_n)
{
    constexpr int kBK = Traits<T>::kBK;
    constexpr int kPieces = (kBM * kStageBytes / 16) / kThreadsD;   // 16-byte pieces per thread per operand: 4
    __shared__ __attribute__((aligned(16))) unsigned char sA[2][kBM * kRowStride];
    __shared__ __attribute__((aligned(16))) unsigned char sB[2][kBN * kRowStride];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = (blockIdx.x / tiles_n) * kBM, n0 = (blockIdx.x % tiles_n) * kBN;
    const int nstages = K / kBK;

    uint4 stA[kPieces], stB[kPieces];
    auto fetch = [&](int stage) {
#pragma unroll
        for (int r = 0; r < kPieces; ++r) {
            const int id = tid + r * kThreadsD;
            const int row = id >> 3, piece = id & 7;
            const int64_t koff = (int64_t)stage * kBK + piece * (16 / (int)sizeof(T));
            stA[r] = make_uint4(0, 0, 0, 0);
            stB[r] = make_uint4(0, 0, 0, 0);
            if (m0 + row < M) stA[r] = *reinterpret_cast<const uint4 *>(A + (int64_t)(m0 + row) * lda + koff);
            if (n0 + row < N) stB[r] = *reinterpret_cast<const uint4 *>(B + (int64_t)(n0 + row) * ldb + koff);
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int r = 0; r < kPieces; ++r) {
            const int id = tid + r * kThreadsD;
            const int row = id >> 3, piece = id & 7;
            *reinterpret_cast<uint4 *>(&sA[buf][row * kRowStride + piece * 16]) = stA[r];
            *reinterpret_cast<uint4 *>(&sB[buf][row * kRowStride + piece * 16]) = stB[r];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    fetch(0);
    park(0);
    __syncthreads();
    for (int stage = 0; stage < nstages; ++stage) {
        const int buf = stage & 1;
        if (stage + 1 < nstages) fetch(stage + 1);
        const unsigned char *pa = &sA[buf][(wm * 64 + (lane & 31)) * kRowStride];
        const unsigned char *pb = &sB[buf][(wn * 64 + (lane & 31)) * kRowStride];
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int ks = 0; ks < kBK / 16; ++ks) {
                const int off = ks * 32 + (lane >> 5) * 16;
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    fa[t] = *reinterpret_cast<const bf16x8 *>(pa + t * 32 * kRowStride + off);
                    fb[t] = *reinterpret_cast<const bf16x8 *>(pb + t * 32 * kRowStride + off);
                }
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < kBK / 2; ++ks) {
                const int off = (ks * 2 + (lane >> 5)) * 4;
                float fa[2], fb[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    fa[t] = *reinterpret_cast<const float *>(pa + t * 32 * kRowStride + off);
                    fb[t] = *reinterpret_cast<const float *>(pb + t * 32 * kRowStride + off);
                }
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a], fb[b], acc[a][b], 0, 0, 0);
            }
        }
        if (stage + 1 < nstages) park(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = n0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M && col < N) C[(int64_t)row * ldc + col] = acc[a][b][v];
            }
        }
}

template <typename T>
hipError_t launch_typed(const void *A, int64_t lda, const void *B, int64_t ldb, int64_t M, int64_t N,
                        int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    const int64_t tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
    if (tiles_m * tiles_n > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    dense_gemm_kernel<T><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreadsD), 0, s>>>(
        static_cast<const T *>(A), lda, static_cast<const T *>(B), ldb, (int)M, (int)N, (int)K, C, ldc,
        (int)tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_dense_ref(const void *A, int64_t lda, const void *B, int64_t ldb, int dtype,
                            int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    // K is a multiple of 32 (checked by the caller); bf16 stages are 64 elements wide
    if (dtype == 1) {
        if (K % Traits<__bf16>::kBK != 0) return hipErrorNotSupported;
        return launch_typed<__bf16>(A, lda, B, ldb, M, N, K, C, ldc, s);
    }
    return launch_typed<float>(A, lda, B, ldb, M, N, K, C, ldc, s);
}

}  // namespace hbmm
