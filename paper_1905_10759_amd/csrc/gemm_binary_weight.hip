// Binary-weight HBMM (beta_a = 1, the paper's HBWN): activations stay fp32, weights are
// delta_w (.) Sign(W).   C[m, n] = sum_j sB[n, j] * sum_{k in segment j} A[m, k] * (+-1)_B[n, k].
//
// The inner sum is a dense contraction of fp32 activations with +-1 weights, so it runs on the
// matrix cores.  An fp32 value is split exactly into three bf16 pieces (8 + 8 + 8 significant
// bits: hi = top half of the fp32 pattern, mid = top half of (a - hi), lo = a - hi - mid), a +-1
// weight is exact in bf16, so each product is exact and the three piece-products accumulate in the
// MFMA's fp32 accumulator: the segment sum is an fp32 sum of exact terms, like the scalar
// definition.  The segment's weight scale is applied once, with one FMA per output, when the
// segment ends (the next segment's first MFMA starts from a zero accumulator).
//
// Layout of the work.  Workgroup = 8 waves, tile 128 (M) x 256 (N); wave = 64 x 64 = 2 x 2 MFMA tiles
// (v_mfma_f32_32x32x16_bf16: lane l feeds row (l mod 32) and 8 consecutive k at 8 * (l div 32)).
// K is walked in stages of 32:
//   * A: 128 rows x 32 fp32 are fetched with 16-byte loads, split into the three bf16 pieces once
//     per workgroup and parked in LDS (row stride 80 bytes: the 16-byte fragment reads of 8
//     consecutive rows land on distinct banks);
//   * B: one packed word per weight row per stage goes through LDS as is; each lane expands its own
//     byte (8 signs) into a bf16x8 fragment with three ALU instructions per pair of elements.
// Global loads run three stages ahead of the multiply (three rotating register sets): a stage is
// only 16 KB per workgroup, and HBM latency is several stages long.
// Tiles that share rows of A are given consecutive slots on the same XCD so that the second read
// of an A tile comes from that XCD's L2.
#include "kernels.h"

namespace hbmm {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBMw = 128, kBNw = 256;
constexpr int kThreadsW = 512;
constexpr int kStageK = 32;
constexpr int kRowBytes = 80;                       // 32 bf16 + 16 bytes of padding
constexpr int kPieceBytes = kBMw * kRowBytes;       // one bf16 piece of the A tile
constexpr int kNumXcd = 8;

// Expand 8 sign bits (bit 1 = +1) into 8 bf16 values +-1.0.  `inv` holds the complemented bits in
// its low byte; element e goes to half (e mod 2) of dword (e div 2).
__device__ __forceinline__ bf16x8 expand_signs(uint32_t inv)
{
    u32x4 d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // complemented bit 2i -> bit 15, complemented bit 2i+1 -> bit 31 (the bf16 sign positions)
        const uint32_t lo = (2 * i <= 15) ? (inv << (15 - 2 * i)) : (inv >> (2 * i - 15));
        const uint32_t hi = inv << (30 - 2 * i);
        d[i] = ((lo | hi) & 0x80008000u) | 0x3f803f80u;
    }
    return __builtin_bit_cast(bf16x8, d);
}

__global__ __launch_bounds__(kThreadsW) void binary_weight_mfma_kernel(
    const float *__restrict__ A, int64_t lda, const uint32_t *__restrict__ b_bits,
    const float *__restrict__ b_scales, int64_t ldw_b, int64_t lds_b, int stages_per_seg, int M, int N,
    int K, float *__restrict__ C, int64_t ldc, int tiles_n, int tiles_total, int slots_per_xcd)
{
    __shared__ __attribute__((aligned(16))) unsigned char sA[2][3 * kPieceBytes];
    __shared__ uint32_t sB[2][kBNw];

    // slot -> tile: consecutive slots of one XCD walk tiles in row-major (m, n) order
    const int slot = (blockIdx.x % kNumXcd) * slots_per_xcd + blockIdx.x / kNumXcd;
    if (slot >= tiles_total) return;
    const int m0 = (slot / tiles_n) * kBMw, n0 = (slot % tiles_n) * kBNw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int nstages = K / kStageK;

    // ---- staging: 2 x (4 fp32 of A) per thread, one word of B for the first 256 threads.  Three
    // register sets rotate so that three stages of global loads are in flight: one stage is only
    // 16 KB per workgroup, far less than what the HBM latency needs to be covered.
    struct Staged {
        float4 a[2];
        uint32_t b;
    };
    // Every load is unconditional (row and stage indices are clamped instead of guarded): a guarded
    // load would make the number of outstanding loads unknown at compile time and force a full
    // wait before every park.  Rows past M / N only feed outputs that are never stored, and the
    // stages past the end are parked but never multiplied.
    const float *a_src[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int id = tid + r * kThreadsW;
        a_src[r] = A + (int64_t)min(m0 + (id >> 3), M - 1) * lda + (id & 7) * 4;
    }
    const uint32_t *b_src = b_bits + (int64_t)min(n0 + (tid & (kBNw - 1)), N - 1) * ldw_b;
    auto fetch = [&](Staged &st, int stage) {
        const int sg = min(stage, nstages - 1);
#pragma unroll
        for (int r = 0; r < 2; ++r) st.a[r] = *reinterpret_cast<const float4 *>(a_src[r] + sg * kStageK);
        st.b = b_src[sg];
    };
    auto split_pair = [](float a, float b, uint32_t &hi, uint32_t &mid, uint32_t &lo) {
        const uint32_t ua = __builtin_bit_cast(uint32_t, a), ub = __builtin_bit_cast(uint32_t, b);
        const uint32_t ha = ua & 0xffff0000u, hb = ub & 0xffff0000u;
        const float ra = a - __builtin_bit_cast(float, ha), rb = b - __builtin_bit_cast(float, hb);
        const uint32_t ma = __builtin_bit_cast(uint32_t, ra) & 0xffff0000u;
        const uint32_t mb = __builtin_bit_cast(uint32_t, rb) & 0xffff0000u;
        const float la = ra - __builtin_bit_cast(float, ma), lb = rb - __builtin_bit_cast(float, mb);
        hi = (ha >> 16) | hb;
        mid = (ma >> 16) | mb;
        lo = (__builtin_bit_cast(uint32_t, la) >> 16) | (__builtin_bit_cast(uint32_t, lb) & 0xffff0000u);
    };
    auto park = [&](const Staged &st, int buf) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int id = tid + r * kThreadsW;
            const int row = id >> 3, c = id & 7;
            uint2 hi, mid, lo;
            split_pair(st.a[r].x, st.a[r].y, hi.x, mid.x, lo.x);
            split_pair(st.a[r].z, st.a[r].w, hi.y, mid.y, lo.y);
            unsigned char *dst = &sA[buf][row * kRowBytes + c * 8];
            *reinterpret_cast<uint2 *>(dst) = hi;
            *reinterpret_cast<uint2 *>(dst + kPieceBytes) = mid;
            *reinterpret_cast<uint2 *>(dst + 2 * kPieceBytes) = lo;
        }
        if (tid < kBNw) sB[buf][tid] = st.b;
    };

    f32x16 acc[2][2], res[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[a][b][v] = 0.f;
                res[a][b][v] = 0.f;
            }

    // per-lane weight-scale rows: output column of accumulator tile tb is n0 + wn*64 + 32*tb + lane%32
    const float *srow[2];
    bool col_ok[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int col = n0 + wn * 64 + tb * 32 + (lane & 31);
        col_ok[tb] = col < N;
        srow[tb] = b_scales + (int64_t)min(col, N - 1) * lds_b;
    }

    float sc[2] = {0.f, 0.f};
    // One K stage: multiply the tile parked in LDS buffer (stage mod 2), request stage + 3 into
    // `incoming`, and park `ready` (stage + 1, requested three stages ago) in the other buffer.
    auto run_stage = [&](int stage, const Staged &ready, Staged &incoming) {
        const int buf = stage & 1;
        fetch(incoming, stage + 3);
        const bool seg_first = stage % stages_per_seg == 0;
        const bool seg_last = (stage + 1) % stages_per_seg == 0;
        if (seg_first) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) sc[tb] = srow[tb][stage / stages_per_seg];
        }
        const unsigned char *pa = &sA[buf][(wm * 64 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
        uint32_t inv[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) inv[tb] = ~sB[buf][wn * 64 + tb * 32 + (lane & 31)] >> ((lane >> 5) * 8);
#pragma unroll
        for (int ks = 0; ks < kStageK / 16; ++ks) {
            bf16x8 fb[2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) fb[tb] = expand_signs((inv[tb] >> (16 * ks)) & 0xffu);
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                bf16x8 fa[2];
#pragma unroll
                for (int ta = 0; ta < 2; ++ta)
                    fa[ta] = *reinterpret_cast<const bf16x8 *>(pa + p * kPieceBytes + ta * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb)
                        acc[ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ta], fb[tb], acc[ta][tb], 0, 0, 0);
            }
        }
        if (seg_last) {
#pragma unroll
            for (int ta = 0; ta < 2; ++ta)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        res[ta][tb][v] = __builtin_fmaf(sc[tb], acc[ta][tb][v], res[ta][tb][v]);
                        acc[ta][tb][v] = 0.f;
                    }
        }
        park(ready, buf ^ 1);   // past the last stage this parks zeros that nobody reads
        __syncthreads();
    };

    Staged s0, s1, s2;
    fetch(s0, 0);
    park(s0, 0);
    fetch(s0, 1);
    fetch(s1, 2);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 3) {
        run_stage(stage, s0, s2);
        if (stage + 1 < nstages) run_stage(stage + 1, s1, s0);
        if (stage + 2 < nstages) run_stage(stage + 2, s2, s1);
    }

#pragma unroll
    for (int ta = 0; ta < 2; ++ta)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            if (!col_ok[tb]) continue;
            const int col = n0 + wn * 64 + tb * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 64 + ta * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M) C[(int64_t)row * ldc + col] = res[ta][tb][v];
            }
        }
}

}  // namespace

hipError_t launch_binary_weight_gemm(const float *A, int64_t lda, const uint32_t *b_bits,
                                     const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                     int64_t M, int64_t N, int64_t K, float *C, int64_t ldc,
                                     hipStream_t s)
{
    if (lda % 4 != 0) return hipErrorNotSupported;   // 16-byte loads of A rows
    const int64_t tiles_m = (M + kBMw - 1) / kBMw, tiles_n = (N + kBNw - 1) / kBNw;
    const int64_t total = tiles_m * tiles_n;
    const int64_t per_xcd = (total + kNumXcd - 1) / kNumXcd;
    if (per_xcd * kNumXcd > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    binary_weight_mfma_kernel<<<dim3((unsigned)(per_xcd * kNumXcd)), dim3(kThreadsW), 0, s>>>(
        A, lda, b_bits, b_scales, ldw_b, lds_b, beta_w / kStageK, (int)M, (int)N, (int)K, C, ldc, (int)tiles_n,
        (int)total, (int)per_xcd);
    return hipGetLastError();
}

}  // namespace hbmm
