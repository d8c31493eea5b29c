// Gradient through the Hadamard binarisation x~ = delta (.) Sign(x) (HadaNets Eq. 6, with the
// straight-through estimator of Eq. 5 for Sign):
//   dC/dx_i = (1/beta) Sign(x_i) * sum_{j in segment(i)} g_j Sign(x_j)  +  delta_segment(i) * g_i * [|x_i| <= 1]
// g = dC/dx~, delta = mean |x| over the segment (recomputed here from x, as the forward pass does).
//
// HBM-bound: 8 bytes read and 4 written per element.  Same work layout as the forward pack kernel:
// a wave owns 4 KB of one row of x and of g (four 16-byte loads of each per lane in flight), lane l
// holds elements 4l .. 4l+3 of a 256-element chunk, the two segment sums (|x| and g*Sign(x)) are
// reduced pairwise over the beta/4 lanes of the segment with DPP, and each lane writes its four
// results with one 16-byte store.
#include "kernels.h"
#include "wave_ops.h"

namespace hbmm {
namespace {

constexpr int kUnrollB = 4;
constexpr int kChunkB = 256;
constexpr int kWavesB = 4;

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float sgn_apply(float x, float g) { return x >= 0.f ? g : -g; }
__device__ __forceinline__ float ste(float x) { return fabsf(x) <= 1.0f ? 1.0f : 0.0f; }

template <int BETA, bool VEC>
__global__ __launch_bounds__(64 * kWavesB) void binarize_backward_kernel(
    const float *__restrict__ x, const float *__restrict__ g, uint32_t total_slots, uint32_t slots_per_row,
    int K, int64_t ldx, int64_t ldg, float *__restrict__ gx, int64_t ldgx)
{
    constexpr int kSegLanes = BETA >= 4 ? BETA / 4 : 1;
    const int lane = threadIdx.x & 63;
    const uint32_t slot = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesB + (threadIdx.x >> 6));
    if (slot >= total_slots) return;
    const uint32_t row = slot / slots_per_row;
    const int kbase = (int)(slot - row * slots_per_row) * (kUnrollB * kChunkB) + 4 * lane;
    const float *xr = x + (int64_t)row * ldx;
    const float *gr = g + (int64_t)row * ldg;
    float *outr = gx + (int64_t)row * ldgx;

    f32x4 xv[kUnrollB], gv[kUnrollB];
#pragma unroll
    for (int u = 0; u < kUnrollB; ++u) {
        const int k = kbase + u * kChunkB;
        xv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        gv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (k < K) {
            if (VEC) {
                xv[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(xr + k));
                gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(gr + k));
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    xv[u][c] = xr[k + c];
                    gv[u][c] = gr[k + c];
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kUnrollB; ++u) {
        const int k = kbase + u * kChunkB;
        f32x4 r;
        if (BETA == 1) {
            // delta = |x|, the segment is the element itself
#pragma unroll
            for (int c = 0; c < 4; ++c) r[c] = gv[u][c] + fabsf(xv[u][c]) * gv[u][c] * ste(xv[u][c]);
        } else if (BETA == 2) {
            const float a0 = (fabsf(xv[u][0]) + fabsf(xv[u][1])) * 0.5f, a1 = (fabsf(xv[u][2]) + fabsf(xv[u][3])) * 0.5f;
            const float d0 = (sgn_apply(xv[u][0], gv[u][0]) + sgn_apply(xv[u][1], gv[u][1])) * 0.5f;
            const float d1 = (sgn_apply(xv[u][2], gv[u][2]) + sgn_apply(xv[u][3], gv[u][3])) * 0.5f;
            r[0] = __builtin_fmaf(a0 * gv[u][0], ste(xv[u][0]), sgn_apply(xv[u][0], d0));
            r[1] = __builtin_fmaf(a0 * gv[u][1], ste(xv[u][1]), sgn_apply(xv[u][1], d0));
            r[2] = __builtin_fmaf(a1 * gv[u][2], ste(xv[u][2]), sgn_apply(xv[u][2], d1));
            r[3] = __builtin_fmaf(a1 * gv[u][3], ste(xv[u][3]), sgn_apply(xv[u][3], d1));
        } else {
            float a = (fabsf(xv[u][0]) + fabsf(xv[u][1])) + (fabsf(xv[u][2]) + fabsf(xv[u][3]));
            float d = (sgn_apply(xv[u][0], gv[u][0]) + sgn_apply(xv[u][1], gv[u][1])) +
                      (sgn_apply(xv[u][2], gv[u][2]) + sgn_apply(xv[u][3], gv[u][3]));
            a = segment_sum<kSegLanes>(a) * (1.0f / BETA);
            d = segment_sum<kSegLanes>(d) * (1.0f / BETA);
#pragma unroll
            for (int c = 0; c < 4; ++c)
                r[c] = __builtin_fmaf(a * gv[u][c], ste(xv[u][c]), sgn_apply(xv[u][c], d));
        }
        if (k < K) {
            if (VEC) {
                *reinterpret_cast<f32x4 *>(outr + k) = r;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) outr[k + c] = r[c];
            }
        }
    }
}

template <int BETA>
hipError_t launch_beta(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx, int64_t ldg,
                       float *gx, int64_t ldgx, hipStream_t s)
{
    const int64_t slots_per_row = (K + kUnrollB * kChunkB - 1) / (kUnrollB * kChunkB);
    const int64_t total = rows * slots_per_row;
    if (total >= ((int64_t)1 << 32)) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)((total + kWavesB - 1) / kWavesB)), block(64 * kWavesB);
    auto al = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    const bool vec = ldx % 4 == 0 && ldg % 4 == 0 && ldgx % 4 == 0 && al(x) && al(g) && al(gx);
    if (vec)
        binarize_backward_kernel<BETA, true><<<grid, block, 0, s>>>(x, g, (uint32_t)total, (uint32_t)slots_per_row, (int)K, ldx, ldg, gx, ldgx);
    else
        binarize_backward_kernel<BETA, false><<<grid, block, 0, s>>>(x, g, (uint32_t)total, (uint32_t)slots_per_row, (int)K, ldx, ldg, gx, ldgx);
    return hipGetLastError();
}

// Any segment length in 1..256 and any K (the last segment may be shorter: then delta is the mean over its own
// length n and its derivative 1/n): one thread per segment, sums in double.  For settings outside the
// paper's table; it reads x and g twice and is not tuned.
__global__ __launch_bounds__(256) void binarize_backward_any_kernel(
    const float *__restrict__ x, const float *__restrict__ g, int64_t rows, int K, int64_t ldx, int64_t ldg, int beta,
    float *__restrict__ gx, int64_t ldgx, int nseg)
{
    const int64_t total = rows * nseg;
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (int64_t)gridDim.x * 256) {
        const int64_t r = id / nseg;
        const int k0 = (int)(id - r * nseg) * beta, n = min(beta, K - k0);
        const float *xr = x + r * ldx + k0, *gr = g + r * ldg + k0;
        double sabs = 0.0, sdot = 0.0;
        for (int i = 0; i < n; ++i) {
            sabs += fabs((double)xr[i]);
            sdot += xr[i] >= 0.f ? (double)gr[i] : -(double)gr[i];
        }
        const float delta = (float)(sabs / (double)n);
        const double mean_dot = sdot / (double)n;
        float *o = gx + r * ldgx + k0;
        for (int i = 0; i < n; ++i) {
            const float xv = xr[i];
            const double ste = fabsf(xv) <= 1.0f ? (double)delta * (double)gr[i] : 0.0;
            o[i] = (float)((xv >= 0.f ? mean_dot : -mean_dot) + ste);
        }
    }
}

}  // namespace

hipError_t launch_binarize_backward_any(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx, int64_t ldg,
                                        int beta, float *gx, int64_t ldgx, hipStream_t s)
{
    const int nseg = (int)((K + beta - 1) / beta);
    const int64_t blocks = (rows * nseg + 255) / 256;
    const unsigned grid = (unsigned)(blocks < 256 * 64 ? blocks : 256 * 64);
    binarize_backward_any_kernel<<<dim3(grid), dim3(256), 0, s>>>(x, g, rows, (int)K, ldx, ldg, beta, gx, ldgx, nseg);
    return hipGetLastError();
}

hipError_t launch_binarize_backward(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx,
                                    int64_t ldg, int beta, float *gx, int64_t ldgx, hipStream_t s)
{
    switch (beta) {
    case 1: return launch_beta<1>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 2: return launch_beta<2>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 4: return launch_beta<4>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 8: return launch_beta<8>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 16: return launch_beta<16>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 32: return launch_beta<32>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 64: return launch_beta<64>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 128: return launch_beta<128>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    case 256: return launch_beta<256>(x, g, rows, K, ldx, ldg, gx, ldgx, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace hbmm
