// Hadamard binarisation of one operand in a single pass: block scales (HadaNets Eq. 1 / Eq. 3),
// Sign (Eq. 2 / Eq. 4) and bit-packing (section 4), for gfx950.
//
// The pass is bound by HBM reads: 4 bytes in per element against 1/8 + 4/beta bytes out.
//
// pack_rows_kernel (source rows x K, K contiguous):
//   A wave covers 256 consecutive K elements of one row with one 16-byte load per lane, keeps
//   kUnroll such loads in flight (4 KB contiguous per wave) and consecutive waves sweep memory
//   linearly.  Lane l holds elements 4l .. 4l+3, i.e. one nibble of the packed
//   word; the eight nibbles of a 32-bit word sit in eight consecutive lanes and are OR-ed together
//   with three DPP steps, so no ballot-reordering is needed.  |x| is summed as
//   (|x0|+|x1|)+(|x2|+|x3|) in the lane and then pairwise over the beta/4 lanes of the segment.
//
// pack_cols_kernel (source K x rows, rows contiguous): a lane owns one output row and walks K, so
//   every load is a coalesced 256-byte wave access; the word is built with shifts and the scale
//   is a sequential double-precision sum rounded once.
#include "kernels.h"
#include "wave_ops.h"

namespace hbmm {
namespace {

constexpr int kUnroll = 4;          // 16-byte loads in flight per lane
constexpr int kChunk = 256;         // K elements per wave per load
constexpr int kWavesPerBlock = 4;

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pick4(const uint32_t (&v)[4], int i)
{
    return i == 0 ? v[0] : i == 1 ? v[1] : i == 2 ? v[2] : v[3];
}
__device__ __forceinline__ float pick4(const float (&v)[4], int i)
{
    return i == 0 ? v[0] : i == 1 ? v[1] : i == 2 ? v[2] : v[3];
}

// One wave = one "slot": kUnroll consecutive 256-element chunks (4 KB) of one row.  Slots are
// numbered row-major, so consecutive waves and workgroups sweep the source linearly.
template <int BETA, bool VEC>
__global__ __launch_bounds__(64 * kWavesPerBlock) void pack_rows_kernel(
    const float *__restrict__ x, uint32_t total_slots, uint32_t slots_per_row, int K, int64_t ldx,
    uint32_t *__restrict__ bits, int64_t ldw, float *__restrict__ scales, int64_t lds, int words_valid)
{
    constexpr int kSegLanes = BETA >= 4 ? BETA / 4 : 1;   // lanes per segment (beta 2: two segments per lane)
    const int lane = threadIdx.x & 63;
    const uint32_t slot = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (slot >= total_slots) return;
    const uint32_t row = slot / slots_per_row;
    const int g = (int)(slot - row * slots_per_row);
    const int kbase = g * (kUnroll * kChunk) + 4 * lane;
    const float *xr = x + (int64_t)row * ldx;

    f32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int k = kbase + u * kChunk;
        v[u] = f32x4{-1.f, -1.f, -1.f, -1.f};   // sign bit 0; kept out of the sums by `live` below
        if (k < K) {
            if (VEC) {
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(xr + k));
            } else {
                v[u].x = xr[k];
                v[u].y = xr[k + 1];
                v[u].z = xr[k + 2];
                v[u].w = xr[k + 3];
            }
        }
    }

    uint32_t w[kUnroll];
    float p[kUnroll], p2[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const bool live = kbase + u * kChunk < K;
        // signs -> nibble -> 32-bit word, OR-ed over the 8 lanes that hold it
        const uint32_t nib = (v[u].x >= 0.f ? 1u : 0u) | (v[u].y >= 0.f ? 2u : 0u) |
                             (v[u].z >= 0.f ? 4u : 0u) | (v[u].w >= 0.f ? 8u : 0u);
        w[u] = pack_word_from_nibbles(nib, lane);
        // sum of |x| over the beta-segment, every lane of the segment gets it
        const float lo = live ? fabsf(v[u].x) + fabsf(v[u].y) : 0.f;
        const float hi = live ? fabsf(v[u].z) + fabsf(v[u].w) : 0.f;
        if (BETA == 2) {
            p[u] = lo;
            p2[u] = hi;
        } else {
            p[u] = segment_sum<kSegLanes>(lo + hi);
            p2[u] = 0.f;
        }
    }

    // Stores.  After the reductions every lane of a group holds the group's value for all kUnroll
    // chunks; lane j (< kUnroll) of each group stores chunk j's value, so the wave writes its 32
    // words (128 bytes) with one instruction.
    {
        const int j = lane & 7, grp = lane >> 3;
        const int widx = g * (kUnroll * kChunk / 32) + j * (kChunk / 32) + grp;
        if (j < kUnroll && widx < words_valid) bits[(int64_t)row * ldw + widx] = pick4(w, j);
    }
    float *srow = scales + (int64_t)row * lds;
    if (BETA >= 16) {
        // same trick for the scales: 4 * 256 / beta values with one instruction
        const int j = lane & (kSegLanes - 1), e = lane / kSegLanes;
        const int k = g * (kUnroll * kChunk) + j * kChunk + e * BETA;
        if (j < kUnroll && k < K) srow[k / BETA] = pick4(p, j) * (1.0f / BETA);
    } else {
        // short segments: at least one scale per two lanes, stored chunk by chunk
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int k = kbase + u * kChunk;
            if (k >= K) continue;
            if (BETA == 2) {
                srow[k / 2] = p[u] * 0.5f;
                srow[k / 2 + 1] = p2[u] * 0.5f;
            } else if ((lane & (kSegLanes - 1)) == 0) {
                srow[k / BETA] = p[u] * (1.0f / BETA);
            }
        }
    }
}

template <int BETA>
__global__ __launch_bounds__(256) void pack_cols_kernel(
    const float *__restrict__ x, int64_t rows, int K, int64_t ldx, uint32_t *__restrict__ bits,
    int64_t ldw, float *__restrict__ scales, int64_t lds, int words_valid)
{
    constexpr int kSpan = 256;   // K elements per thread: a whole number of segments for every beta
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    const int k0 = blockIdx.y * kSpan;
    const int k1 = min(K, k0 + kSpan);
    double acc = 0.0;
    for (int kw = k0; kw < k1; kw += 32) {
        uint32_t w = 0;
#pragma unroll 8
        for (int b = 0; b < 32; ++b) {
            const float v = x[(int64_t)(kw + b) * ldx + r];
            w |= (v >= 0.f ? 1u : 0u) << b;
            acc += fabs((double)v);
            if (BETA < 32 && ((b + 1) & (BETA - 1)) == 0) {
                scales[r * lds + (kw + b) / BETA] = (float)(acc / (double)BETA);
                acc = 0.0;
            }
        }
        bits[r * ldw + (kw >> 5)] = w;
        if (BETA >= 32 && ((kw + 32) & (BETA - 1)) == 0) {
            scales[r * lds + kw / BETA] = (float)(acc / (double)BETA);
            acc = 0.0;
        }
    }
    if (k1 == K)
        for (int w = K >> 5; w < words_valid; ++w) bits[r * ldw + w] = 0u;
}

// Any segment length in 2..256 and any K, either layout: element (r, k) is x[r * sr + k * sk].
// One thread per output word (its 32 signs) and one per scale (a sequential double-precision sum of
// the segment's |x|, divided by the segment's own length -- the last one may be shorter).  This is
// the path for settings outside the paper's table (its segment lengths are powers of two dividing
// K); it reads every element twice and is not tuned.
__global__ __launch_bounds__(256) void pack_any_kernel(
    const float *__restrict__ x, int64_t rows, int K, int64_t sr, int64_t sk, int beta, uint32_t *__restrict__ bits,
    int64_t ldw, float *__restrict__ scales, int64_t lds, int words_valid, int nseg)
{
    const int per_row = words_valid + nseg;
    const int64_t total = rows * per_row;
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (int64_t)gridDim.x * 256) {
        const int64_t r = id / per_row;
        const int item = (int)(id - r * per_row);
        const float *xr = x + r * sr;
        if (item < words_valid) {
            uint32_t w = 0;
            const int k0 = item * 32, n = min(32, K - k0);   // n <= 0: a padding word
            for (int b = 0; b < n; ++b) w |= (xr[(int64_t)(k0 + b) * sk] >= 0.f ? 1u : 0u) << b;
            bits[r * ldw + item] = w;
        } else {
            const int j = item - words_valid;
            const int k0 = j * beta, n = min(beta, K - k0);
            double acc = 0.0;
            for (int b = 0; b < n; ++b) acc += fabs((double)xr[(int64_t)(k0 + b) * sk]);
            scales[r * lds + j] = (float)(acc / (double)n);
        }
    }
}

// An activation tensor seen as `rows` rows of W contiguous elements (rows = batch * channels * height), for
// any segment length: the sign bits are packed flat (element e = r * W + y is bit e mod 32 of word e div 32,
// rows are not padded), the scales are rows x ceil(W / beta), segments starting anew in every row and the
// last one of a row averaged over its own length.  One thread per output word and one per scale; for
// widths that beta does not divide (7 x 7 feature maps), not tuned.
__global__ __launch_bounds__(256) void pack_activations_any_kernel(
    const float *__restrict__ x, int64_t rows, int W, int beta, uint32_t *__restrict__ bits, float *__restrict__ scales,
    int64_t nwords, int nseg)
{
    const int64_t count = rows * W, nscales = rows * nseg;
    for (int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x; id < nwords + nscales; id += (int64_t)gridDim.x * 256) {
        if (id < nwords) {
            uint32_t w = 0;
            const int64_t e0 = id * 32;
            const int n = (int)(count - e0 < 32 ? count - e0 : 32);
            for (int b = 0; b < n; ++b) w |= (x[e0 + b] >= 0.f ? 1u : 0u) << b;
            bits[id] = w;
        } else {
            const int64_t sid = id - nwords, r = sid / nseg;
            const int j = (int)(sid - r * nseg);
            const int y0 = j * beta, n = min(beta, W - y0);
            double acc = 0.0;
            for (int b = 0; b < n; ++b) acc += fabs((double)x[r * W + y0 + b]);
            scales[sid] = (float)(acc / (double)n);
        }
    }
}

template <int BETA>
hipError_t pack_rows_beta(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *bits,
                          int64_t ldw, float *scales, int64_t lds, hipStream_t s)
{
    const int64_t slots_per_row = (K + kUnroll * kChunk - 1) / (kUnroll * kChunk);
    const int64_t total = rows * slots_per_row;
    if (total >= ((int64_t)1 << 32)) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)((total + kWavesPerBlock - 1) / kWavesPerBlock));
    dim3 block(64 * kWavesPerBlock);
    const int wv = (int)packed_words(K);
    const bool vec = (ldx % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
    if (vec)
        pack_rows_kernel<BETA, true><<<grid, block, 0, s>>>(x, (uint32_t)total, (uint32_t)slots_per_row, (int)K, ldx,
                                                             bits, ldw, scales, lds, wv);
    else
        pack_rows_kernel<BETA, false><<<grid, block, 0, s>>>(x, (uint32_t)total, (uint32_t)slots_per_row, (int)K, ldx,
                                                              bits, ldw, scales, lds, wv);
    return hipGetLastError();
}

template <int BETA>
hipError_t pack_cols_beta(const float *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *bits,
                          int64_t ldw, float *scales, int64_t lds, hipStream_t s)
{
    dim3 grid((unsigned)((rows + 255) / 256), (unsigned)((K + 255) / 256));
    pack_cols_kernel<BETA><<<grid, dim3(256), 0, s>>>(x, rows, (int)K, ldx, bits, ldw, scales, lds,
                                                      (int)packed_words(K));
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pack_rows(const float *x, int64_t rows, int64_t K, int64_t ldx, int beta,
                            uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s)
{
    switch (beta) {
    case 2: return pack_rows_beta<2>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 4: return pack_rows_beta<4>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 8: return pack_rows_beta<8>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 16: return pack_rows_beta<16>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 32: return pack_rows_beta<32>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 64: return pack_rows_beta<64>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 128: return pack_rows_beta<128>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 256: return pack_rows_beta<256>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_pack_cols(const float *x, int64_t rows, int64_t K, int64_t ldx, int beta,
                            uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s)
{
    switch (beta) {
    case 2: return pack_cols_beta<2>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 4: return pack_cols_beta<4>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 8: return pack_cols_beta<8>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 16: return pack_cols_beta<16>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 32: return pack_cols_beta<32>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 64: return pack_cols_beta<64>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 128: return pack_cols_beta<128>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    case 256: return pack_cols_beta<256>(x, rows, K, ldx, bits, ldw, scales, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_pack_any(const float *x, int64_t rows, int64_t K, int64_t ldx, int layout, int beta,
                           uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s)
{
    const int wv = (int)packed_words(K), nseg = (int)((K + beta - 1) / beta);
    const int64_t total = rows * (wv + nseg);
    const int64_t blocks = (total + 255) / 256;
    const unsigned grid = (unsigned)(blocks < 256 * 64 ? blocks : 256 * 64);
    pack_any_kernel<<<dim3(grid), dim3(256), 0, s>>>(x, rows, (int)K, layout == 0 ? ldx : 1, layout == 0 ? 1 : ldx, beta,
                                                     bits, ldw, scales, lds, wv, nseg);
    return hipGetLastError();
}

hipError_t launch_pack_activations_any(const float *x, int64_t rows, int64_t W, int beta, uint32_t *bits, float *scales,
                                       hipStream_t s)
{
    const int64_t nwords = (rows * W + 31) / 32;
    const int nseg = (int)((W + beta - 1) / beta);
    const int64_t blocks = (nwords + rows * nseg + 255) / 256;
    const unsigned grid = (unsigned)(blocks < 256 * 64 ? blocks : 256 * 64);
    pack_activations_any_kernel<<<dim3(grid), dim3(256), 0, s>>>(x, rows, (int)W, beta, bits, scales, nwords, nseg);
    return hipGetLastError();
}

}  // namespace hbmm
