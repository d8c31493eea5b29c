// fp8 matrix-core kernel for the HBMM contraction (Eq. 7 of HadaNets) with SHORT segments:
// G = min(beta_a, beta_w) in {16, 32}, both operands binarised with beta >= 16.
//
// v_mfma_f32_32x32x16_fp8_fp8 multiplies 16 elements of K per step, which is the shortest segment
// whose operands can both keep their +-1 form (E4M3: 0x38 = +1.0, 0xB8 = -1.0), and accumulates in
// fp32, where a segment's signed agreement count d is exact.  Then  C += d * (sA * sB)  per segment,
// the popcount kernel's epilogue (for G = 32 the result is bit-identical to it).  Compared with the
// bf16 kernel used for short segments otherwise (one operand rebuilt as fp32 values and split into
// three pieces) this is one product per element pair instead of three, at twice the rate, for one
// more multiplication per output per segment.
//
// Operand layout of the instruction (checked on the device with single-entry operands): lane l
// feeds row (l mod 32) and the 8 consecutive k at 8 * (l div 32), one byte each, k ascending.
//
// Expansion of a 16-bit segment h into 16 bytes, nine vector instructions: both operands are
// expanded the same way, so the order of the 16 elements inside a step is free.  With
// x = h | (h << 12), the mask 0x01010101 << p picks bits {p, p + 8, p + 4, p + 12} of h, one per byte,
// and a shift by 7 - p puts them on the sign bits of four bytes that are otherwise 0x38 (expand16).
// p = 0, 1 give the 8 bytes of lanes 0..31, p = 2, 3 those of lanes 32..63.
//
// Workgroup = 8 waves (4 x 2), tile 256 (M) x 128 (N); wave = 64 x 64 = 2 x 2 MFMA tiles.  K is walked
// in stages of 128 bits = 4 words = 8 MFMA steps, one barrier per stage; global loads (8 bytes of
// packed bits per unit plus the stage's scales) run two stages ahead (a stage is ~5000 cycles) through
// two alternating register sets and are unconditional (clamped indices).  LDS holds, per stage, operand, step and lane half,
// 8 bytes per row (planes padded so that parks and fragment reads are conflict-free).
#include "kernels.h"
#include "tile_map.h"

namespace hbmm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM8 = 256, kBN8 = 128;
constexpr int kThreads8 = 512;
constexpr int kStageWords8 = 4;
constexpr int kSteps8 = 8;                         // MFMA steps (16 bits) per stage
constexpr int kPlaneA8 = kBM8 * 8 + 16, kPlaneB8 = kBN8 * 8 + 16;   // bytes per (step, half) plane

struct MfmaFp8Args {
    const uint32_t *a_bits, *b_bits;
    const float *a_scales, *b_scales;
    float *C;
    int64_t ldc;
    int32_t ldw_a, ldw_b, lds_a, lds_b;
    int32_t M, N, kwords;       // kwords = K / 32
    int32_t shift_a, shift_b;   // log2(beta / G)
    int32_t tiles_m, tiles_n;
};

// 16 sign bits -> 16 fp8 values; lo = the 8 bytes of lanes 0..31, hi = those of lanes 32..63.  E4M3 +1.0
// (0x38) and -1.0 (0xB8) differ in the top bit of the byte only, so a register is 0x38383838 with four
// bits dropped into bits 7, 15, 23, 31: with x = h | h << 12 the bits p, p + 8, p + 16, p + 24 of x are
// the segment's bits p, p + 8, p + 4, p + 12, and one mask plus one v_lshl_or_b32 (written as asm: the
// optimiser turns the C expression into shift, and, or) moves them there.  A set bit gives -1 and a
// clear bit +1 -- for both operands, so every product is the one the signs define; which element of
// the segment sits in which byte does not matter as long as both operands agree.
template <int SHIFT>
__device__ __forceinline__ uint32_t lshl_or8(uint32_t x, uint32_t c)
{
    uint32_t d;
    asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "n"(SHIFT), "s"(c));
    return d;
}
__device__ __forceinline__ void expand16(uint32_t h, uint2 &lo, uint2 &hi)
{
    constexpr uint32_t kOnes = 0x38383838u;   // four times +1.0
    const uint32_t x = h | (h << 12);
    lo.x = lshl_or8<7>(x & 0x01010101u, kOnes);
    lo.y = lshl_or8<6>(x & 0x02020202u, kOnes);
    hi.x = lshl_or8<5>(x & 0x04040404u, kOnes);
    hi.y = lshl_or8<4>(x & 0x08080808u, kOnes);
}

// SEG = segments per stage: 8 (G = 16) or 4 (G = 32).
template <int SEG>
__global__ __launch_bounds__(kThreads8) void mfma_fp8_gemm_kernel(const MfmaFp8Args a)
{
    constexpr int kStepsPerSeg = kSteps8 / SEG;   // 1 or 2
    __shared__ __attribute__((aligned(16))) unsigned char s_a[2][kSteps8 * 2 * kPlaneA8];   // [buf][step][half][row][8 B]
    __shared__ __attribute__((aligned(16))) unsigned char s_b[2][kSteps8 * 2 * kPlaneB8];
    __shared__ __attribute__((aligned(16))) float s_sa[2][SEG][kBM8];
    __shared__ __attribute__((aligned(16))) float s_sb[2][SEG][kBN8];

    // workgroup -> tile: super-tiles of 4 (M) x 8 (N) tiles, an equal share of them per XCD, as in the fp4 kernel
    int tile_m, tile_n;
    if (!xcd_map_tile(blockIdx.x, a.tiles_n, a.tiles_m, 8, 4, tile_n, tile_m)) return;
    const int m0 = tile_m * kBM8, n0 = tile_n * kBN8;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nstages = a.kwords / kStageWords8;                  // packed rows are whole stages (ldw is a multiple of 4)
    const int nseg_total = (a.kwords * SEG) / kStageWords8;      // K / G

    // ---- staging units: unit u = tid + 512 j (j < 2, u < 768): u < 512: A row u / 2, words 2 (u mod 2) .. + 1 of
    // the stage; else B row (u - 512) / 2.  Threads 256.. have one unit only (their second load is a clamped repeat).
    const uint32_t *ubits[2];
    int uword[2], udst[2];
    bool uis_a[2], ulive[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = min(tid + j * kThreads8, 767);
        ulive[j] = tid + j * kThreads8 < 768;
        uis_a[j] = u < 512;
        const int r = uis_a[j] ? u >> 1 : (u - 512) >> 1;
        uword[j] = 2 * (u & 1);
        ubits[j] = uis_a[j] ? a.a_bits + (int64_t)min(m0 + r, a.M - 1) * a.ldw_a : a.b_bits + (int64_t)min(n0 + r, a.N - 1) * a.ldw_b;
        // LDS byte offset of (step 2 * uword, half 0, row r); later steps / the other half are whole planes further
        udst[j] = (2 * uword[j]) * 2 * (uis_a[j] ? kPlaneA8 : kPlaneB8) + r * 8;
    }
    // ---- scale rows: thread t < 256 owns A row t, 256 <= t < 384 owns B row t - 256
    const bool s_is_a = tid < kBM8, s_any = tid < kBM8 + kBN8;
    const int srow = s_is_a ? tid : min(tid - kBM8, kBN8 - 1);
    const bool srow_ok = s_any && (s_is_a ? (m0 + srow < a.M) : (n0 + srow < a.N));
    const float *gscale = s_is_a ? a.a_scales + (int64_t)min(m0 + srow, a.M - 1) * a.lds_a
                                 : a.b_scales + (int64_t)min(n0 + srow, a.N - 1) * a.lds_b;
    const int sshift = s_is_a ? a.shift_a : a.shift_b;

    struct Staged {
        uint2 bits[2];
        float scale[SEG];
    };
    auto fetch = [&](Staged &st, int stage) {
        const int sg = min(stage, nstages - 1);
#pragma unroll
        for (int j = 0; j < 2; ++j) st.bits[j] = *reinterpret_cast<const uint2 *>(ubits[j] + sg * kStageWords8 + uword[j]);
#pragma unroll
        for (int s = 0; s < SEG; ++s) st.scale[s] = gscale[min(sg * SEG + s, nseg_total - 1) >> sshift];
    };
    auto park = [&](const Staged &st, int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (j == 1 && !ulive[1]) continue;
            unsigned char *base = (uis_a[j] ? &s_a[buf][0] : &s_b[buf][0]) + udst[j];
            const int plane = uis_a[j] ? kPlaneA8 : kPlaneB8;
            const uint32_t w[2] = {st.bits[j].x, st.bits[j].y};
#pragma unroll
            for (int q = 0; q < 4; ++q) {   // the unit's four 16-bit segments = four MFMA steps
                uint2 lo, hi;
                expand16((w[q >> 1] >> (16 * (q & 1))) & 0xffffu, lo, hi);
                *reinterpret_cast<uint2 *>(base + (2 * q) * plane) = lo;
                *reinterpret_cast<uint2 *>(base + (2 * q + 1) * plane) = hi;
            }
        }
        // a scale of 0 switches off rows past M / N (K is a whole number of stages, so no segment lies past it)
        if (s_any) {
#pragma unroll
            for (int s = 0; s < SEG; ++s) (s_is_a ? s_sa[buf][s] : s_sb[buf][s])[srow] = srow_ok ? st.scale[s] : 0.f;
        }
    };

    f32x16 acc[2][2], res[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[x][y][v] = 0.f;
                res[x][y][v] = 0.f;
            }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // buf = stage mod 2 is passed as a literal, so that every LDS address of the stage is a register
    // plus an immediate offset
    auto run_stage = [&](int stage, const int buf, const Staged &ready, Staged &incoming) {
        fetch(incoming, stage + 2);
        const int rl = lane & 31, hi = lane >> 5;
        float sb_r[2];
        float4 sa_r[2][4];
#pragma unroll
        for (int ks = 0; ks < kSteps8; ++ks) {
            long fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int ra = wm * 64 + t * 32 + rl, rb = wn * 64 + t * 32 + rl;
                fa[t] = *reinterpret_cast<const long *>(&s_a[buf][(2 * ks + hi) * kPlaneA8 + ra * 8]);
                fb[t] = *reinterpret_cast<const long *>(&s_b[buf][(2 * ks + hi) * kPlaneB8 + rb * 8]);
            }
            const bool seg_first = ks % kStepsPerSeg == 0;   // compile-time
            if (seg_first) {
                const int sgm = ks / kStepsPerSeg;
#pragma unroll
                for (int y = 0; y < 2; ++y) sb_r[y] = s_sb[buf][sgm][wn * 64 + y * 32 + (lane & 31)];
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        sa_r[x][q] = *reinterpret_cast<const float4 *>(&s_sa[buf][sgm][wm * 64 + x * 32 + 4 * (lane >> 5) + 8 * q]);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(fa[x], fb[y], seg_first ? zero16 : acc[x][y], 0, 0, 0);
            // pinned: otherwise the optimiser sinks the products down to their only use, the epilogue
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) asm volatile("" : "+v"(acc[x][y]));
            if ((ks + 1) % kStepsPerSeg == 0) {
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    const float sb = sb_r[y];
#pragma unroll
                    for (int x = 0; x < 2; ++x) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4 sa4 = sa_r[x][q];
                            res[x][y][4 * q + 0] = __builtin_fmaf(acc[x][y][4 * q + 0], sa4.x * sb, res[x][y][4 * q + 0]);
                            res[x][y][4 * q + 1] = __builtin_fmaf(acc[x][y][4 * q + 1], sa4.y * sb, res[x][y][4 * q + 1]);
                            res[x][y][4 * q + 2] = __builtin_fmaf(acc[x][y][4 * q + 2], sa4.z * sb, res[x][y][4 * q + 2]);
                            res[x][y][4 * q + 3] = __builtin_fmaf(acc[x][y][4 * q + 3], sa4.w * sb, res[x][y][4 * q + 3]);
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(res[x][y][v]));
                    }
                }
            }
        }
        park(ready, buf ^ 1);   // past the last stage this parks data that nobody reads
        __syncthreads();
    };

    Staged s0, s1;
    fetch(s0, 0);
    park(s0, 0);
    fetch(s0, 1);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 2) {
        run_stage(stage, 0, s0, s1);
        if (stage + 1 < nstages) run_stage(stage + 1, 1, s1, s0);
    }

#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int col = n0 + wn * 64 + y * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 64 + x * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.M && col < a.N) a.C[(int64_t)row * a.ldc + col] = res[x][y][v];
            }
        }
}

int ilog2f8(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

hipError_t launch_mfma_fp8_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                                int64_t lds_a, int beta_a, const uint32_t *b_bits,
                                const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    const int G = beta_a < beta_w ? beta_a : beta_w;
    if (G != 16 && G != 32) return hipErrorNotSupported;
    if (K % 128 != 0) return hipErrorNotSupported;   // whole stages: the caller falls back otherwise
    MfmaFp8Args a{};
    a.a_bits = a_bits; a.b_bits = b_bits; a.a_scales = a_scales; a.b_scales = b_scales;
    a.C = C; a.ldc = ldc;
    a.ldw_a = (int32_t)ldw_a; a.ldw_b = (int32_t)ldw_b; a.lds_a = (int32_t)lds_a; a.lds_b = (int32_t)lds_b;
    a.M = (int32_t)M; a.N = (int32_t)N; a.kwords = (int32_t)(K / 32);
    a.shift_a = ilog2f8(beta_a / G);
    a.shift_b = ilog2f8(beta_w / G);
    const int64_t tiles_m = (M + kBM8 - 1) / kBM8, tiles_n = (N + kBN8 - 1) / kBN8;
    if (tiles_m * tiles_n > 0x7fffff00LL) return hipErrorInvalidConfiguration;
    const int64_t nblocks = xcd_map_blocks(tiles_m * tiles_n);
    a.tiles_m = (int32_t)tiles_m; a.tiles_n = (int32_t)tiles_n;
    const dim3 grid((unsigned)nblocks), block(kThreads8);
    if (G == 16)
        mfma_fp8_gemm_kernel<8><<<grid, block, 0, s>>>(a);
    else
        mfma_fp8_gemm_kernel<4><<<grid, block, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hbmm
