// fp4 matrix-core variant of the HBMM contraction (Eq. 7 of HadaNets).
//
// +-1 is exactly representable in the 4-bit float format of gfx950's v_mfma_scale_f32_32x32x64_f8f6f4
// (E2M1: 0x2 = +1.0, 0xA = -1.0), whose rate is four times that of bf16 and whose accumulator is
// fp32: a segment's signed agreement count d = sum_k (+-1)(+-1) comes out exactly (|d| <= 256), and
// the epilogue  C += d * (sA * sB)  is the popcount kernel's, rounding for rounding, so the outputs
// are bit-identical to it.  The operands stay 1 bit per element in memory; they are expanded to
// 4 bits per element on chip, once per workgroup.
//
// Operand layout of the instruction (checked on the device against single-entry operands): lane l
// feeds row (l mod 32) and the 32 consecutive k at 32 * (l div 32) -- exactly one packed word of
// that row -- as 32 nibbles in four registers, k ascending from the low nibble of the first one.
//
// Expansion of a packed word into four registers of 8 nibbles, eight vector instructions: both
// operands are expanded the same way, so the order of the 32 elements inside an MFMA step is free,
// and register s takes the bits 4i + s, i = 0..7, of the word: shifted left by 3 - s they sit on the
// sign bits of the eight nibbles.
//
// Workgroup = 8 waves (4 x 2), tile 256 (M) x 128 (N), one per CU (or 4 waves, 128 x 128, two per CU, for
// problems with few tiles); wave = 64 x 64 = 2 x 2 MFMA tiles.
// K is walked in stages of 256 bits = 8 words = 4 MFMA steps, one barrier per stage.  Global loads
// (8 bytes of packed bits per item, three items per thread, plus the scales of the stage's segments)
// run three stages ahead through rotating register sets and are unconditional (clamped indices).
// LDS holds, per stage and operand, eight planes (one per word) of 16 bytes per row, so the
// fragment read of 32 consecutive rows is one contiguous 512-byte run.
#include "kernels.h"
#include "tile_map.h"

namespace hbmm {
namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBN4 = 128;
constexpr int kStageWords4 = 8;
constexpr int kPlaneB = kBN4 * 16 + 16;   // bytes per word plane

struct MfmaFp4Args {
    const uint32_t *a_bits, *b_bits;
    const float *a_scales, *b_scales;
    float *C;
    int64_t ldc;
    int32_t ldw_a, ldw_b, lds_a, lds_b;
    int32_t M, N, kwords;       // kwords = K / 32
    int32_t shift_a, shift_b;   // log2(beta / G)
    int32_t tiles_m, tiles_n;
};

// 32 sign bits -> 32 fp4 values in the order described above: E2M1 +1.0 (0x2) and -1.0 (0xA) differ in
// the top bit of the nibble only, so a register is 0x22222222 with eight bits of the word dropped into
// bits 4i + 3: mask them where they are (v_and_b32 with a literal), then shift and merge in one
// v_lshl_or_b32 -- written as asm, because the optimiser rewrites the C expression into shift, and, or.
// A set bit gives -1 and a clear bit +1 -- for both operands, so every product (+-1)(+-1) is the one
// the signs define.
template <int SHIFT>
__device__ __forceinline__ int lshl_or(uint32_t x, uint32_t c)
{
    int d;
    asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "n"(SHIFT), "s"(c));
    return d;
}
__device__ __forceinline__ i32x4v expand32(uint32_t w)
{
    constexpr uint32_t kOnes = 0x22222222u;   // eight times +1.0
    i32x4v e;
    e[0] = lshl_or<3>(w & 0x11111111u, kOnes);
    e[1] = lshl_or<2>(w & 0x22222222u, kOnes);
    e[2] = lshl_or<1>(w & 0x44444444u, kOnes);
    e[3] = lshl_or<0>(w & 0x88888888u, kOnes);
    return e;
}

// SEG = segments of G = min(beta_a, beta_w) bits per stage: 1, 2 or 4 (G = 256, 128, 64).
// kBM4 = rows of A per workgroup: 256 (8 waves, one workgroup per CU) or 128 (4 waves, two per CU).
template <int SEG, int kBM4>
__global__ __launch_bounds__(2 * kBM4, kBM4 == 128 ? 2 : 1) void mfma_fp4_gemm_kernel(const MfmaFp4Args a)
{
    constexpr int kThreads4 = 2 * kBM4;
    constexpr int kItems4 = (4 * kBM4 + 4 * kBN4) / kThreads4;   // (row, pair of words) items per thread per stage
    constexpr int kPlaneA = kBM4 * 16 + 16;
    constexpr int kStepsPerSeg = 4 / SEG;   // MFMA steps (64 bits) per segment
    // [buf][word][row][16 B]; every word plane is padded by 16 bytes: eight consecutive lanes park two
    // rows x four word pairs (two planes apart), which then fall into eight different 16-byte bank groups
    // (measured: no LDS bank conflicts left)
    __shared__ __attribute__((aligned(16))) unsigned char s_a[2][kStageWords4 * kPlaneA];
    __shared__ __attribute__((aligned(16))) unsigned char s_b[2][kStageWords4 * kPlaneB];
    __shared__ __attribute__((aligned(16))) float s_sa[2][SEG][kBM4];
    __shared__ __attribute__((aligned(16))) float s_sb[2][SEG][kBN4];

    // Workgroup -> tile.  Workgroups are dealt to the 8 XCDs round-robin and every XCD has its own L2,
    // so tiles are grouped into super-tiles of 4 (M) x 8 (N) that one XCD works on at a time (their 4 A
    // tiles and 8 B tiles fit that L2 and are fetched into it once), and every XCD gets an equal
    // share of the sequence of super-tiles (tile_map.h).
    int tile_m, tile_n;
    if (!xcd_map_tile(blockIdx.x, a.tiles_n, a.tiles_m, 8, 4, tile_n, tile_m)) return;
    const int m0 = tile_m * kBM4, n0 = tile_n * kBN4;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nstages = (a.kwords + kStageWords4 - 1) / kStageWords4;
    const int nseg_total = (a.kwords * SEG) / kStageWords4;      // K / G

    // ---- staging items: item i = tid + 512 j; i < 1024: A row i / 4, words 2 (i mod 4) .. + 1 of the
    // stage; else B row (i - 1024) / 4
    const uint32_t *ibits[kItems4];
    int iword[kItems4], idst[kItems4];
    bool irow_ok[kItems4];
    int ildw[kItems4];
#pragma unroll
    for (int j = 0; j < kItems4; ++j) {
        const int i = tid + j * kThreads4;
        const bool is_a = i < 4 * kBM4;
        const int r = is_a ? i >> 2 : (i - 4 * kBM4) >> 2;
        iword[j] = 2 * (i & 3);
        irow_ok[j] = is_a ? (m0 + r < a.M) : (n0 + r < a.N);
        ildw[j] = is_a ? a.ldw_a : a.ldw_b;
        ibits[j] = is_a ? a.a_bits + (int64_t)min(m0 + r, a.M - 1) * a.ldw_a : a.b_bits + (int64_t)min(n0 + r, a.N - 1) * a.ldw_b;
        // LDS byte offset of (word iword, row r) inside the operand's buffer; the second word is one plane further
        idst[j] = iword[j] * (is_a ? kPlaneA : kPlaneB) + r * 16;
    }
    // ---- scale rows: thread t < 256 owns A row t, 256 <= t < 384 owns B row t - 256
    const bool s_is_a = tid < kBM4, s_any = tid < kBM4 + kBN4;
    const int srow = s_is_a ? tid : min(tid - kBM4, kBN4 - 1);
    const bool srow_ok = s_any && (s_is_a ? (m0 + srow < a.M) : (n0 + srow < a.N));
    const float *gscale = s_is_a ? a.a_scales + (int64_t)min(m0 + srow, a.M - 1) * a.lds_a
                                 : a.b_scales + (int64_t)min(n0 + srow, a.N - 1) * a.lds_b;
    const int sshift = s_is_a ? a.shift_a : a.shift_b;

    struct Staged {
        uint2 bits[kItems4];
        float scale[SEG];
    };
    auto fetch = [&](Staged &st, int stage) {
        const int sg = min(stage, nstages - 1);
#pragma unroll
        for (int j = 0; j < kItems4; ++j) {
            // rows are ldw words long (a multiple of 4, pad words zero); a stage's last pairs may lie past that
            const int w = min(sg * kStageWords4 + iword[j], ildw[j] - 2);
            st.bits[j] = *reinterpret_cast<const uint2 *>(ibits[j] + w);
        }
#pragma unroll
        for (int s = 0; s < SEG; ++s) st.scale[s] = gscale[min(sg * SEG + s, nseg_total - 1) >> sshift];
    };
    auto park = [&](const Staged &st, int stage, int buf) {
#pragma unroll
        for (int j = 0; j < kItems4; ++j) {
            const bool is_a = tid + j * kThreads4 < 4 * kBM4;   // uniform per j
            unsigned char *base = (is_a ? &s_a[buf][0] : &s_b[buf][0]) + idst[j];
            const int plane = is_a ? kPlaneA : kPlaneB;
            // (word pairs past the end of the row hold whatever the clamped load returned: they lie in
            // segments past K, whose scale is parked as 0)
            const uint32_t w0 = st.bits[j].x, w1 = st.bits[j].y;
            *reinterpret_cast<i32x4v *>(base) = expand32(w0);
            *reinterpret_cast<i32x4v *>(base + plane) = expand32(w1);
        }
        // a scale of 0 switches off segments past K (their pad bits expand to -1 and would count) and rows past M / N
        if (s_any) {
#pragma unroll
            for (int s = 0; s < SEG; ++s) {
                const bool live = srow_ok && stage * SEG + s < nseg_total;
                (s_is_a ? s_sa[buf][s] : s_sb[buf][s])[srow] = live ? st.scale[s] : 0.f;
            }
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
        fetch(incoming, stage + 3);
        const int rl = lane & 31, hi = lane >> 5;
        float sb_r[2];
        float4 sa_r[2][4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            i32x8 fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int ra = wm * 64 + t * 32 + rl, rb = wn * 64 + t * 32 + rl;
                const i32x4v va = *reinterpret_cast<const i32x4v *>(&s_a[buf][(2 * ks + hi) * kPlaneA + ra * 16]);
                const i32x4v vb = *reinterpret_cast<const i32x4v *>(&s_b[buf][(2 * ks + hi) * kPlaneB + rb * 16]);
                fa[t] = i32x8{va[0], va[1], va[2], va[3], 0, 0, 0, 0};
                fb[t] = i32x8{vb[0], vb[1], vb[2], vb[3], 0, 0, 0, 0};
            }
            const bool seg_first = ks % kStepsPerSeg == 0;   // compile-time: the segment's first step starts from 0
            if (seg_first) {
                // the segment's scales are requested before its MFMAs, so that they are in registers
                // when the epilogue starts instead of costing an LDS round trip per group of rows
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
                    acc[x][y] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[x], fb[y], seg_first ? zero16 : acc[x][y], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            // Pin the products here: they are pure values whose only use is the segment's epilogue, and
            // without a use at this point the optimiser sinks all four steps down to it (behind the
            // staging code and the barrier), which needs every step's operands in registers at once.
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
                        for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(res[x][y][v]));   // same reason; per element,
                        // so that each FMA can stay in its two-address form (v_fmac_f32 issues faster than v_fma_f32)
                    }
                }
            }
        }
        park(ready, stage + 1, buf ^ 1);   // past the last stage this parks data that nobody reads
        __syncthreads();
    };

    Staged s0, s1, s2;
    fetch(s0, 0);
    park(s0, 0, 0);
    fetch(s0, 1);
    fetch(s1, 2);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 6) {
        run_stage(stage, 0, s0, s2);
        if (stage + 1 < nstages) run_stage(stage + 1, 1, s1, s0);
        if (stage + 2 < nstages) run_stage(stage + 2, 0, s2, s1);
        if (stage + 3 < nstages) run_stage(stage + 3, 1, s0, s2);
        if (stage + 4 < nstages) run_stage(stage + 4, 0, s1, s0);
        if (stage + 5 < nstages) run_stage(stage + 5, 1, s2, s1);
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

int ilog2f4(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

hipError_t launch_mfma_fp4_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                                int64_t lds_a, int beta_a, const uint32_t *b_bits,
                                const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    const int G = beta_a < beta_w ? beta_a : beta_w;
    if (G < 64) return hipErrorNotSupported;   // one MFMA step is 64 bits of K
    MfmaFp4Args a{};
    a.a_bits = a_bits; a.b_bits = b_bits; a.a_scales = a_scales; a.b_scales = b_scales;
    a.C = C; a.ldc = ldc;
    a.ldw_a = (int32_t)ldw_a; a.ldw_b = (int32_t)ldw_b; a.lds_a = (int32_t)lds_a; a.lds_b = (int32_t)lds_b;
    a.M = (int32_t)M; a.N = (int32_t)N; a.kwords = (int32_t)(K / 32);
    a.shift_a = ilog2f4(beta_a / G);
    a.shift_b = ilog2f4(beta_w / G);
    // 256-row workgroups, or 128-row ones (twice as many, two per CU; same speed on large problems)
    // when the larger tile would leave compute units without a workgroup
    const int64_t tiles_n = (N + kBN4 - 1) / kBN4;
    const bool small = ((M + 255) / 256) * tiles_n < 256;
    const int bm = small ? 128 : 256;
    const int64_t tiles_m = (M + bm - 1) / bm;
    if (tiles_m * tiles_n > 0x7fffff00LL) return hipErrorInvalidConfiguration;
    const int64_t nblocks = xcd_map_blocks(tiles_m * tiles_n);
    a.tiles_m = (int32_t)tiles_m; a.tiles_n = (int32_t)tiles_n;
    const dim3 grid((unsigned)nblocks), block(2 * bm);
#define HBMM_FP4_LAUNCH(SEGV)                                          \
    do {                                                               \
        if (small)                                                     \
            mfma_fp4_gemm_kernel<SEGV, 128><<<grid, block, 0, s>>>(a); \
        else                                                           \
            mfma_fp4_gemm_kernel<SEGV, 256><<<grid, block, 0, s>>>(a); \
    } while (0)
    if (G == 256)
        HBMM_FP4_LAUNCH(1);
    else if (G == 128)
        HBMM_FP4_LAUNCH(2);
    else
        HBMM_FP4_LAUNCH(4);
#undef HBMM_FP4_LAUNCH
    return hipGetLastError();
}

}  // namespace hbmm
