// int8 +-1 matrix-core variant of the HBMM contraction (Eq. 7 of HadaNets), kept as a comparison
// point for the XNOR + popcount kernel: the segment dot products d[m, n, g] come out of
// v_mfma_i32_32x32x32_i8 on operands expanded from the packed bits to +-1 bytes, and the same
// fp32 block-scale epilogue is applied.  Integer work is exact, so d is identical to the popcount
// kernel's and the outputs differ only by the order of the same fp32 roundings.
//
// Workgroup = 4 waves (2 x 2), tile 128 (M) x 128 (N), two workgroups per CU; wave = 64 x 64 = 2 x 2 MFMA
// tiles.  K is walked in stages of 128 bits.  Each thread owns one row of one operand tile: it
// fetches the row's 4 packed words and the scales of the segments inside the stage, and while
// parking the stage in LDS expands every nibble into four +-1 bytes with a 16-entry table held in
// LDS (16 consecutive banks: any mix of indices is conflict-free), so the expansion is done once
// per workgroup and shared by the two waves that use the row.  The 16-byte chunks of a row are
// XOR-swizzled with the row number, so the fragment reads of 8 consecutive rows (lane l feeds row
// l mod 32 and the 16 consecutive k at 16 * (l div 32)) hit distinct banks without padding.
// At the end of a segment of G = min(beta_a, beta_w) bits:
//   C += float(d) * (sA[m] * sB[n]),   then the integer accumulator restarts from zero (the same
// rounding steps as the popcount kernel, so the two give bit-identical outputs).
#include "kernels.h"

namespace hbmm {
namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBMi = 128, kBNi = 128;
constexpr int kThreadsI = 256;
constexpr int kStageWords = 4;    // 128 bits of K per stage
constexpr int kMaxSeg = 4;        // segments per stage at G = 32
constexpr int kRowBytesI = kStageWords * 32;   // one +-1 byte per bit

struct MfmaI8Args {
    const uint32_t *a_bits, *b_bits;
    const float *a_scales, *b_scales;
    float *C;
    int64_t ldc;
    int32_t ldw_a, ldw_b, lds_a, lds_b;
    int32_t M, N, kwords;       // kwords = K / 32
    int32_t log2_g;             // log2(G), G in {32, 64, 128, 256}
    int32_t shift_a, shift_b;   // log2(beta / G)
    int32_t tiles_n;
};

__global__ __launch_bounds__(kThreadsI, 2) void mfma_i8_gemm_kernel(const MfmaI8Args a)
{
    __shared__ __attribute__((aligned(16))) unsigned char s_bytes[2][2][kBMi * kRowBytesI];   // [buf][operand][row][128 swizzled bytes]
    __shared__ __attribute__((aligned(16))) float s_scale[2][2][kMaxSeg][kBMi];          // [buf][operand][seg][row]
    __shared__ uint32_t s_lut[16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = (blockIdx.x / a.tiles_n) * kBMi, n0 = (blockIdx.x % a.tiles_n) * kBNi;
    const int nstages = (a.kwords + kStageWords - 1) / kStageWords;
    const int G = 1 << a.log2_g;
    const int words_per_seg = G >> 5;
    // segments that end inside one stage (0 when a segment spans two stages)
    const int seg_per_stage = (kStageWords * 32) >> a.log2_g;

    if (tid < 16) {
        // nibble -> four bytes, bit 1 -> 0x01 (+1), bit 0 -> 0xff (-1)
        uint32_t v = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) v |= (((tid >> b) & 1) ? 0x01u : 0xffu) << (8 * b);
        s_lut[tid] = v;
    }

    // ---- staging: thread t handles row (t mod 128) of operand (t div 128)
    const int op = tid >> 7, srow = tid & 127;
    const bool row_ok = op == 0 ? (m0 + srow < a.M) : (n0 + srow < a.N);
    const uint32_t *gbits = op == 0 ? a.a_bits + (int64_t)min(m0 + srow, a.M - 1) * a.ldw_a
                                    : a.b_bits + (int64_t)min(n0 + srow, a.N - 1) * a.ldw_b;
    const float *gscale = op == 0 ? a.a_scales + (int64_t)min(m0 + srow, a.M - 1) * a.lds_a
                                  : a.b_scales + (int64_t)min(n0 + srow, a.N - 1) * a.lds_b;
    const int shift_op = op == 0 ? a.shift_a : a.shift_b;
    const int nseg_total = a.kwords / words_per_seg;            // K / G
    const int nseg_stage = seg_per_stage > 0 ? seg_per_stage : 1;
    // Loads are unconditional (indices clamped, results masked afterwards) so that the compiler knows
    // how many are outstanding and three stages can be in flight; they rotate through three sets.
    struct Staged {
        uint4 bits;
        float scale[kMaxSeg];
    };
    auto fetch = [&](Staged &st, int stage) {
        const int sg = min(stage, nstages - 1);
        st.bits = *reinterpret_cast<const uint4 *>(gbits + sg * kStageWords);   // ldw is a multiple of 4, pad words are zero
#pragma unroll
        for (int s = 0; s < kMaxSeg; ++s) {
            // segment s of this stage: global index gseg, this operand's block gseg >> shift
            const int gseg = seg_per_stage > 0 ? sg * seg_per_stage + s : sg >> 1;
            st.scale[s] = gscale[min(gseg, nseg_total - 1) >> shift_op];
        }
    };
    auto park = [&](const Staged &st, int stage, int buf) {
        // 4 words -> 8 chunks of 16 bytes; chunk c of row r lives at position c ^ (r & 7)
        unsigned char *dst = &s_bytes[buf][op][srow * kRowBytesI];
        const uint32_t wds[4] = {st.bits.x, st.bits.y, st.bits.z, st.bits.w};
#pragma unroll
        for (int c = 0; c < 2 * kStageWords; ++c) {
            const uint32_t h = wds[c >> 1] >> (16 * (c & 1));
            i32x4 v;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (int)s_lut[(h >> (4 * i)) & 15u];
            *reinterpret_cast<i32x4 *>(dst + ((c ^ (srow & 7)) << 4)) = v;
        }
        // a scale of 0 switches off segments past K (pad words expand to -1 bytes and would count) and rows past M / N
#pragma unroll
        for (int s = 0; s < kMaxSeg; ++s) {
            const int gseg = seg_per_stage > 0 ? stage * seg_per_stage + s : stage >> 1;
            const bool live = row_ok && s < nseg_stage && gseg < nseg_total;
            s_scale[buf][op][s][srow] = live ? st.scale[s] : 0.f;
        }
    };

    i32x16 acc[2][2];
    f32x16 res[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[x][y][v] = 0;
                res[x][y][v] = 0.f;
            }

    auto run_stage = [&](int stage, const Staged &ready, Staged &incoming) {
        const int buf = stage & 1;
        fetch(incoming, stage + 3);

        const int rl = lane & 31, hi = lane >> 5;
#pragma unroll
        for (int w = 0; w < kStageWords; ++w) {
            i32x4 fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int ra = wm * 64 + t * 32 + rl, rb = wn * 64 + t * 32 + rl;
                fa[t] = *reinterpret_cast<const i32x4 *>(&s_bytes[buf][0][ra * kRowBytesI + (((2 * w + hi) ^ (ra & 7)) << 4)]);
                fb[t] = *reinterpret_cast<const i32x4 *>(&s_bytes[buf][1][rb * kRowBytesI + (((2 * w + hi) ^ (rb & 7)) << 4)]);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[x], fb[y], acc[x][y], 0, 0, 0);

            const int wglob = stage * kStageWords + w;
            if (((wglob + 1) & (words_per_seg - 1)) == 0) {
                // the segment that ends here; its slot among this stage's staged scales
                const int s = seg_per_stage > 0 ? (w >> (a.log2_g - 5)) : 0;
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    const float sb = s_scale[buf][1][s][wn * 64 + y * 32 + (lane & 31)];
#pragma unroll
                    for (int x = 0; x < 2; ++x) {
                        const float *sa = &s_scale[buf][0][s][wm * 64 + x * 32 + 4 * (lane >> 5)];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4 sa4 = *reinterpret_cast<const float4 *>(sa + 8 * q);
                            res[x][y][4 * q + 0] = __builtin_fmaf((float)acc[x][y][4 * q + 0], sa4.x * sb, res[x][y][4 * q + 0]);
                            res[x][y][4 * q + 1] = __builtin_fmaf((float)acc[x][y][4 * q + 1], sa4.y * sb, res[x][y][4 * q + 1]);
                            res[x][y][4 * q + 2] = __builtin_fmaf((float)acc[x][y][4 * q + 2], sa4.z * sb, res[x][y][4 * q + 2]);
                            res[x][y][4 * q + 3] = __builtin_fmaf((float)acc[x][y][4 * q + 3], sa4.w * sb, res[x][y][4 * q + 3]);
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[x][y][v] = 0;
                    }
                }
            }
        }
        park(ready, stage + 1, buf ^ 1);   // past the last stage this parks data that nobody reads
        __syncthreads();
    };

    Staged s0, s1, s2;
    fetch(s0, 0);
    __syncthreads();   // the table must be complete before the first expansion reads it
    park(s0, 0, 0);
    fetch(s0, 1);
    fetch(s1, 2);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 3) {
        run_stage(stage, s0, s2);
        if (stage + 1 < nstages) run_stage(stage + 1, s1, s0);
        if (stage + 2 < nstages) run_stage(stage + 2, s2, s1);
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

int ilog2(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

hipError_t launch_mfma_i8_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                               int64_t lds_a, int beta_a, const uint32_t *b_bits,
                               const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                               int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s)
{
    const int G = beta_a < beta_w ? beta_a : beta_w;
    MfmaI8Args a{};
    a.a_bits = a_bits; a.b_bits = b_bits; a.a_scales = a_scales; a.b_scales = b_scales;
    a.C = C; a.ldc = ldc;
    a.ldw_a = (int32_t)ldw_a; a.ldw_b = (int32_t)ldw_b; a.lds_a = (int32_t)lds_a; a.lds_b = (int32_t)lds_b;
    a.M = (int32_t)M; a.N = (int32_t)N; a.kwords = (int32_t)(K / 32);
    a.log2_g = ilog2(G);
    a.shift_a = ilog2(beta_a / G);
    a.shift_b = ilog2(beta_w / G);
    const int64_t tiles_m = (M + kBMi - 1) / kBMi, tiles_n = (N + kBNi - 1) / kBNi;
    if (tiles_m * tiles_n > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.tiles_n = (int32_t)tiles_n;
    mfma_i8_gemm_kernel<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreadsI), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace hbmm
