// int8 +-1 matrix-core variant of the HBMM contraction (Eq. 7 of HadaNets), kept as a comparison
// point for the XNOR + popcount kernel: the segment dot products d[m, n, g] come out of
// v_mfma_i32_32x32x32_i8 on operands expanded from the packed bits to +-1 bytes, and the same
// fp32 block-scale epilogue is applied.  Integer work is exact, so the result differs from the
// popcount kernel only by nothing at all in d and by the same fp32 roundings in the epilogue.
//
// Workgroup = 4 waves (2 x 2), tile 128 (M) x 128 (N); wave = 64 x 64 = 2 x 2 MFMA tiles.  K is walked
// in stages of 128 bits: the 4 packed words of every row of both operand tiles (4 KB in all) and
// the scales of the segments inside the stage go through LDS.  For each 32-bit step a lane takes
// its 16 bits (lane l feeds row l mod 32 and the 16 consecutive k at 16 * (l div 32)), and turns
// each nibble into four +-1 bytes with a 16-entry table held in LDS (16 consecutive banks: any
// mix of indices is conflict-free).  At the end of a segment of G = min(beta_a, beta_w) bits:
//   C += float(d) * sA[m] * sB[n],   then the integer accumulator restarts from zero.
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

__global__ __launch_bounds__(kThreadsI) void mfma_i8_gemm_kernel(const MfmaI8Args a)
{
    __shared__ __attribute__((aligned(16))) uint32_t s_bits[2][2][kBMi * kStageWords];   // [buf][operand][row*4 + w]
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
    uint4 st_bits;
    float st_scale[kMaxSeg];
    auto fetch = [&](int stage) {
        st_bits = make_uint4(0, 0, 0, 0);
        if (row_ok && stage * kStageWords < a.kwords)   // ldw is a multiple of 4 and pad words are zero
            st_bits = *reinterpret_cast<const uint4 *>(gbits + stage * kStageWords);
        // scale of segment s of this stage: global segment index gseg, operand block gseg >> shift
#pragma unroll
        for (int s = 0; s < kMaxSeg; ++s) {
            st_scale[s] = 0.f;
            const int nseg = seg_per_stage > 0 ? seg_per_stage : 1;
            if (s < nseg) {
                const int gseg = seg_per_stage > 0 ? stage * seg_per_stage + s : stage >> 1;
                if (row_ok && gseg * words_per_seg < a.kwords) st_scale[s] = gscale[gseg >> shift_op];
            }
        }
    };
    auto park = [&](int buf) {
        *reinterpret_cast<uint4 *>(&s_bits[buf][op][srow * kStageWords]) = st_bits;
#pragma unroll
        for (int s = 0; s < kMaxSeg; ++s) s_scale[buf][op][s][srow] = st_scale[s];
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

    // 16 bits -> 16 bytes of +-1 through the nibble table
    auto expand16 = [&](uint32_t bits16) {
        i32x4 f;
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = (int)s_lut[(bits16 >> (4 * i)) & 15u];
        return f;
    };

    fetch(0);
    park(0);
    __syncthreads();
    for (int stage = 0; stage < nstages; ++stage) {
        const int buf = stage & 1;
        if (stage + 1 < nstages) fetch(stage + 1);

        uint4 wa[2], wb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            wa[t] = *reinterpret_cast<const uint4 *>(&s_bits[buf][0][(wm * 64 + t * 32 + (lane & 31)) * kStageWords]);
            wb[t] = *reinterpret_cast<const uint4 *>(&s_bits[buf][1][(wn * 64 + t * 32 + (lane & 31)) * kStageWords]);
        }
        const int half = (lane >> 5) * 16;
#pragma unroll
        for (int w = 0; w < kStageWords; ++w) {
            i32x4 fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t xa = w == 0 ? wa[t].x : w == 1 ? wa[t].y : w == 2 ? wa[t].z : wa[t].w;
                const uint32_t xb = w == 0 ? wb[t].x : w == 1 ? wb[t].y : w == 2 ? wb[t].z : wb[t].w;
                fa[t] = expand16((xa >> half) & 0xffffu);
                fb[t] = expand16((xb >> half) & 0xffffu);
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
                            res[x][y][4 * q + 0] = __builtin_fmaf((float)acc[x][y][4 * q + 0] * sa4.x, sb, res[x][y][4 * q + 0]);
                            res[x][y][4 * q + 1] = __builtin_fmaf((float)acc[x][y][4 * q + 1] * sa4.y, sb, res[x][y][4 * q + 1]);
                            res[x][y][4 * q + 2] = __builtin_fmaf((float)acc[x][y][4 * q + 2] * sa4.z, sb, res[x][y][4 * q + 2]);
                            res[x][y][4 * q + 3] = __builtin_fmaf((float)acc[x][y][4 * q + 3] * sa4.w, sb, res[x][y][4 * q + 3]);
                        }
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[x][y][v] = 0;
                    }
                }
            }
        }
        if (stage + 1 < nstages) park(buf ^ 1);
        __syncthreads();
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
