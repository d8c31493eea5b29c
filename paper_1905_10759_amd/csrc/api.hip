// C-ABI layer of libhbmm: argument validation and dispatch.  See include/hbmm.h for the contract.
// Nothing here allocates, frees or synchronises; every path either returns an error before any
// launch or enqueues its kernels on the caller's stream.
#include "../../include/hbmm.h"
#include "kernels.h"

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int log2_exact(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

bool supported_beta(int beta) { return beta == 32 || beta == 64 || beta == 128 || beta == 256; }
bool supported_pack_beta(int beta) { return beta >= 2 && beta <= 256 && (beta & (beta - 1)) == 0; }
// What the general (untuned) kernels take: any segment length up to 256, 1 = unquantised
bool any_beta(int beta) { return beta >= 1 && beta <= 256; }
constexpr int64_t kMaxAnyK = ((int64_t)1 << 24) - 1;   // their k div beta is a 32-bit multiply-high

int from_hip(hipError_t e)
{
    if (e == hipSuccess) return HBMM_OK;
    return e == hipErrorNotSupported ? HBMM_EUNSUPPORTED : HBMM_ELAUNCH;
}

// Zero an M x N block of 4-byte elements (K == 0 products).  A kernel rather than a memset so that
// the call can be captured into a HIP graph like every other launch of this library.
__global__ void zero_block_kernel(uint32_t *dst, int64_t ld, int64_t M, int64_t N)
{
    const int64_t total = M * N;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        dst[(i / N) * ld + i % N] = 0u;
}
hipError_t zero_block(void *dst, int64_t ld, int64_t M, int64_t N, hipStream_t s)
{
    const int64_t total = M * N;
    const unsigned blocks = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    zero_block_kernel<<<dim3(blocks), dim3(256), 0, s>>>(static_cast<uint32_t *>(dst), ld, M, N);
    return hipGetLastError();
}

constexpr int64_t kMaxDim = (int64_t)1 << 30;   // rows, K: index arithmetic stays inside 32/64 bits
constexpr int64_t kMaxPackK = (int64_t)1 << 26; // pack: K and k-offsets inside a row are 32-bit
constexpr int64_t kMaxPackColsK = (int64_t)65535 * 256;   // layout 1 walks K in gridDim.y slices of 256

}  // namespace

extern "C" {

const char *hbmm_strerror(int code)
{
    switch (code) {
    case HBMM_OK: return "ok";
    case HBMM_EINVAL: return "invalid argument (null or misaligned pointer, bad shape or leading dimension)";
    case HBMM_EUNSUPPORTED: return "unsupported beta, K, algo or dtype";
    case HBMM_ELAUNCH: return "HIP error at kernel launch";
    }
    return "unknown hbmm error code";
}

int64_t hbmm_num_blocks(int64_t K, int32_t beta)
{
    if (K < 0 || beta < 1) return 0;
    return (K + beta - 1) / beta;
}

int64_t hbmm_packed_ld_words(int64_t K)
{
    if (K < 0) return 0;
    return hbmm::packed_words(K);
}

int hbmm_quantize_pack(const float *x, int64_t rows, int64_t K, int64_t ldx, int32_t layout,
                       int32_t beta, uint32_t *bits, int64_t ldw, float *scales, int64_t lds,
                       void *stream)
{
    if (rows < 0 || K < 0 || rows > kMaxDim || K > kMaxPackK) return HBMM_EINVAL;
    if (layout != 0 && layout != 1) return HBMM_EINVAL;
    if (beta < 1) return HBMM_EINVAL;
    if (beta == 1 || !any_beta(beta)) return HBMM_EUNSUPPORTED;
    // the tuned kernels take the paper's settings (power-of-two segments that divide K, whole words);
    // everything else goes to the general kernel
    const bool tuned = supported_pack_beta(beta) && K % beta == 0 && K % 32 == 0;
    if (tuned && layout == 1 && K > kMaxPackColsK) return HBMM_EINVAL;
    if (rows == 0 || K == 0) return HBMM_OK;
    if (!x || !bits || !scales) return HBMM_EINVAL;
    if (!aligned16(x) || !aligned16(bits) || !aligned16(scales)) return HBMM_EINVAL;
    if (ldx < (layout == 0 ? K : rows)) return HBMM_EINVAL;
    if (ldw < hbmm::packed_words(K) || ldw % 4 != 0) return HBMM_EINVAL;
    if (lds < (K + beta - 1) / beta) return HBMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!tuned) return from_hip(hbmm::launch_pack_any(x, rows, K, ldx, layout, beta, bits, ldw, scales, lds, s));
    if (layout == 0) return from_hip(hbmm::launch_pack_rows(x, rows, K, ldx, beta, bits, ldw, scales, lds, s));
    return from_hip(hbmm::launch_pack_cols(x, rows, K, ldx, beta, bits, ldw, scales, lds, s));
}

int hbmm_binarize_backward(const float *x, const float *grad_out, int64_t rows, int64_t K, int64_t ldx,
                           int64_t ldg, int32_t beta, float *grad_in, int64_t ldgi, void *stream)
{
    if (rows < 0 || K < 0 || rows > kMaxDim || K > kMaxPackK) return HBMM_EINVAL;
    if (beta < 1) return HBMM_EINVAL;
    if (!any_beta(beta)) return HBMM_EUNSUPPORTED;
    // the tuned kernel takes the paper's settings; any other segment length or K goes to the general one
    const bool tuned = (beta == 1 || supported_pack_beta(beta)) && K % beta == 0 && K % 4 == 0;
    if (rows == 0 || K == 0) return HBMM_OK;
    if (!x || !grad_out || !grad_in) return HBMM_EINVAL;
    if (!aligned16(x) || !aligned16(grad_out) || !aligned16(grad_in)) return HBMM_EINVAL;
    if (ldx < K || ldg < K || ldgi < K) return HBMM_EINVAL;
    if (!tuned)
        return from_hip(hbmm::launch_binarize_backward_any(x, grad_out, rows, K, ldx, ldg, beta, grad_in, ldgi,
                                                           static_cast<hipStream_t>(stream)));
    return from_hip(hbmm::launch_binarize_backward(x, grad_out, rows, K, ldx, ldg, beta, grad_in, ldgi,
                                                   static_cast<hipStream_t>(stream)));
}

static int check_packed(const uint32_t *bits, int64_t rows, int64_t K, int64_t ldw)
{
    if (!bits || !aligned16(bits)) return HBMM_EINVAL;
    if (ldw < hbmm::packed_words(K) || ldw % 4 != 0) return HBMM_EINVAL;
    if (rows * ldw >= ((int64_t)1 << 29)) return HBMM_EINVAL;   // byte offsets of rows fit 32 bits
    return HBMM_OK;
}

// Pick which operand is held per lane (tile 128) and which is broadcast (tile 64): the one that
// wastes fewer padded outputs; B per lane is preferred because then a wave stores along a row of C.
static bool b_is_lane_side(int64_t M, int64_t N)
{
    auto up = [](int64_t v, int64_t t) { return (v + t - 1) / t * t; };
    const double cost_b = (double)up(N, 128) * (double)up(M, 64);
    const double cost_a = (double)up(M, 128) * (double)up(N, 64) * 1.05;
    return cost_b <= cost_a;
}

// One operand of hbmm_gemm as the caller gave it; beta == 1 means `scales` is the raw fp32 operand.
struct GemmOperand {
    const uint32_t *bits;
    const float *scales;
    int64_t ldw, lds, rows;
    int32_t beta;
};

static int check_operand(const GemmOperand &o, int64_t K)
{
    if (!o.scales || !aligned16(o.scales)) return HBMM_EINVAL;
    if (o.lds >= ((int64_t)1 << 31)) return HBMM_EINVAL;
    if (o.beta == 1) {
        if (o.bits != nullptr) return HBMM_EINVAL;     // raw operand travels through `scales`
        return o.lds < K ? HBMM_EINVAL : HBMM_OK;
    }
    if (o.lds < (K + o.beta - 1) / o.beta) return HBMM_EINVAL;
    return check_packed(o.bits, o.rows, K, o.ldw);
}

static hbmm::SplitGemmOperand to_split(const GemmOperand &o)
{
    hbmm::SplitGemmOperand r{};
    if (o.beta == 1) {
        r.raw = o.scales;
        r.ld_raw = o.lds;
    } else {
        r.bits = o.bits;
        r.scales = o.scales;
        r.ldw = o.ldw;
        r.lds = o.lds;
    }
    r.rows = o.rows;
    r.beta = o.beta;
    return r;
}

int hbmm_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a, int64_t lds_a,
              int32_t beta_a, const uint32_t *b_bits, const float *b_scales, int64_t ldw_b,
              int64_t lds_b, int32_t beta_w, int64_t M, int64_t N, int64_t K, float *C, int64_t ldc,
              int32_t algo, void *stream)
{
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return HBMM_EINVAL;
    if (beta_a < 1 || beta_w < 1) return HBMM_EINVAL;
    if (algo < -1 || algo > 3) return HBMM_EUNSUPPORTED;
    // -1: whichever kernel is fastest for these segment lengths
    if (algo == -1) {
        const int g = beta_a < beta_w ? beta_a : beta_w;
        const int gmax = beta_a < beta_w ? beta_w : beta_a;
        // (a short segment against a long one is as fast on the bf16 kernel: its epilogue is rare there)
        algo = g >= 64 ? 2 : (g >= 16 && gmax <= 32 && K % 128 == 0) ? 3 : 0;
        // The matrix-core variants work on 128 x 128 tiles at least; on a grid of a few tiles the popcount
        // kernel, which has a 64-row form for small grids, is as fast or faster (64 x 64 x 512: 11 against 18 us).
        if (algo >= 2 && beta_a >= 32 && beta_w >= 32 && ((M + 127) / 128) * ((N + 127) / 128) < 32) algo = 0;
    }
    const bool word_a = supported_beta(beta_a), word_w = supported_beta(beta_w);   // 32 .. 256
    if (!any_beta(beta_a) || !any_beta(beta_w)) return HBMM_EUNSUPPORTED;
    // The paper's settings: power-of-two segments that divide K (and whole 32-bit words).  Anything else
    // -- other segment lengths, a shorter last segment, K not a multiple of 32 -- is the general path below.
    const bool tuned = (beta_a == 1 || supported_pack_beta(beta_a)) && (beta_w == 1 || supported_pack_beta(beta_w)) &&
                       K % beta_w == 0 && K % beta_a == 0 && K % 32 == 0 &&
                       (beta_a != 1 || lds_a % 4 == 0) && (beta_w != 1 || lds_b % 4 == 0);   // 16-byte row loads
    // (word-sized power-of-two segments with a K that they or 32 do not divide: the popcount kernel itself, whose
    // tail loop takes the shorter last segment; the matrix-core variants do not)
    const bool popcount_any_k = word_a && word_w && !tuned;
    if (popcount_any_k && algo == -1) algo = 0;
    if (!tuned && (algo > 0 || (K > kMaxAnyK && !popcount_any_k))) return HBMM_EUNSUPPORTED;
    if ((algo == 1 || algo == 2) && !(word_a && word_w)) return HBMM_EUNSUPPORTED;
    if (algo == 2 && (beta_a < 64 || beta_w < 64)) return HBMM_EUNSUPPORTED;   // one fp4 MFMA step is 64 bits of K
    if (algo == 3) {
        // one fp8 MFMA step is 16 bits of K; the kernel is written for segments of 16 or 32 and whole 128-bit stages
        const int g = beta_a < beta_w ? beta_a : beta_w;
        if (beta_a < 16 || beta_w < 16 || g > 32 || K % 128 != 0) return HBMM_EUNSUPPORTED;
    }
    // Two unquantised operands are a plain dense product (hbmm_dense_ref_gemm).
    if (beta_a == 1 && beta_w == 1) return HBMM_EUNSUPPORTED;
    if (M == 0 || N == 0) return HBMM_OK;
    if (!C || !aligned16(C) || ldc < N) return HBMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (K == 0) return from_hip(zero_block(C, ldc, M, N, s));

    const GemmOperand oa{a_bits, a_scales, ldw_a, lds_a, M, beta_a};
    const GemmOperand ob{b_bits, b_scales, ldw_b, lds_b, N, beta_w};
    if (int rc = check_operand(ob, K)) return rc;
    if (int rc = check_operand(oa, K)) return rc;

    if (!tuned && !popcount_any_k) {
        // both sides rebuilt as fp32 values element by element; an unquantised operand is the "x" side
        if (beta_w != 1) return from_hip(hbmm::launch_mfma_split_any(to_split(oa), to_split(ob), K, C, ldc, 1, s));
        return from_hip(hbmm::launch_mfma_split_any(to_split(ob), to_split(oa), K, C, 1, ldc, s));
    }

    if (algo == 3)
        return from_hip(hbmm::launch_mfma_fp8_gemm(a_bits, a_scales, ldw_a, lds_a, beta_a, b_bits, b_scales,
                                                   ldw_b, lds_b, beta_w, M, N, K, C, ldc, s));

    if (!(word_a && word_w)) {
        // Matrix-core path.  The operand with the longer segment (at least 16) keeps its signs and has
        // its scale applied once per segment; the other one is rebuilt as fp32 values.  If neither
        // segment reaches 16 both are rebuilt; an unquantised operand is always the rebuilt ("x") side.
        const bool b_is_y = beta_a == 1 ? true
                          : beta_w == 1 ? false
                          : (beta_a < 16 && beta_w < 16) ? true
                          : beta_w >= 16 && (beta_w >= beta_a || beta_a < 16);
        if (b_is_y)
            return from_hip(hbmm::launch_mfma_split_gemm(to_split(oa), to_split(ob), K, C, ldc, 1, s));
        return from_hip(hbmm::launch_mfma_split_gemm(to_split(ob), to_split(oa), K, C, 1, ldc, s));
    }

    if (algo == 1)
        return from_hip(hbmm::launch_mfma_i8_gemm(a_bits, a_scales, ldw_a, lds_a, beta_a, b_bits, b_scales,
                                                  ldw_b, lds_b, beta_w, M, N, K, C, ldc, s));
    if (algo == 2)
        return from_hip(hbmm::launch_mfma_fp4_gemm(a_bits, a_scales, ldw_a, lds_a, beta_a, b_bits, b_scales,
                                                   ldw_b, lds_b, beta_w, M, N, K, C, ldc, s));

    const int G = beta_a < beta_w ? beta_a : beta_w;
    hbmm::PopcountGemmArgs g{};
    const bool b_lane = b_is_lane_side(M, N);
    if (b_lane) {
        g.p_bits = b_bits; g.p_scales = b_scales; g.ldw_p = (int32_t)ldw_b; g.lds_p = (int32_t)lds_b;
        g.P = (int32_t)N; g.shift_p = log2_exact(beta_w / G);
        g.q_bits = a_bits; g.q_scales = a_scales; g.ldw_q = (int32_t)ldw_a; g.lds_q = (int32_t)lds_a;
        g.Q = (int32_t)M; g.shift_q = log2_exact(beta_a / G);
        g.ld_out_p = 1; g.ld_out_q = ldc;
    } else {
        g.p_bits = a_bits; g.p_scales = a_scales; g.ldw_p = (int32_t)ldw_a; g.lds_p = (int32_t)lds_a;
        g.P = (int32_t)M; g.shift_p = log2_exact(beta_a / G);
        g.q_bits = b_bits; g.q_scales = b_scales; g.ldw_q = (int32_t)ldw_b; g.lds_q = (int32_t)lds_b;
        g.Q = (int32_t)N; g.shift_q = log2_exact(beta_w / G);
        g.ld_out_p = ldc; g.ld_out_q = 1;
    }
    g.out = C;
    g.kwords = (int32_t)hbmm::packed_words(K);
    g.ngran = (int32_t)(K / G);
    g.tail_bits = (int32_t)(K % G);
    g.kw_used = (int32_t)((K + 31) / 32);
    g.nblk_p = (int32_t)((K + (G << g.shift_p) - 1) / (G << g.shift_p));
    g.nblk_q = (int32_t)((K + (G << g.shift_q) - 1) / (G << g.shift_q));
    g.K = (int32_t)K;
    return from_hip(hbmm::launch_popcount_gemm(g, G, 0, s));
}

int hbmm_gemm_fused(const float *A, int64_t lda, int32_t beta_a, const uint32_t *b_bits,
                    const float *b_scales, int64_t ldw_b, int64_t lds_b, int32_t beta_w, int64_t M,
                    int64_t N, int64_t K, float *C, int64_t ldc, void *stream)
{
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return HBMM_EINVAL;
    if (beta_a < 1 || beta_w < 1) return HBMM_EINVAL;
    if (!supported_beta(beta_a) || !supported_beta(beta_w)) return HBMM_EUNSUPPORTED;
    if (K % beta_a != 0 || K % beta_w != 0) return HBMM_EUNSUPPORTED;
    if (N > 128) return HBMM_EUNSUPPORTED;
    if (M == 0 || N == 0) return HBMM_OK;
    if (!C || !aligned16(C) || ldc < N) return HBMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (K == 0) return from_hip(zero_block(C, ldc, M, N, s));
    if (!A || !aligned16(A) || lda < K || lda % 4 != 0) return HBMM_EINVAL;
    if (!b_scales || !aligned16(b_scales) || lds_b < K / beta_w || lds_b >= ((int64_t)1 << 31)) return HBMM_EINVAL;
    if (int rc = check_packed(b_bits, N, K, ldw_b)) return rc;

    const int G = beta_a < beta_w ? beta_a : beta_w;
    hbmm::PopcountGemmArgs g{};
    g.p_src = A; g.ld_p_src = lda; g.beta_p = beta_a;
    g.P = (int32_t)M; g.shift_p = log2_exact(beta_a / G);
    g.q_bits = b_bits; g.q_scales = b_scales; g.ldw_q = (int32_t)ldw_b; g.lds_q = (int32_t)lds_b;
    g.Q = (int32_t)N; g.shift_q = log2_exact(beta_w / G);
    g.ld_out_p = ldc; g.ld_out_q = 1;
    g.out = C;
    g.kwords = (int32_t)hbmm::packed_words(K);
    g.ngran = (int32_t)(K / G);
    g.tail_bits = (int32_t)(K % G);
    g.kw_used = (int32_t)((K + 31) / 32);
    g.nblk_p = (int32_t)((K + (G << g.shift_p) - 1) / (G << g.shift_p));
    g.nblk_q = (int32_t)((K + (G << g.shift_q) - 1) / (G << g.shift_q));
    g.K = (int32_t)K;
    return from_hip(hbmm::launch_popcount_gemm(g, G, 0, s));
}

// The 2-D view (rows x K) under which a flat tensor of `count` elements is packed: K the largest
// power of two <= 4096 that divides count.  With K a multiple of 128 the packed rows carry no
// padding, so the words and scales of the view are those of the flat tensor.
static int64_t tensor_view_k(int64_t count)
{
    int64_t k = 4096;
    while (k > 1 && count % k != 0) k >>= 1;
    return k;
}

int hbmm_quantize_pack_tensor(const float *x, int64_t count, int32_t beta, uint32_t *bits, float *scales,
                              void *stream)
{
    if (count < 0 || count > ((int64_t)1 << 31) - 1) return HBMM_EINVAL;
    if (beta < 1) return HBMM_EINVAL;
    if (!supported_pack_beta(beta)) return HBMM_EUNSUPPORTED;
    const int64_t K = tensor_view_k(count);
    if (count == 0) return HBMM_OK;
    if (K < 128 || K % beta != 0) return HBMM_EUNSUPPORTED;
    return hbmm_quantize_pack(x, count / K, K, K, 0, beta, bits, K / 32, scales, K / beta, stream);
}

int hbmm_quantize_pack_activations(const float *x, int64_t rows, int64_t W, int32_t beta, uint32_t *bits, float *scales,
                                   void *stream)
{
    if (rows < 0 || W < 0 || rows > kMaxDim || W > kMaxDim) return HBMM_EINVAL;
    if ((double)rows * (double)W > 2147483647.0) return HBMM_EINVAL;
    if (beta < 1) return HBMM_EINVAL;
    if (beta == 1 || !any_beta(beta)) return HBMM_EUNSUPPORTED;
    if (rows == 0 || W == 0) return HBMM_OK;
    if (!x || !bits || !scales || !aligned16(x) || !aligned16(bits) || !aligned16(scales)) return HBMM_EINVAL;
    // widths that beta divides, in the tuned kernels' range: the flat view is the same layout
    const int64_t count = rows * W;
    if (supported_pack_beta(beta) && W % beta == 0 && count % 128 == 0 && tensor_view_k(count) % beta == 0)
        return hbmm_quantize_pack_tensor(x, count, beta, bits, scales, stream);
    return from_hip(hbmm::launch_pack_activations_any(x, rows, W, beta, bits, scales, static_cast<hipStream_t>(stream)));
}

int hbmm_binarize_backward_tensor(const float *x, const float *grad_out, int64_t count, int32_t beta, float *grad_in,
                                   void *stream)
{
    if (count < 0 || count > ((int64_t)1 << 31) - 1) return HBMM_EINVAL;
    if (beta < 1) return HBMM_EINVAL;
    if (!(beta == 1 || supported_pack_beta(beta))) return HBMM_EUNSUPPORTED;
    const int64_t K = tensor_view_k(count);
    if (count == 0) return HBMM_OK;
    if (K < 128 || K % beta != 0) return HBMM_EUNSUPPORTED;
    return hbmm_binarize_backward(x, grad_out, count / K, K, K, K, beta, grad_in, K, stream);
}

int hbmm_conv2d(const uint32_t *a_bits, const float *a_scales, int32_t beta_a, const uint32_t *w_bits,
                const float *w_scales, int64_t ldw_w, int64_t lds_w, int32_t beta_w, int64_t B, int64_t C,
                int64_t H, int64_t W, int64_t N, int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                float *out, int32_t algo, void *stream)
{
    if (algo != 0 && algo != 1) return HBMM_EINVAL;
    if (B < 0 || C < 0 || H < 0 || W < 0 || N < 0 || KH < 1 || KW < 1 || stride < 1 || pad < 0) return HBMM_EINVAL;
    if (B > kMaxDim || C > kMaxDim || H > kMaxDim || W > kMaxDim || N > kMaxDim) return HBMM_EINVAL;
    if (KH > 32 || KW > 32 || pad > 32 || stride > 32) return HBMM_EINVAL;
    if (beta_a < 1 || beta_w < 1) return HBMM_EINVAL;
    if (!(beta_a == 1 || supported_pack_beta(beta_a)) || !supported_pack_beta(beta_w)) return HBMM_EUNSUPPORTED;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return HBMM_EINVAL;
    const int64_t OH = (H + 2 * pad - KH) / stride + 1, OW = (W + 2 * pad - KW) / stride + 1;
    const int64_t K = C * KH * KW;
    if ((double)B * (double)C * (double)H * (double)W > 2147483647.0) return HBMM_EUNSUPPORTED;
    if ((double)B * (double)OH * (double)OW > 2147483647.0) return HBMM_EUNSUPPORTED;
    if (B == 0 || N == 0) return HBMM_OK;
    if (C == 0 || H == 0 || W == 0) return HBMM_EINVAL;
    if (W % beta_a != 0 || K % beta_w != 0 || K % 32 != 0 || KH * KW > 32) return HBMM_EUNSUPPORTED;
    if (!out || !aligned16(out)) return HBMM_EINVAL;
    if (!a_scales || !aligned16(a_scales)) return HBMM_EINVAL;
    if (beta_a == 1 ? a_bits != nullptr : (!a_bits || !aligned16(a_bits))) return HBMM_EINVAL;
    if (!w_scales || !aligned16(w_scales) || lds_w < K / beta_w) return HBMM_EINVAL;
    if (int rc = check_packed(w_bits, N, K, ldw_w)) return rc;
    hbmm::ConvActivations x{a_bits, a_scales, beta_a};
    hbmm::SplitGemmOperand y{};
    y.bits = w_bits; y.scales = w_scales; y.ldw = ldw_w; y.lds = lds_w; y.rows = N; y.beta = beta_w;
    hbmm::ConvGeometry g{B, C, H, W, KH, KW, stride, pad, algo};
    return from_hip(hbmm::launch_mfma_split_conv(x, y, g, out, static_cast<hipStream_t>(stream)));
}

// Shape checks shared by the two entry points of the prepared-filter convolution.
static int check_conv_filter_shape(int64_t N, int64_t C, int32_t KH, int32_t KW)
{
    if (N < 0 || C < 0 || KH < 1 || KW < 1 || N > kMaxDim || C > kMaxDim || KH > 32 || KW > 32) return HBMM_EINVAL;
    if ((double)C * KH * KW > (double)kMaxAnyK) return HBMM_EUNSUPPORTED;   // k div beta is a 32-bit multiply-high
    return HBMM_OK;
}

int64_t hbmm_conv_filter_pieces_bytes(int64_t N, int64_t C, int32_t KH, int32_t KW, int32_t form)
{
    if (check_conv_filter_shape(N, C, KH, KW) != HBMM_OK || form < 0 || form > 1) return 0;
    return hbmm::conv_filter_pieces_bytes(N, C, KH, KW, form);
}

int hbmm_conv_prepare_filters(const uint32_t *w_bits, const float *w_scales, int64_t ldw_w, int64_t lds_w,
                              int32_t beta_w, int64_t N, int64_t C, int32_t KH, int32_t KW, int32_t form, void *pieces,
                              void *stream)
{
    if (int rc = check_conv_filter_shape(N, C, KH, KW)) return rc;
    if (form < 0 || form > 1) return HBMM_EUNSUPPORTED;
    if (beta_w < 1) return HBMM_EINVAL;
    if (!any_beta(beta_w)) return HBMM_EUNSUPPORTED;
    if (N == 0 || C == 0) return HBMM_OK;
    const int64_t K = C * KH * KW;
    if (!pieces || !aligned16(pieces)) return HBMM_EINVAL;
    if (!w_scales || !aligned16(w_scales)) return HBMM_EINVAL;
    if (beta_w == 1) {
        if (w_bits != nullptr || lds_w < K) return HBMM_EINVAL;   // unquantised filters travel through w_scales
    } else {
        if (lds_w < (K + beta_w - 1) / beta_w) return HBMM_EINVAL;
        if (int rc = check_packed(w_bits, N, K, ldw_w)) return rc;
    }
    return from_hip(hbmm::launch_conv_prepare_filters(w_bits, w_scales, ldw_w, lds_w, beta_w, N, C, KH, KW, form, pieces,
                                                      static_cast<hipStream_t>(stream)));
}

int hbmm_conv2d_prepared(const uint32_t *a_bits, const float *a_scales, int32_t beta_a, const void *pieces, int32_t form,
                         int64_t B, int64_t C, int64_t H, int64_t W, int64_t N, int32_t KH, int32_t KW, int32_t stride,
                         int32_t pad, float *out, void *stream)
{
    if (form < 0 || form > 1) return HBMM_EUNSUPPORTED;
    if (B < 0 || H < 0 || W < 0 || stride < 1 || pad < 0 || B > kMaxDim || H > kMaxDim || W > kMaxDim) return HBMM_EINVAL;
    if (int rc = check_conv_filter_shape(N, C, KH, KW)) return rc;
    if (pad > 32 || stride > 32) return HBMM_EINVAL;
    if (beta_a < 1) return HBMM_EINVAL;
    if (!any_beta(beta_a)) return HBMM_EUNSUPPORTED;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return HBMM_EINVAL;
    const int64_t OH = (H + 2 * pad - KH) / stride + 1, OW = (W + 2 * pad - KW) / stride + 1;
    if ((double)B * (double)C * (double)H * (double)W > 2147483647.0) return HBMM_EUNSUPPORTED;
    if ((double)B * (double)OH * (double)OW * (double)(N > 0 ? N : 1) > 9.0e18) return HBMM_EUNSUPPORTED;
    if ((double)B * (double)OH * (double)OW > 2147483647.0) return HBMM_EUNSUPPORTED;
    if (B == 0 || N == 0) return HBMM_OK;
    if (C == 0 || H == 0 || W == 0) return HBMM_EINVAL;
    hbmm::ConvGeometry g{B, C, H, W, KH, KW, stride, pad, 0};
    if (!hbmm::conv_direct_fits(g)) return HBMM_EUNSUPPORTED;
    if (!out || !aligned16(out)) return HBMM_EINVAL;
    if (!pieces || !aligned16(pieces)) return HBMM_EINVAL;
    if (!a_scales || !aligned16(a_scales)) return HBMM_EINVAL;
    if (beta_a == 1 ? a_bits != nullptr : (!a_bits || !aligned16(a_bits))) return HBMM_EINVAL;
    hbmm::ConvActivations x{a_bits, a_scales, beta_a};
    return from_hip(hbmm::launch_conv_direct(x, pieces, N, g, form, out, static_cast<hipStream_t>(stream)));
}

int hbmm_probe_mfma_rate(int32_t steps, int32_t blocks, float *sink, void *stream)
{
    if (steps < 0 || blocks < 0 || steps > (1 << 24) || blocks > (1 << 16)) return HBMM_EINVAL;
    if (steps == 0 || blocks == 0) return HBMM_OK;
    if (!sink || !aligned16(sink)) return HBMM_EINVAL;
    return from_hip(hbmm::launch_probe_mfma(steps, blocks, sink, static_cast<hipStream_t>(stream)));
}

int hbmm_gemm_int(const uint32_t *a_bits, int64_t ldw_a, const uint32_t *b_bits, int64_t ldw_b,
                  int64_t M, int64_t N, int64_t K, int32_t *D, int64_t ldd, void *stream)
{
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return HBMM_EINVAL;
    if (M == 0 || N == 0) return HBMM_OK;
    if (!D || !aligned16(D) || ldd < N) return HBMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (K == 0) return from_hip(zero_block(D, ldd, M, N, s));
    if (int rc = check_packed(a_bits, M, K, ldw_a)) return rc;
    if (int rc = check_packed(b_bits, N, K, ldw_b)) return rc;

    hbmm::PopcountGemmArgs g{};
    if (b_is_lane_side(M, N)) {
        g.p_bits = b_bits; g.ldw_p = (int32_t)ldw_b; g.P = (int32_t)N;
        g.q_bits = a_bits; g.ldw_q = (int32_t)ldw_a; g.Q = (int32_t)M;
        g.ld_out_p = 1; g.ld_out_q = ldd;
    } else {
        g.p_bits = a_bits; g.ldw_p = (int32_t)ldw_a; g.P = (int32_t)M;
        g.q_bits = b_bits; g.ldw_q = (int32_t)ldw_b; g.Q = (int32_t)N;
        g.ld_out_p = ldd; g.ld_out_q = 1;
    }
    g.out = D;
    g.kwords = (int32_t)hbmm::packed_words(K);
    g.K = (int32_t)K;
    return from_hip(hbmm::launch_popcount_gemm(g, 64, 1, s));
}

int hbmm_dense_ref_gemm(const void *A, int64_t lda, const void *B, int64_t ldb, int32_t dtype,
                        int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, void *stream)
{
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return HBMM_EINVAL;
    if (dtype != 0 && dtype != 1) return HBMM_EUNSUPPORTED;
    if (K % 32 != 0) return HBMM_EUNSUPPORTED;
    if (M == 0 || N == 0) return HBMM_OK;
    if (!C || !aligned16(C) || ldc < N) return HBMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (K == 0) return from_hip(zero_block(C, ldc, M, N, s));
    if (!A || !B || !aligned16(A) || !aligned16(B) || lda < K || ldb < K) return HBMM_EINVAL;
    if (lda % 8 != 0 || ldb % 8 != 0) return HBMM_EINVAL;   // 16-byte row starts for either dtype
    return from_hip(hbmm::launch_dense_ref(A, lda, B, ldb, dtype, M, N, K, C, ldc, s));
}

}  // extern "C"
