// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
// Every launcher validates nothing: shapes, alignment and supported sets are checked by the
// caller in api.hip before any of these is reached.  Each returns the hipError_t of its launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbmm {

// Words written per packed row: ceil(K/32) rounded up to a multiple of 4.
inline int64_t packed_words(int64_t K) { return ((K + 31) / 32 + 3) / 4 * 4; }

// ---- pack.hip ---------------------------------------------------------------------------------
hipError_t launch_pack_rows(const float *x, int64_t rows, int64_t K, int64_t ldx, int beta,
                            uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s);
hipError_t launch_pack_cols(const float *x, int64_t rows, int64_t K, int64_t ldx, int beta,
                            uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s);

// Any beta in 2..256 and any K >= 1 (the last segment may be shorter); layout 0: x is rows x K, 1: K x rows.
hipError_t launch_pack_any(const float *x, int64_t rows, int64_t K, int64_t ldx, int layout, int beta,
                           uint32_t *bits, int64_t ldw, float *scales, int64_t lds, hipStream_t s);

// An activation tensor as rows x W (rows = batch * channels * height): flat sign bits (ceil(rows * W / 32) words),
// scales rows x ceil(W / beta) with a shorter last segment per row.  Any beta in 2..256, any W.
hipError_t launch_pack_activations_any(const float *x, int64_t rows, int64_t W, int beta, uint32_t *bits, float *scales,
                                       hipStream_t s);

// ---- backward.hip -----------------------------------------------------------------------------
hipError_t launch_binarize_backward(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx,
                                    int64_t ldg, int beta, float *gx, int64_t ldgx, hipStream_t s);

// Any beta in 1..256 and any K >= 1 (a shorter last segment).
hipError_t launch_binarize_backward_any(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx, int64_t ldg,
                                        int beta, float *gx, int64_t ldgx, hipStream_t s);

// ---- gemm_popcount.hip ------------------------------------------------------------------------
// One operand ("P") is held per lane, the other ("Q") is broadcast through scalar registers.
// out[p * ld_out_p + q * ld_out_q] receives the result for P-row p and Q-row q, so either of
// A / B can play either role.
struct PopcountGemmArgs {
    const float *p_src;  // fused mode: P as fp32 (rows x K, leading dimension ld_p_src); else nullptr
    int64_t ld_p_src;
    int32_t beta_p;      // fused mode: segment length of P
    const uint32_t *p_bits;
    const float *p_scales;
    const uint32_t *q_bits;
    const float *q_scales;
    void *out;           // float* (scaled) or int32_t* (integer mode)
    int64_t ld_out_p;
    int64_t ld_out_q;
    int32_t P, Q;        // rows of each operand
    int32_t ldw_p, ldw_q;
    int32_t lds_p, lds_q;
    int32_t kwords;      // words per row that are read: packed_words(K)
    int32_t ngran;       // K div G: whole segments of the finer operand (scaled mode)
    int32_t tail_bits;   // K mod G: length of the shorter last segment, 0 if G divides K
    int32_t kw_used;     // ceil(K / 32): words of a row that hold elements
    int32_t nblk_p, nblk_q;   // scales per row of each operand: ceil(K / beta)
    int32_t shift_p;     // log2(beta_p / G)
    int32_t shift_q;     // log2(beta_q / G)
    int32_t K;           // bits (integer mode: D = K - 2 * hamming)
    int32_t tiles_p;     // ceil(P / tile)        (this and the fields below are filled by the launcher)
    int32_t tiles_q;
    int32_t sup_p;       // P tiles per super-tile (128 tiles that one XCD works on together); 0: plain map
};
// G = min(beta_p, beta_q) in {32, 64, 128, 256}; integer != 0 selects the unscaled whole-row mode.
hipError_t launch_popcount_gemm(const PopcountGemmArgs &a, int G, int integer, hipStream_t s);

// ---- gemm_mfma_split.hip ---------------------------------------------------------------------
// One operand of the matrix-core HBMM.  beta == 1: `raw` is the fp32 operand itself (rows x K,
// leading dimension ld_raw) and bits / scales are unused; otherwise the packed form.
struct SplitGemmOperand {
    const float *raw;
    int64_t ld_raw;
    const uint32_t *bits;
    const float *scales;
    int64_t ldw, lds;
    int64_t rows;
    int beta;
};
// out[x * ld_out_x + y * ld_out_y] = sum_k X~[x, k] * Y~[y, k] on the matrix cores.
// x: any supported beta (1 = raw fp32).  y: packed, beta >= 2; with beta >= 16 it keeps its signs and
// its scale is applied once per segment, with a shorter segment it is rebuilt as fp32 values like x.
// K must be a multiple of 32.
hipError_t launch_mfma_split_gemm(const SplitGemmOperand &x, const SplitGemmOperand &y, int64_t K, float *out,
                                  int64_t ld_out_x, int64_t ld_out_y, hipStream_t s);
// The same product for any beta in 1..256 on either side (y: >= 2) and any 1 <= K < 2^24, including
// segment lengths that are not powers of two and a shorter last segment: both sides are rebuilt as fp32
// values element by element.
hipError_t launch_mfma_split_any(const SplitGemmOperand &x, const SplitGemmOperand &y, int64_t K, float *out,
                                 int64_t ld_out_x, int64_t ld_out_y, hipStream_t s);
// Convolution layer on the same kernel: the dense side is an activation tensor B x C x H x W packed
// flat with segments of `beta` along W (beta divides W), read through the KH x KW window of each
// output position; the other side holds the filters packed as rows of C*KH*KW (beta >= 2).
// out is B x y.rows x OH x OW.  C*KH*KW must be a multiple of 32, KH*KW <= 32.
struct ConvActivations {
    const uint32_t *bits;
    const float *scales;
    int beta;
};
struct ConvGeometry {
    int64_t B, C, H, W;
    int KH, KW, stride, pad;
    int algo;   // 0: activations staged once per workgroup when the layer fits, else 1; 1: per-tap gather
};
hipError_t launch_mfma_split_conv(const ConvActivations &x, const SplitGemmOperand &y, const ConvGeometry &g, float *out,
                                  hipStream_t s);

// ---- conv_direct.hip ---------------------------------------------------------------------------
// The same layer with the filters prepared once (the pieces of every weight, in the order the matrix
// cores consume them) and the activation fragments read straight from a patch in LDS.  form 0: three
// bf16 pieces per number, six piece products (exact split); form 1: two fp16 pieces of the number scaled
// by a power of two, three piece products (22 significant bits).
// Bytes of the prepared form of N filters of C x KH x KW:
int64_t conv_filter_pieces_bytes(int64_t N, int64_t C, int KH, int KW, int form);
// Filters packed as rows of C*KH*KW with any beta in 2..256 (or beta = 1: w_scales is the fp32 filter
// matrix itself, N x lds) -> pieces.
hipError_t launch_conv_prepare_filters(const uint32_t *w_bits, const float *w_scales, int64_t ldw, int64_t lds, int beta,
                                       int64_t N, int64_t C, int KH, int KW, int form, void *pieces, hipStream_t s);
// Whether the layer fits the kernel: output rows of at most 128 positions, and the input patch of one
// output row within the LDS and the staging registers ((OW - 1) stride + KW) * KH <= 640 pixels).
bool conv_direct_fits(const ConvGeometry &g);
hipError_t launch_conv_direct(const ConvActivations &x, const void *pieces, int64_t N, const ConvGeometry &g, int form,
                              float *out, hipStream_t s);

// ---- gemm_mfma_i8.hip -------------------------------------------------------------------------
hipError_t launch_mfma_i8_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                               int64_t lds_a, int beta_a, const uint32_t *b_bits,
                               const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                               int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s);

// ---- gemm_mfma_fp4.hip ------------------------------------------------------------------------
// Same contract as launch_mfma_i8_gemm; min(beta_a, beta_w) >= 64.
hipError_t launch_mfma_fp4_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                                int64_t lds_a, int beta_a, const uint32_t *b_bits,
                                const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s);

// ---- gemm_mfma_fp8.hip ------------------------------------------------------------------------
// Same contract; both beta >= 16, min(beta_a, beta_w) in {16, 32}, K a multiple of 128.
hipError_t launch_mfma_fp8_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a,
                                int64_t lds_a, int beta_a, const uint32_t *b_bits,
                                const float *b_scales, int64_t ldw_b, int64_t lds_b, int beta_w,
                                int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s);

// ---- probe.hip ---------------------------------------------------------------------------------
// `blocks` workgroups of eight waves, each wave steps * 24 MFMAs (32 x 32 x 16, bf16); sink: blocks * 512 floats.
hipError_t launch_probe_mfma(int steps, int blocks, float *sink, hipStream_t s);

// ---- dense_ref.hip ----------------------------------------------------------------------------
hipError_t launch_dense_ref(const void *A, int64_t lda, const void *B, int64_t ldb, int dtype,
                            int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, hipStream_t s);

}  // namespace hbmm
