/*
 * libhbmm -- Hadamard Binary Matrix Multiply (HBMM) of HadaNets for AMD MI355X (gfx950).
 *
 * Plain C ABI.  Conventions shared by every entry point:
 *
 *  - Every buffer is a DEVICE pointer owned by the caller.  The library never allocates,
 *    frees or synchronises: each call validates its arguments on the host, enqueues its
 *    kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *    returns.  There is no global state; calls on different streams may overlap as long as
 *    their output buffers do not.
 *  - Return value: HBMM_OK, or a negative HBMM_E* code.  Nothing is thrown or aborted; on an
 *    error no kernel has been launched and no output has been touched.
 *  - Matrices are row-major (paper, section 4: tensors are stored row-major and binarised
 *    row-wise).  Leading dimensions (`ld*`) are in elements of the pointed-to type.
 *  - Pointers must be 16-byte aligned.  `ldw*` must be a multiple of 4 words.
 *
 * Operand convention (paper, section 3.1.1 and section 4.2).  A is the activation operand,
 * M x K.  B is the weight operand in the paper's reshaped form W^f = Reshape(W, (filters, -1)):
 * N x K, so that both operands have K contiguous and the product is C = A~ . B~^T, M x N.
 * A~ = delta_a (.) Sign(A) and B~ = delta_w (.) Sign(B) (Eq. 2, Eq. 4), where delta is the mean
 * of |x| over consecutive segments of beta elements along K inside one row (Eq. 1, Eq. 3).
 *
 * Packed form of an operand with `rows` rows:
 *   bits    rows x ldw uint32.  Element k of a row is bit (k mod 32) of word (k div 32);
 *           bit 1 <=> x >= 0 (Sign = +1; Sign(0) = +1, -0.0 counts as 0, NaN gives bit 0),
 *           bit 0 <=> Sign = -1 (section 4: the row -1 1 1 -1 -1 1 packs to 011001).
 *           Words [0, hbmm_packed_ld_words(K)) of every row are written; bits at k >= K
 *           inside them are 0.  Words past that (if ldw is larger) are not touched.
 *   scales  rows x lds fp32, entry j of a row = mean |x| over k in [j*beta, (j+1)*beta) (the last
 *           segment ends at K and is averaged over its own length when beta does not divide K);
 *           hbmm_num_blocks(K, beta) entries per row are written (section 4.2: the
 *           full-precision side shrinks by the factor beta).
 */
#ifndef HBMM_H
#define HBMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HBMM_OK 0
#define HBMM_EINVAL (-1)       /* null pointer, bad shape, misaligned pointer, ld too small */
#define HBMM_EUNSUPPORTED (-2) /* beta / K / algo / dtype outside the supported set */
#define HBMM_ELAUNCH (-3)      /* HIP reported an error when the kernel was enqueued */

/* Human-readable text for a return code (static storage, never NULL). */
const char *hbmm_strerror(int code);

/* ceil(K / beta): scale entries per row (Eq. 7 sums over this many segments). 0 if K < 0 or beta < 1. */
int64_t hbmm_num_blocks(int64_t K, int32_t beta);

/* 32-bit words per packed row: ceil(K / 32) rounded up to a multiple of 4 (16-byte rows). */
int64_t hbmm_packed_ld_words(int64_t K);

/*
 * Hadamard binarisation of one operand: block scales (Eq. 1 / Eq. 3), Sign (Eq. 2 / Eq. 4) and
 * bit-packing (section 4), in one pass over x.
 *
 *   x       fp32 source.  layout 0: rows x K, element (r, k) at x[r*ldx + k]   (ldx >= K).
 *                         layout 1: K x rows, element (r, k) at x[k*ldx + r]   (ldx >= rows);
 *                         this is a right-hand operand written the usual K x N way; the result
 *                         is identical to packing its transpose.
 *   beta    segment length, 2 .. 256.  The paper's settings -- a power of two that divides K, K a
 *           multiple of 32 -- take the tuned kernels.  Any other beta in that range and any K >= 1 is
 *           accepted too: the last segment is then the shorter remainder and its scale is the mean of
 *           |x| over its own length (Eq. 1 applied to the elements that exist); bits at k >= K are 0.
 *   bits    out, rows x ldw (ldw >= hbmm_packed_ld_words(K), multiple of 4).
 *   scales  out, rows x lds (lds >= hbmm_num_blocks(K, beta)).
 *
 * rows == 0 or K == 0 is a valid no-op.  The fp32 scale is a pairwise fp32 sum for layout 0
 * (relative error <= (log2(beta) + 1) * 2^-24) and a double-precision sequential sum rounded
 * once for layout 1 and for the general kernel.
 */
int hbmm_quantize_pack(const float *x, int64_t rows, int64_t K, int64_t ldx, int32_t layout,
                       int32_t beta, uint32_t *bits, int64_t ldw, float *scales, int64_t lds,
                       void *stream);

/*
 * Gradient through the Hadamard binarisation (Eq. 6, with the straight-through estimator of Eq. 5):
 *
 *   grad_in[r, i] = (1/beta) * Sign(x[r, i]) * sum_{j in segment(i)} grad_out[r, j] * Sign(x[r, j])
 *                   + delta[r, segment(i)] * grad_out[r, i] * (|x[r, i]| <= 1 ? 1 : 0)
 *
 * x is the full-precision tensor that was binarised (rows x K, segments of beta along K, as in
 * hbmm_quantize_pack layout 0), grad_out the gradient with respect to delta (.) Sign(x), delta the mean
 * of |x| over the segment (recomputed from x).  The upper limit of the sum printed in Eq. 6 is read
 * as exclusive (beta terms).  beta in 1 .. 256; the tuned kernel takes a power of two with K a multiple of beta
 * and of 4, any other beta or K goes to a general kernel, where a shorter last segment has delta averaged
 * over its own length n and 1/n in place of 1/beta.
 * grad_in may not alias x or grad_out.  fp32 arithmetic; error <= (log2(beta) + 3) * 2^-24 times
 * ((1/beta) sum_j |grad_out_j| + delta |grad_out_i|).
 */
int hbmm_binarize_backward(const float *x, const float *grad_out, int64_t rows, int64_t K, int64_t ldx,
                           int64_t ldg, int32_t beta, float *grad_in, int64_t ldgi, void *stream);

/*
 * HBMM proper (Eq. 7, with popcount(xnor) read as the signed agreement count):
 *
 *   C[m, n] = sum over segments g of  sA[m, g*G / beta_a] * sB[n, g*G / beta_w] * d[m, n, g],
 *   d[m, n, g] = G - 2 * popcount(a_bits[m, g] xor b_bits[n, g])     (the +-1 inner product)
 *
 * with G = min(beta_a, beta_w) (section 4.2: the finer segmentation sets the granularity).
 * Integer work is exact; the scaled terms are accumulated in fp32 in ascending g.
 *
 *   a_bits, a_scales  packed A (M rows), from hbmm_quantize_pack with beta_a.
 *   b_bits, b_scales  packed B (N rows), from hbmm_quantize_pack with beta_w.
 *   beta_a, beta_w    each in 1 .. 256.  The paper's settings -- powers of two (or 1) with K a multiple
 *                     of both and of 32 -- are described first; the general case is at the end.
 *                     beta == 1 means that operand is not binarised (the paper's beta = 1; beta_a = 1
 *                     is its HBWN): its bits pointer must be NULL, its scales pointer is the raw fp32
 *                     operand (rows x K, leading dimension lds, a multiple of 4), and e.g. for
 *                     beta_a = 1:  C[m, n] = sum_j sB[n, j] * sum_{k in j} A[m, k] * Sign(B)[n, k].
 *                     Both >= 32: the XNOR + popcount kernel.  Otherwise (a segment shorter than a
 *                     32-bit word, or an unquantised operand) the product runs on the matrix cores:
 *                     the operand with the longer segment (>= 16) keeps its signs, the other is
 *                     rebuilt as fp32 values (or is the unquantised operand itself) split exactly
 *                     into three bf16 pieces; if neither segment reaches 16 both are rebuilt (this
 *                     covers the paper's binary-weight networks, beta_a = 1 with beta_w = 4 or 8, and
 *                     its HadaNets with beta_a = beta_w = 4).  Not supported: beta = 1 for both (that
 *                     is hbmm_dense_ref_gemm).
 *                     General case (a segment length that is not a power of two, a K that beta does not
 *                     divide, K not a multiple of 32; algo 0 or -1): the operands are as
 *                     hbmm_quantize_pack writes them for that beta and K (scales per row:
 *                     hbmm_num_blocks(K, beta), the last segment shorter, bits at k >= K zero).
 *                     Both beta powers of two >= 32: still the XNOR + popcount kernel; the last segment
 *                     of G contributes (K mod G) - 2 * popcount.  Otherwise (K < 2^24) both operands are
 *                     rebuilt as fp32 values on the matrix-core kernel, C[m, n] = sum_k A~[m, k] * B~[n, k]
 *                     with X~[r, k] = sX[r, k div beta] * Sign(X)[r, k].  An unquantised operand needs no
 *                     particular leading dimension here.
 *   C                 out, M x N fp32, leading dimension ldc >= N.
 *   algo              0: the method's kernel as described above.
 *                     1: (both beta >= 32 only) the same d[m, n, g] from int8 +-1 matrix-core (MFMA)
 *                        products, kept as a comparison point; same epilogue, bit-identical result.
 *                     2: (both beta >= 64 only) the same d[m, n, g] from 4-bit-float +-1 matrix-core
 *                        products (the operands are expanded from their bits on chip); same epilogue,
 *                        bit-identical result.
 *                     3: (both beta >= 16, the shorter one 16 or 32, K a multiple of 128) the same
 *                        d[m, n, g] from 8-bit-float +-1 matrix-core products, 16 elements of K per step;
 *                        same epilogue (bit-identical to 0 when both beta >= 32).
 *                    -1: the fastest of these for the given segment lengths and output size (2 when both
 *                        beta >= 64, 3 when both are 16 or 32 and K is a multiple of 128, else 0; and 0
 *                        when both beta >= 32 and the output has fewer than 32 tiles of 128 x 128).
 *
 * M == 0 or N == 0 is a valid no-op; K == 0 writes zeros.
 */
int hbmm_gemm(const uint32_t *a_bits, const float *a_scales, int64_t ldw_a, int64_t lds_a,
              int32_t beta_a, const uint32_t *b_bits, const float *b_scales, int64_t ldw_b,
              int64_t lds_b, int32_t beta_w, int64_t M, int64_t N, int64_t K, float *C, int64_t ldc,
              int32_t algo, void *stream);

/*
 * Binarise a whole tensor stored contiguously (Eq. 3-4 for an activation tensor B x C x H x W whose
 * width W is the contiguous axis and a multiple of beta: the segments of beta consecutive elements
 * then are the width segments of Eq. 3 and never leave a row).
 *   x       device, fp32, count elements, 16-byte aligned.
 *   beta    power of two in 2 .. 256.
 *   bits    out, device, count / 32 words: element e is bit (e mod 32) of word (e div 32), 1 = (x >= 0).
 *   scales  out, device, count / beta fp32: mean |x| of elements [j * beta, (j + 1) * beta).
 * count must be a multiple of 128 and of beta (else HBMM_EUNSUPPORTED) and below 2^31.
 */
int hbmm_quantize_pack_tensor(const float *x, int64_t count, int32_t beta, uint32_t *bits, float *scales,
                              void *stream);

/*
 * Hadamard binarisation of an activation tensor with Eq. 3's segments for any segment length: the tensor is
 * `rows` rows of W contiguous elements (rows = batch * channels * height, W the width), segments of beta run
 * along the width and start anew in every row; when beta does not divide W (the paper only asks
 * beta <= w_in; e.g. 7 x 7 feature maps with beta = 4) the last segment of a row is the shorter remainder and
 * its scale the mean of |x| over its own length.
 *   bits    out, ceil(rows * W / 32) words: element e = r * W + y is bit e mod 32 of word e div 32 (rows are not
 *           padded; bits past the last element are 0).
 *   scales  out, rows x ceil(W / beta) fp32, contiguous.
 * beta in 2 .. 256; rows * W below 2^31.  When beta is a power of two that divides W (and rows * W is a multiple
 * of 128) this is the layout hbmm_quantize_pack_tensor writes, and that kernel is used.  Scales otherwise:
 * double-precision sums rounded once.
 */
int hbmm_quantize_pack_activations(const float *x, int64_t rows, int64_t W, int32_t beta, uint32_t *bits, float *scales,
                                   void *stream);

/*
 * hbmm_binarize_backward for a whole tensor stored contiguously, segments of beta consecutive elements
 * (the counterpart of hbmm_quantize_pack_tensor: for an activation tensor whose width is a multiple
 * of beta this is the gradient through Eq. 3-4).  count: a multiple of 128 and of beta, below 2^31.
 */
int hbmm_binarize_backward_tensor(const float *x, const float *grad_out, int64_t count, int32_t beta, float *grad_in,
                                   void *stream);

/*
 * A convolution layer of a HadaNet, computed directly from the packed tensors (no im2col matrix is
 * formed): activations binarised by Eq. 3-4, filters by Eq. 1-2, then
 *   out[b, n, oz, oy] = sum_{c, dz, dy} A~[b, c, oz*stride - pad + dz, oy*stride - pad + dy] * W~[n, c, dz, dy]
 * with zero contribution from positions outside the input (zero padding).
 *   a_bits, a_scales   the activation tensor B x C x H x W as written by hbmm_quantize_pack_tensor
 *                      with beta_a (beta_a in 2 .. 256 must divide W).  beta_a = 1: the activations are
 *                      not binarised (binary-weight layer); a_bits must be NULL and a_scales is the
 *                      fp32 tensor itself.
 *   w_bits, w_scales   the filters N x C x KH x KW as written by hbmm_quantize_pack (layout 0) on the
 *                      N x (C*KH*KW) matrix with beta_w; ldw_w / lds_w its leading dimensions.
 *                      beta_w in 2 .. 256.
 *   out                device, fp32, B x N x OH x OW contiguous, OH = (H + 2 pad - KH) / stride + 1,
 *                      OW likewise; 16-byte aligned.
 * C*KH*KW must be a multiple of 32 and of beta_w, KH*KW <= 32, B*C*H*W and B*OH*OW below 2^31; other
 * shapes return HBMM_EUNSUPPORTED.  The activation values run on the matrix cores as three exact
 * bf16 pieces of the fp32 scale, the filter signs as +-1, the filter scale is applied per segment in
 * fp32: every output is an fp32 sum of exact terms.  With beta_w < 16 (a filter segment shorter than
 * one matrix-core step) the filter values are rebuilt and split the same way and the six largest of
 * the nine piece products are added (what is dropped is below 2^-24 of a term); algo is then ignored.
 *   algo   0: each workgroup stages the input patch of its output rows once per channel in on-chip
 *             memory and gathers the window elements from there (used when the layer fits: window of
 *             at least 2 taps, OW <= 128, patch of at most 1024 elements per channel); otherwise as 1.
 *          1: every window element is gathered from device memory (any supported shape).
 *          Both give the same sums in the same order.
 */
int hbmm_conv2d(const uint32_t *a_bits, const float *a_scales, int32_t beta_a, const uint32_t *w_bits,
                const float *w_scales, int64_t ldw_w, int64_t lds_w, int32_t beta_w, int64_t B, int64_t C,
                int64_t H, int64_t W, int64_t N, int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                float *out, int32_t algo, void *stream);

/*
 * The same layer with the filters prepared ahead of time -- they do not change between calls -- which is
 * the fast form: hbmm_conv_prepare_filters turns the packed filters into the three bf16 pieces of every
 * weight (delta_w * Sign(w), Eq. 1-2), laid out in the order the matrix cores consume them, and
 * hbmm_conv2d_prepared multiplies them with the activations (Eq. 3-4) read through the window of each
 * output position.  The sum runs over (channel group of 32, tap, channel), a fixed order: results are the
 * same from call to call.  `form` chooses how the fp32 values of both sides reach the matrix cores, and must
 * be the same in all three calls:
 *   HBMM_PIECES_BF16X3 (0)  every value split exactly into three bf16 pieces; the six largest of the nine
 *                           piece products are added in fp32 (what is dropped is below 2^-24 of a term).
 *   HBMM_PIECES_F16X2 (1)   every value scaled by a power of two (per filter; per workgroup for the
 *                           activations, following the largest magnitude met so far, with an exact
 *                           rescale of the partial sums when it grows) and written as two fp16 pieces,
 *                           22 significant bits; three piece products: half the multiplies.
 *                           |error| <= 3 * 2^-22 * sum |A~ W~| over the window, plus 2^-39 of (largest
 *                           |A~| in the workgroup's input patch x sum |W~|) and of (largest |W~| of the filter
 *                           x sum |A~|) from the remainders that fall below fp16's smallest subnormal; values
 *                           below 2^-113 count as 0.  Measured 1.15-1.4 times faster on ResNet-18's layers at batch 64.
 *
 *   hbmm_conv_filter_pieces_bytes   size of `pieces` for N filters of C x KH x KW (0 for an invalid shape or
 *                                   form): 6 (form 0) or 4 (form 1) bytes per weight, N rounded up to 32 and
 *                                   C to 32, plus 4 bytes per filter in form 1.
 *   hbmm_conv_prepare_filters       w_bits / w_scales as for hbmm_conv2d, with any beta_w in 2 .. 256
 *                                   (a shorter last segment included: lds_w >= hbmm_num_blocks(C*KH*KW, beta_w)),
 *                                   or beta_w = 1: filters not binarised, w_bits NULL and w_scales the
 *                                   fp32 N x (C*KH*KW) matrix with leading dimension lds_w.
 *                                   pieces: out, device, 16-byte aligned, hbmm_conv_filter_pieces_bytes(...) bytes.
 *                                   C*KH*KW < 2^24; KH, KW <= 32.
 *   hbmm_conv2d_prepared            a_bits / a_scales / out and the geometry as for hbmm_conv2d, with any beta_a
 *                                   in 1 .. 256: the activations as written by hbmm_quantize_pack_activations
 *                                   (flat bits, scales (B*C*H) x ceil(W / beta_a): for a beta_a that divides W
 *                                   that is also what hbmm_quantize_pack_tensor writes); beta_a = 1: a_bits
 *                                   NULL, a_scales the fp32 tensor.
 *                                   pieces from hbmm_conv_prepare_filters for the same N, C, KH, KW, form.
 *                                   The layer must fit the kernel: OW <= 128 and
 *                                   ((OW - 1) * stride + KW) * KH <= 640 (the input patch of one output
 *                                   row in on-chip memory), and the images of one tile within 32-bit byte
 *                                   offsets (C*H*W below 2^30 / images per tile; a tile holds several images
 *                                   only when a whole image is at most 64 positions); otherwise
 *                                   HBMM_EUNSUPPORTED (use hbmm_conv2d).
 *                                   No restriction on C*KH*KW being a multiple of 32 or of beta_w.
 */
#define HBMM_PIECES_BF16X3 0
#define HBMM_PIECES_F16X2 1
int64_t hbmm_conv_filter_pieces_bytes(int64_t N, int64_t C, int32_t KH, int32_t KW, int32_t form);
int hbmm_conv_prepare_filters(const uint32_t *w_bits, const float *w_scales, int64_t ldw_w, int64_t lds_w,
                              int32_t beta_w, int64_t N, int64_t C, int32_t KH, int32_t KW, int32_t form, void *pieces,
                              void *stream);
int hbmm_conv2d_prepared(const uint32_t *a_bits, const float *a_scales, int32_t beta_a, const void *pieces, int32_t form,
                         int64_t B,
                         int64_t C, int64_t H, int64_t W, int64_t N, int32_t KH, int32_t KW, int32_t stride,
                         int32_t pad, float *out, void *stream);

/*
 * Fused form for the activation operand: the same C as
 *     hbmm_quantize_pack(A, layout 0, beta_a)  followed by  hbmm_gemm(..., algo 0)
 * (bit for bit: same scale arithmetic, same contraction, same epilogue order), but A is binarised
 * inside the product kernel, tile by tile, and its packed form is never written to memory.  Meant
 * for the im2col shapes with few output channels and many rows (N <= 128), where packing A costs
 * more than the product and the product then hides behind the fp32 read of A; every group of 64
 * columns of C re-reads A, hence the limit.
 *   A        fp32, M x K, leading dimension lda (multiple of 4), not binarised beforehand.
 *   beta_a, beta_w  each in {32, 64, 128, 256}; K a multiple of both.  N <= 128.
 */
int hbmm_gemm_fused(const float *A, int64_t lda, int32_t beta_a, const uint32_t *b_bits,
                    const float *b_scales, int64_t ldw_b, int64_t lds_b, int32_t beta_w, int64_t M,
                    int64_t N, int64_t K, float *C, int64_t ldc, void *stream);

/*
 * Unscaled whole-row +-1 inner products, for exact parity checks of the contraction:
 *   D[m, n] = K - 2 * popcount(a_row xor b_row),  int32, M x N, leading dimension ldd >= N.
 * Uses the same inner loop as hbmm_gemm(algo 0).  K need not be a multiple of 32 (pad bits are 0
 * in both operands and cancel).
 */
int hbmm_gemm_int(const uint32_t *a_bits, int64_t ldw_a, const uint32_t *b_bits, int64_t ldw_b,
                  int64_t M, int64_t N, int64_t K, int32_t *D, int64_t ldd, void *stream);

/*
 * Dense comparison product on unquantised operands (the full-precision matrix multiply that
 * section 4.2 times its kernel against):  C = A . B^T, A M x K, B N x K, both K contiguous.
 *   dtype 0: fp32 operands.  dtype 1: bf16 operands (raw uint16 bit patterns).
 * fp32 accumulation and fp32 C in both cases.  K must be a multiple of 32 (fp32) or 64 (bf16); lda and
 * ldb must be multiples of 8 elements.
 */
int hbmm_dense_ref_gemm(const void *A, int64_t lda, const void *B, int64_t ldb, int32_t dtype,
                        int64_t M, int64_t N, int64_t K, float *C, int64_t ldc, void *stream);

/*
 * Diagnostic, not part of the method: runs `blocks` workgroups of eight waves, each wave steps * 24
 * matrix-core instructions of the kind the fp32-as-three-bf16-pieces kernels use (32 x 32 x 16, bf16, 32768
 * flops each) on pseudo-random register operands with nothing else in the loop, so that a caller who times
 * the call learns the rate the machine sustains under that load (with every compute unit busy the clock,
 * and so the rate, is below the published peak).  sink: device, blocks * 512 floats, written with values of
 * no meaning.  steps <= 2^24, blocks <= 65536.
 */
int hbmm_probe_mfma_rate(int32_t steps, int32_t blocks, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HBMM_H */
