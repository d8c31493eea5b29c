/*
 * CPU oracle for the Hadamard Binary Matrix Multiply (HBMM) of HadaNets.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code, header, table or helper with the HIP
 * path, and nothing on the product path may call it: only the tests, the smoke check and
 * the benchmark's cpu_baseline leg load it.
 *
 * Everything is written out from the paper's definitions, in double precision, with
 * no blocking, fusion or reordering.  OpenMP only spreads independent output rows over
 * cores; the arithmetic that produces any single output is sequential and in the order
 * the definition states.
 *
 * Notation (paper section 3 and section 4.2):
 *   x        full-precision operand, `rows` x K, row-major, K contiguous (section 4:
 *            tensors are stored row-major and binarised row by row).
 *   beta     segment length (the paper's measure of how aggressive the binarisation is);
 *            segments are consecutive runs of beta elements along K inside one row.
 *   delta    scale of a segment = mean of |x| over the segment (Eq. 1 / Eq. 3; the sums
 *            there are read as beta terms, r = 0 .. beta-1, to agree with the 1/beta
 *            factor and with section 3, which describes delta as a mean of absolute
 *            values over a segment).
 *   x~       delta (Hadamard product) Sign(x)  (Eq. 2 / Eq. 4), Sign(0) = +1.
 *   O        Eq. 7: sum over segments of W_f,j * A_f,j * (signed agreement count).  Eq. 7
 *            prints popcount(xnor(.)), the number p of agreeing signs; the +-1 inner
 *            product it stands for is 2p - n = n - 2*popcount(xor), n the segment length.
 *
 * Readings taken where the paper is silent:
 *   - a last segment shorter than beta is averaged over its own length;
 *   - bit k of a row is bit (k mod 32) of 32-bit word (k div 32), -1 -> 0, +1 -> 1
 *     (the 6-element example of section 4 fixes the value mapping, not the endianness);
 *   - bits past K inside the last word, and pad words, are 0;
 *   - the stored scale is fp32 (sum in double, divide, round once);
 *   - beta = 1 means no binarisation: x~ = x (with -0.0 -> +0.0).
 *
 * Parity pins: every function below is pinned by tests/test_oracle_pins.py (brute
 * force on tiny inputs, closed forms, the paper's packing example, special cases that
 * reduce to a plain matrix product or to XNOR-Net per-row scaling).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int sgn_ge0(float v) { return (v >= 0.0f) ? 1 : 0; } /* -0.0 -> 1, NaN -> 0 */

/* Eq. 1 / Eq. 3: delta[r, j] = mean_{k in segment j} |x[r, k]|, stored as fp32.
 * s is rows x lds, ceil(K/beta) valid entries per row. */
void oracle_block_scales(const float *x, int64_t rows, int64_t K, int64_t ldx, int64_t beta,
                         float *s, int64_t lds)
{
    int64_t nb = (K + beta - 1) / beta;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t j = 0; j < nb; ++j) {
            int64_t k0 = j * beta;
            int64_t k1 = k0 + beta < K ? k0 + beta : K;
            double acc = 0.0;
            for (int64_t k = k0; k < k1; ++k)
                acc += fabs((double)x[r * ldx + k]);
            s[r * lds + j] = (float)(acc / (double)(k1 - k0));
        }
    }
}

/* Sign + bit-pack (section 4's example: the row -1 1 1 -1 -1 1 is stored as 011001).
 * bits is rows x ldw uint32; every word of the row, pad words included, is written. */
void oracle_sign_pack(const float *x, int64_t rows, int64_t K, int64_t ldx,
                      uint32_t *bits, int64_t ldw)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t w = 0; w < ldw; ++w)
            bits[r * ldw + w] = 0u;
        for (int64_t k = 0; k < K; ++k)
            if (sgn_ge0(x[r * ldx + k]))
                bits[r * ldw + (k >> 5)] |= (uint32_t)1 << (k & 31);
    }
}

/* Eq. 2 / Eq. 4: xt[r, k] = delta[r, k div beta] * Sign(x[r, k]) in double (xt is rows x K,
 * dense).  beta == 1 keeps the operand itself (section 3.1: beta = 1 is the unquantised
 * setting), which is also what |x| * Sign(x) gives. */
void oracle_materialize(const float *x, int64_t rows, int64_t K, int64_t ldx, int64_t beta,
                        const float *s, int64_t lds, double *xt)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t k = 0; k < K; ++k) {
            float v = x[r * ldx + k];
            if (beta == 1)
                xt[r * K + k] = (v == 0.0f) ? 0.0 : (double)v;
            else
                xt[r * K + k] = sgn_ge0(v) ? (double)s[r * lds + k / beta]
                                           : -(double)s[r * lds + k / beta];
        }
    }
}

/* Plain definition of the product HBMM reaches: C[m, n] = sum_k At[m, k] * Bt[n, k],
 * both operands dense double, K contiguous, k ascending. */
void oracle_dense_f64_gemm(const double *At, const double *Bt, int64_t M, int64_t N, int64_t K,
                           double *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += At[m * K + k] * Bt[n * K + k];
            C[m * N + n] = acc;
        }
    }
}

/* popcount of (a xor b) restricted to bit range [k0, k1) of two packed rows. */
static int64_t hamming_range(const uint32_t *a, const uint32_t *b, int64_t k0, int64_t k1)
{
    int64_t h = 0;
    for (int64_t w = k0 >> 5; w <= (k1 - 1) >> 5; ++w) {
        int64_t lo = w << 5;
        uint32_t x = a[w] ^ b[w];
        if (k0 > lo)
            x &= ~(uint32_t)0 << (k0 - lo);
        if (k1 < lo + 32)
            x &= ~(uint32_t)0 >> (lo + 32 - k1);
        h += __builtin_popcount(x);
    }
    return h;
}

/* Eq. 7 on packed operands: the K axis is cut wherever a segment of either operand ends
 * (section 4.2: with different beta the finer one sets the granularity); on every piece
 * d = n - 2 * popcount(a xor b) is the exact +-1 inner product and contributes
 * sA * sB * d.  C and T are M x N doubles; T (may be NULL) receives the sum of the
 * absolute values of the contributions, the scale of fp32 accumulation error. */
void oracle_popcount_gemm(const uint32_t *a_bits, int64_t ldw_a, const float *a_s, int64_t lds_a,
                          int64_t beta_a, const uint32_t *b_bits, int64_t ldw_b, const float *b_s,
                          int64_t lds_b, int64_t beta_w, int64_t M, int64_t N, int64_t K,
                          double *C, double *T)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, tacc = 0.0;
            int64_t k0 = 0;
            while (k0 < K) {
                int64_t ea = (k0 / beta_a + 1) * beta_a;
                int64_t ew = (k0 / beta_w + 1) * beta_w;
                int64_t k1 = ea < ew ? ea : ew;
                if (k1 > K)
                    k1 = K;
                int64_t h = hamming_range(a_bits + m * ldw_a, b_bits + n * ldw_b, k0, k1);
                int64_t d = (k1 - k0) - 2 * h;
                double term = (double)a_s[m * lds_a + k0 / beta_a] *
                              (double)b_s[n * lds_b + k0 / beta_w] * (double)d;
                acc += term;
                tacc += fabs(term);
                k0 = k1;
            }
            C[m * N + n] = acc;
            if (T)
                T[m * N + n] = tacc;
        }
    }
}

/* Whole-row +-1 inner product: D[m, n] = K - 2 * hamming(a_row, b_row). */
void oracle_int_dot(const uint32_t *a_bits, int64_t ldw_a, const uint32_t *b_bits, int64_t ldw_b,
                    int64_t M, int64_t N, int64_t K, int32_t *D)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            D[m * N + n] = (int32_t)(K - 2 * hamming_range(a_bits + m * ldw_a, b_bits + n * ldw_b, 0, K));
}

/* Binary-weight form (beta_a = 1, the paper's HBWN): activations stay full precision,
 *   C[m, n] = sum_j sB[n, j] * sum_{k in segment j} A[m, k] * (+-1)_B[n, k].
 * T (may be NULL) receives sum_k |A[m, k]| * sB[n, k div beta_w]. */
void oracle_binary_weight_gemm(const float *A, int64_t lda, const uint32_t *b_bits, int64_t ldw_b,
                               const float *b_s, int64_t lds_b, int64_t beta_w, int64_t M, int64_t N,
                               int64_t K, double *C, double *T)
{
    int64_t nb = (K + beta_w - 1) / beta_w;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, tacc = 0.0;
            for (int64_t j = 0; j < nb; ++j) {
                int64_t k0 = j * beta_w;
                int64_t k1 = k0 + beta_w < K ? k0 + beta_w : K;
                double seg = 0.0, aseg = 0.0;
                for (int64_t k = k0; k < k1; ++k) {
                    double a = (double)A[m * lda + k];
                    int bit = (b_bits[n * ldw_b + (k >> 5)] >> (k & 31)) & 1u;
                    seg += bit ? a : -a;
                    aseg += fabs(a);
                }
                acc += (double)b_s[n * lds_b + j] * seg;
                tacc += (double)b_s[n * lds_b + j] * aseg;
            }
            C[m * N + n] = acc;
            if (T)
                T[m * N + n] = tacc;
        }
    }
}

/* Gradient through the Hadamard binarisation (Eq. 6, with the straight-through estimator of Eq. 5
 * for Sign).  For a row x, incoming gradient g = dC/dx~ and segment s(i) of n elements (beta, or
 * fewer in a ragged last segment; the printed upper limit of the sum is read as exclusive):
 *   dC/dx_i = (1/n) * Sign(x_i) * sum_{j in s(i)} g_j * Sign(x_j)  +  delta_{s(i)} * g_i * [|x_i| <= 1]
 * delta is the stored fp32 scale of the forward pass (mean |x| over the segment).  T (may be NULL)
 * receives (1/n) * sum_j |g_j| + delta * |g_i| * [|x_i| <= 1], the scale of the fp32 rounding error. */
void oracle_binarize_backward(const float *x, const float *g, int64_t rows, int64_t K, int64_t ldx,
                              int64_t ldg, int64_t beta, double *gx, double *T)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t k0 = 0; k0 < K; k0 += beta) {
            int64_t k1 = k0 + beta < K ? k0 + beta : K;
            double n = (double)(k1 - k0), sabs = 0.0, sdot = 0.0, sg = 0.0;
            for (int64_t k = k0; k < k1; ++k) {
                double gv = (double)g[r * ldg + k];
                sabs += fabs((double)x[r * ldx + k]);
                sdot += sgn_ge0(x[r * ldx + k]) ? gv : -gv;
                sg += fabs(gv);
            }
            double delta = (double)(float)(sabs / n);
            for (int64_t k = k0; k < k1; ++k) {
                float xv = x[r * ldx + k];
                double gv = (double)g[r * ldg + k];
                double ste = (fabsf(xv) <= 1.0f) ? 1.0 : 0.0;
                double sign = sgn_ge0(xv) ? 1.0 : -1.0;
                gx[r * K + k] = sign * sdot / n + delta * gv * ste;
                if (T)
                    T[r * K + k] = sg / n + delta * fabs(gv) * ste;
            }
        }
    }
}

/* Convolution of a Hadamard-binarised activation tensor with Hadamard-binarised filters, written
 * from the definition of a (cross-correlation) convolution layer with zero padding:
 *   O[b, n, oz, oy] = sum_{c, dz, dy} At[b, c, oz*stride - pad + dz, oy*stride - pad + dy] * Wt[n, c, dz, dy]
 * where positions outside the input contribute nothing.  At (B x C x H x W, W contiguous: the
 * width index y of Eq. 3 is the contiguous one) and Wt (N x C x KH x KW) are the materialised
 * tensors delta (.) Sign(.): At by Eq. 3-4 (segments of beta_a along the width of each row of each
 * channel), Wt by Eq. 1-2 (segments of beta_w along the filter flattened to C*KH*KW).  The caller
 * materialises them with oracle_materialize on the corresponding rows x K views.  The terms are
 * added in the order c, dz, dy (the flattened filter order).  T (may be NULL) receives the sum of
 * the absolute values of the terms. */
void oracle_conv2d_f64(const double *At, const double *Wt, int64_t B, int64_t C, int64_t H, int64_t W,
                       int64_t N, int64_t KH, int64_t KW, int64_t stride, int64_t pad, double *O,
                       double *T)
{
    const int64_t OH = (H + 2 * pad - KH) / stride + 1;
    const int64_t OW = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t oz = 0; oz < OH; ++oz) {
                for (int64_t oy = 0; oy < OW; ++oy) {
                    double acc = 0.0, tabs = 0.0;
                    for (int64_t c = 0; c < C; ++c) {
                        for (int64_t dz = 0; dz < KH; ++dz) {
                            for (int64_t dy = 0; dy < KW; ++dy) {
                                const int64_t z = oz * stride - pad + dz;
                                const int64_t y = oy * stride - pad + dy;
                                if (z < 0 || z >= H || y < 0 || y >= W)
                                    continue;
                                const double term = At[((b * C + c) * H + z) * W + y] *
                                                    Wt[((n * C + c) * KH + dz) * KW + dy];
                                acc += term;
                                tabs += fabs(term);
                            }
                        }
                    }
                    O[((b * N + n) * OH + oz) * OW + oy] = acc;
                    if (T)
                        T[((b * N + n) * OH + oz) * OW + oy] = tabs;
                }
            }
        }
    }
}
