"""GPU parity: every entry point of libhbmm against the CPU oracle, element by element, on the
same seeded inputs.  Packed words and integer sums must be bit-exact; scales and fp32 outputs
within the documented tolerances."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_1905_10759_amd import synth

from gpu_common import assert_close_to_oracle, dev, words

pytestmark = pytest.mark.gpu

hbmm = None


@pytest.fixture(scope="module", autouse=True)
def _load():
    global hbmm
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_1905_10759_amd import hbmm as mod
    hbmm = mod
    yield
    torch.cuda.synchronize()


def scale_tol(beta: int) -> float:
    # pairwise fp32 sum of beta magnitudes: log2(beta) roundings, plus the oracle's own final rounding
    return (np.log2(beta) + 1) * 2.0 ** -24


# ------------------------------------------------------------------------------ quantize_pack
@pytest.mark.parametrize("beta", [2, 4, 8, 16, 32, 64, 128, 256])
@pytest.mark.parametrize("rows,K", [(1, 256), (5, 768), (67, 1280), (130, 4608), (3, 256 * 9)])
def test_pack_rows(beta, rows, K):
    x = synth.normal(100 + beta + rows, (rows, K))
    x[0, :4] = [0.0, -0.0, 1e-38, -1e-38]
    bits, scales = hbmm.quantize_pack(dev(x), beta)
    torch.cuda.synchronize()
    assert np.array_equal(words(bits), oracle.sign_pack(x))
    ref = oracle.block_scales(x, beta)
    got = scales.cpu().numpy()
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= scale_tol(beta) * ref)


@pytest.mark.parametrize("beta", [2, 4, 8, 16])
def test_pack_rows_short_segments_ragged(beta):
    """Short segments with K = 96 + 32 j (not a multiple of the 256-element wave chunk) and an odd
    scale leading dimension."""
    for K in (96, 160, 1056):
        x = synth.normal(150 + beta + K, (9, K))
        nb = K // beta
        scales = torch.full((9, nb + 3), -7.0, dtype=torch.float32, device="cuda")
        bits, _ = hbmm.quantize_pack(dev(x), beta, 0, None, scales[:, :nb])
        assert np.array_equal(words(bits), oracle.sign_pack(x))
        ref = oracle.block_scales(x, beta)
        got = scales.cpu().numpy()
        assert np.all(np.abs(got[:, :nb] - ref) <= scale_tol(beta) * ref)
        assert (got[:, nb:] == -7.0).all()


def test_pack_rows_ragged_k_and_strided_source():
    """K = 576 (two and a quarter wave chunks), source with a padded leading dimension, and a
    source whose rows are not 16-byte aligned (scalar-load variant)."""
    K, beta = 576, 64
    x = synth.relu_normal(7, (37, K))
    wide = torch.zeros((37, K + 24), dtype=torch.float32, device="cuda")
    wide[:, :K] = dev(x)
    for src in (wide[:, :K], ):
        bits, scales = hbmm.quantize_pack(src, beta)
        assert np.array_equal(words(bits), oracle.sign_pack(x))
        ref = oracle.block_scales(x, beta)
        assert np.all(np.abs(scales.cpu().numpy() - ref) <= scale_tol(beta) * ref + 1e-30)
    odd = torch.zeros((37, K + 3), dtype=torch.float32, device="cuda")
    odd[:, :K] = dev(x)
    bits, scales = hbmm.quantize_pack(odd[:, :K], beta)
    assert np.array_equal(words(bits), oracle.sign_pack(x))
    assert (words(bits)[:, K // 32:] == 0).all()


@pytest.mark.parametrize("beta", [2, 4, 8, 16, 32, 64, 128, 256])
def test_pack_cols(beta):
    K, rows = 1024, 333
    xkn = synth.normal(200 + beta, (K, rows))
    bits, scales = hbmm.quantize_pack(dev(xkn), beta, layout=1)
    xt = oracle.as_rows_by_k(xkn, 1)
    assert np.array_equal(words(bits), oracle.sign_pack(xt))
    # double-precision sequential sum in the same order as the oracle: identical fp32 scales
    assert np.array_equal(scales.cpu().numpy(), oracle.block_scales(xt, beta))


def _random_pack_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        beta = int(rng.choice([2, 4, 8, 16, 32, 64, 128, 256]))
        K = max(32, beta) * int(rng.integers(1, 40))
        cases.append((int(rng.integers(1, 300)), K, beta, int(rng.integers(0, 2)), int(rng.choice([0, 4, 5, 64])), int(rng.integers(0, 3))))
    return cases


@pytest.mark.parametrize("rows,K,beta,layout,pad,kind", _random_pack_cases(32, 20260103))
def test_pack_seeded_random_sweep(rows, K, beta, layout, pad, kind):
    """Shapes, segment lengths, both source layouts and padded (aligned and unaligned) leading dimensions
    drawn from a fixed seed; backward of the same operand on the way."""
    make = [synth.normal, synth.relu_normal, synth.uniform_pm1]
    x = make[kind](6000 + rows + K, (rows, K))
    src_shape = (rows, K) if layout == 0 else (K, rows)
    wide = torch.zeros((src_shape[0], src_shape[1] + pad), dtype=torch.float32, device="cuda")
    wide[:, :src_shape[1]] = dev(x if layout == 0 else np.ascontiguousarray(x.T))
    bits, scales = hbmm.quantize_pack(wide[:, :src_shape[1]], beta, layout=layout)
    assert np.array_equal(words(bits), oracle.sign_pack(x))
    ref = oracle.block_scales(x, beta)
    assert np.all(np.abs(scales.cpu().numpy() - ref) <= scale_tol(beta) * ref + 1e-30)
    if layout == 0:
        g = synth.normal(6001 + rows, (rows, K))
        gw = torch.zeros_like(wide)
        gw[:, :K] = dev(g)
        rb, Tb = oracle.binarize_backward(x, g, beta, want_T=True)
        got = hbmm.binarize_backward(wide[:, :K], gw[:, :K], beta).cpu().numpy()
        assert np.all(np.abs(got.astype(np.float64) - rb) <= (np.log2(beta) + 3) * 2.0 ** -24 * Tb + 1e-30)


def test_pack_all_zero_and_negative():
    x = np.zeros((4, 256), dtype=np.float32)
    x[1] = -1.0
    x[2] = -0.0
    bits, scales = hbmm.quantize_pack(dev(x), 128)
    w = words(bits)
    assert (w[0, :8] == 0xFFFFFFFF).all() and (w[1] == 0).all() and (w[2, :8] == 0xFFFFFFFF).all()
    assert np.array_equal(scales.cpu().numpy(), np.array([[0, 0], [1, 1], [0, 0], [0, 0]], dtype=np.float32))


def test_pack_non_finite_inputs():
    """NaN and infinities are outside the method's domain, but the pass must treat them as the
    comparison x >= 0 does and keep their damage inside their own segment."""
    x = synth.normal(77, (70, 1024))
    x[3, 5], x[3, 300], x[40, 1023], x[69, 0] = np.nan, np.inf, -np.inf, -np.nan
    for beta in (4, 32, 256):
        bits, scales = hbmm.quantize_pack(dev(x), beta)
        assert np.array_equal(words(bits), oracle.sign_pack(x))
        got, ref = scales.cpu().numpy(), oracle.block_scales(x, beta)
        bad = ~np.isfinite(ref)
        assert bad.sum() == 4 and np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
        assert np.all(np.abs(got[~bad] - ref[~bad]) <= 16 * 2.0 ** -24 * ref[~bad])


# ---------------------------------------------------------------------------------- gemm_int
@pytest.mark.parametrize("M,N,K", [(64, 64, 512), (1, 1, 32), (300, 130, 1000), (257, 129, 544), (40, 600, 4608),
                                   (513, 17, 96), (2100, 1990, 1000), (700, 4100, 352)])
def test_gemm_int_bit_exact(M, N, K):
    A, B = synth.normal(300 + M, (M, K)), synth.normal(301 + N, (N, K))
    a, b = oracle.sign_pack(A), oracle.sign_pack(B)
    D = hbmm.gemm_int(dev(a.view(np.int32)), dev(b.view(np.int32)), K)
    assert np.array_equal(D.cpu().numpy(), oracle.int_dot(a, b, K))


# -------------------------------------------------------------------------------------- gemm
def run_gemm_case(A, B, beta_a, beta_w, algo=0):
    """GEMM parity with the SAME packed words and fp32 scales on both sides (oracle-made), so that
    only the contraction and its epilogue are under test."""
    M, K = A.shape
    a_bits, b_bits = oracle.sign_pack(A), oracle.sign_pack(B)
    a_s, b_s = oracle.block_scales(A, beta_a), oracle.block_scales(B, beta_w)
    ref, T = oracle.popcount_gemm(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T=True)
    got = hbmm.gemm(dev(a_bits.view(np.int32)), dev(a_s), beta_a, dev(b_bits.view(np.int32)), dev(b_s), beta_w, K,
                    algo=algo)
    return assert_close_to_oracle(got.cpu().numpy(), ref, T, f"gemm {A.shape}x{B.shape} b=({beta_a},{beta_w})")


# (small grids run on 64-row workgroups, large ones on 256-row workgroups: the last two shapes are ragged
# in both dimensions and large enough for the latter)
@pytest.mark.parametrize("beta", [32, 64, 128, 256])
@pytest.mark.parametrize("M,N,K", [(64, 64, 512), (300, 200, 1024), (129, 257, 1536), (5, 3, 256), (260, 140, 4608),
                                   (2100, 1990, 1024), (4100, 700, 768)])
def test_gemm_equal_beta(beta, M, N, K):
    run_gemm_case(synth.normal(400 + M, (M, K)), synth.uniform_pm1(401 + N, (N, K)), beta, beta)


@pytest.mark.parametrize("beta_a,beta_w", [(32, 32), (64, 128), (128, 128), (256, 64)])
@pytest.mark.parametrize("M,N", [(1000, 2066), (1185, 2599), (1259, 2599), (520, 9001)])
def test_gemm_grids_between_whole_rounds(beta_a, beta_w, M, N):
    """Shapes whose 64-row tiling leaves the last round of workgroups nearly empty: the launcher then takes
    fewer rows of the broadcast operand per wave (12, 13 or 14 instead of 16).  Odd sizes on both sides, so
    every tile size meets a ragged edge."""
    run_gemm_case(synth.normal(300 + M, (M, 512)), synth.normal(301 + N, (N, 512)), beta_a, beta_w)


@pytest.mark.parametrize("beta_a,beta_w", [(32, 64), (64, 32), (32, 256), (256, 32), (128, 64), (64, 256)])
def test_gemm_mixed_beta(beta_a, beta_w):
    run_gemm_case(synth.relu_normal(500, (150, 1280)), synth.normal(501, (270, 1280), std=0.04), beta_a, beta_w)
    run_gemm_case(synth.relu_normal(502, (2050, 1280)), synth.normal(503, (1100, 1280), std=0.04), beta_a, beta_w)


@pytest.mark.parametrize("beta", [32, 64, 128, 256])
@pytest.mark.parametrize("M,N,K", [(64, 64, 512), (300, 200, 1024), (129, 257, 1536), (5, 3, 256), (260, 140, 4608)])
def test_gemm_mfma_i8_equal_beta(beta, M, N, K):
    """The int8 matrix-core comparison variant must give the same product -- bit for bit, since its
    integer dots are the same and its epilogue rounds in the same places."""
    A, B = synth.normal(400 + M, (M, K)), synth.uniform_pm1(401 + N, (N, K))
    run_gemm_case(A, B, beta, beta, algo=1)
    ab, as_ = hbmm.quantize_pack(dev(A), beta)
    bb, bs = hbmm.quantize_pack(dev(B), beta)
    assert torch.equal(hbmm.gemm(ab, as_, beta, bb, bs, beta, K, algo=0), hbmm.gemm(ab, as_, beta, bb, bs, beta, K, algo=1))


@pytest.mark.parametrize("beta_a,beta_w,K", [(32, 64, 1280), (256, 32, 1280), (128, 64, 1280), (64, 256, 1280),
                                             (32, 32, 1248), (64, 64, 576), (32, 96 // 3, 96)])
def test_gemm_mfma_i8_mixed_and_ragged(beta_a, beta_w, K):
    """Mixed segment lengths, and K whose word count is not a multiple of the 4-word stage."""
    run_gemm_case(synth.normal(510, (150, K)), synth.normal(511, (270, K), std=0.04), beta_a, beta_w, algo=1)


@pytest.mark.parametrize("beta", [64, 128, 256])
@pytest.mark.parametrize("M,N,K", [(64, 64, 512), (300, 200, 1024), (129, 257, 1536), (5, 3, 256), (260, 140, 4608), (513, 130, 768)])
def test_gemm_mfma_fp4_equal_beta(beta, M, N, K):
    """The 4-bit-float matrix-core variant: +-1 products are exact, segment sums are exact small
    integers in fp32 and the epilogue is the popcount kernel's, so the result is the same bit for bit."""
    A, B = synth.normal(600 + M, (M, K)), synth.uniform_pm1(601 + N, (N, K))
    run_gemm_case(A, B, beta, beta, algo=2)
    ab, as_ = hbmm.quantize_pack(dev(A), beta)
    bb, bs = hbmm.quantize_pack(dev(B), beta)
    assert torch.equal(hbmm.gemm(ab, as_, beta, bb, bs, beta, K, algo=0), hbmm.gemm(ab, as_, beta, bb, bs, beta, K, algo=2))


@pytest.mark.parametrize("beta_a,beta_w,K", [(64, 128, 1280), (256, 64, 1280), (128, 64, 1280), (64, 256, 1280),
                                             (64, 64, 576), (128, 128, 640), (64, 64, 64), (64, 64, 1984)])
def test_gemm_mfma_fp4_mixed_and_ragged(beta_a, beta_w, K):
    """Mixed segment lengths, and K whose word count is not a multiple of the 8-word stage (the
    stage's tail words lie past the row or are pad words: they must not count)."""
    run_gemm_case(synth.normal(610, (150, K)), synth.normal(611, (270, K), std=0.04), beta_a, beta_w, algo=2)


@pytest.mark.parametrize("beta_a,beta_w", [(32, 64), (64, 64), (256, 128), (8, 32), (1, 64)])
def test_gemm_fastest_algo_gives_the_same_bits(beta_a, beta_w):
    A, B = synth.normal(620, (140, 512)), synth.normal(621, (200, 512), std=0.05)
    bb, bs = hbmm.quantize_pack(dev(B), beta_w)
    if beta_a == 1:
        ab, as_ = None, dev(A)
    else:
        ab, as_ = hbmm.quantize_pack(dev(A), beta_a)
    assert torch.equal(hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, 512, algo=hbmm.ALGO_FASTEST),
                       hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, 512, algo=hbmm.ALGO_POPCOUNT))


@pytest.mark.parametrize("beta_a,beta_w,M,N,K", [
    (ba, bw, M, N, K)
    for (ba, bw) in [(16, 16), (32, 32), (16, 32), (32, 16), (16, 256), (128, 32), (64, 16)]
    for (M, N, K) in [(64, 64, 512), (300, 200, 1024), (129, 257, 1536), (5, 3, 128), (513, 130, 640)]
    if K % max(ba, bw) == 0])
def test_gemm_mfma_fp8_short_segments(beta_a, beta_w, M, N, K):
    """8-bit-float matrix-core kernel for segments of 16 or 32: against the oracle, and bit for bit
    against the popcount kernel where that one applies (both beta >= 32)."""
    A, B = synth.normal(700 + M, (M, K)), synth.uniform_pm1(701 + N, (N, K))
    run_gemm_case(A, B, beta_a, beta_w, algo=3)
    if beta_a >= 32 and beta_w >= 32:
        ab, as_ = hbmm.quantize_pack(dev(A), beta_a)
        bb, bs = hbmm.quantize_pack(dev(B), beta_w)
        assert torch.equal(hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K, algo=0), hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K, algo=3))


def test_gemm_mfma_fp8_unsupported():
    A, B = synth.normal(1, (8, 96)), synth.normal(2, (8, 96))
    ab, as_ = hbmm.quantize_pack(dev(A), 16)
    bb, bs = hbmm.quantize_pack(dev(B), 16)
    with pytest.raises(hbmm.HbmmError):
        hbmm.gemm(ab, as_, 16, bb, bs, 16, 96, algo=3)       # K not a multiple of 128
    A, B = synth.normal(1, (8, 128)), synth.normal(2, (8, 128))
    ab, as_ = hbmm.quantize_pack(dev(A), 8)
    bb, bs = hbmm.quantize_pack(dev(B), 16)
    with pytest.raises(hbmm.HbmmError):
        hbmm.gemm(ab, as_, 8, bb, bs, 16, 128, algo=3)       # a segment shorter than 16
    ab, as_ = hbmm.quantize_pack(dev(A), 64)
    bb, bs = hbmm.quantize_pack(dev(B), 64)
    with pytest.raises(hbmm.HbmmError):
        hbmm.gemm(ab, as_, 64, bb, bs, 64, 128, algo=3)      # both segments longer than 32


def test_gemm_mfma_fp4_unsupported():
    A, B = synth.normal(1, (8, 64)), synth.normal(2, (8, 64))
    ab, as_ = hbmm.quantize_pack(dev(A), 32)
    bb, bs = hbmm.quantize_pack(dev(B), 64)
    with pytest.raises(hbmm.HbmmError):
        hbmm.gemm(ab, as_, 32, bb, bs, 64, 64, algo=2)


def test_gemm_against_dense_f64_path_end_to_end():
    """Whole hot path on the GPU (pack A, pack B, gemm) against the dense double-precision oracle
    that materialises delta (.) Sign(.) and multiplies.  GPU-made scales differ from the oracle's
    by a few ulp, which the same tolerance absorbs."""
    M, N, K, beta = 200, 136, 2048, 64
    A, B = synth.normal(600, (M, K)), synth.normal(601, (N, K))
    ab, as_ = hbmm.quantize_pack(dev(A), beta)
    bb, bs = hbmm.quantize_pack(dev(B), beta)
    got = hbmm.gemm(ab, as_, beta, bb, bs, beta, K).cpu().numpy()
    ref = oracle.hbmm_dense(A, B, beta, beta)
    _, T = oracle.hbmm_popcount(A, B, beta, beta, want_T=True)
    assert_close_to_oracle(got, ref, T, "end to end")


def test_gemm_whole_row_scale_is_xnor_net():
    """beta = K = 256 for both operands: C = sA[m] sB[n] D[m, n]."""
    K = 256
    A, B = synth.normal(610, (70, K)), synth.normal(611, (90, K))
    ab, as_ = hbmm.quantize_pack(dev(A), K)
    bb, bs = hbmm.quantize_pack(dev(B), K)
    C = hbmm.gemm(ab, as_, K, bb, bs, K, K).cpu().numpy().astype(np.float64)
    D = hbmm.gemm_int(ab, bb, K).cpu().numpy().astype(np.float64)
    want = as_.cpu().numpy().astype(np.float64) * bs.cpu().numpy().astype(np.float64).T * D
    assert np.allclose(C, want, rtol=3e-7, atol=0)


@pytest.mark.parametrize("beta_w", [32, 64, 128, 256])
@pytest.mark.parametrize("M,N,K", [(64, 64, 512), (100, 70, 1280), (33, 130, 4608)])
def test_gemm_binary_weight(beta_w, M, N, K):
    """beta_a = 1: fp32 activations against packed weights."""
    A, B = synth.relu_normal(700 + M, (M, K)), synth.normal(701 + N, (N, K), std=float(np.sqrt(2.0 / K)))
    b_bits, b_s = oracle.sign_pack(B), oracle.block_scales(B, beta_w)
    ref, T = oracle.binary_weight_gemm(A, b_bits, b_s, beta_w, want_T=True)
    got = hbmm.gemm(None, dev(A), 1, dev(b_bits.view(np.int32)), dev(b_s), beta_w, K)
    assert_close_to_oracle(got.cpu().numpy(), ref, T, "binary weight")


def split_case(A, B, beta_a, beta_w):
    """Matrix-core path (a segment shorter than 32 or an unquantised operand on one side): the
    oracle is the dense definition; T = |A~| . |B~|^T."""
    At, Bt = oracle.materialize(A, beta_a), oracle.materialize(B, beta_w)
    ref, T = oracle.dense_f64_gemm(At, Bt), oracle.dense_f64_gemm(np.abs(At), np.abs(Bt))
    K = A.shape[1]

    def operand(x, beta):
        if beta == 1:
            return None, dev(x)
        return dev(oracle.sign_pack(x).view(np.int32)), dev(oracle.block_scales(x, beta))

    (ab, as_), (bb, bs) = operand(A, beta_a), operand(B, beta_w)
    got = hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K)
    return assert_close_to_oracle(got.cpu().numpy(), ref, T, f"split {A.shape}x{B.shape} b=({beta_a},{beta_w})")


@pytest.mark.parametrize("beta_a,beta_w", [(1, 16), (2, 16), (4, 16), (8, 16), (16, 16), (2, 32), (4, 64), (8, 128),
                                           (16, 256), (2, 256), (16, 2), (32, 4), (256, 8), (64, 16), (16, 32),
                                           (16, 1), (128, 1), (1, 256),
                                           (1, 2), (1, 4), (1, 8), (2, 1), (4, 1), (8, 1)])
def test_gemm_short_segments(beta_a, beta_w):
    """Segments of 2..16 on either side (the settings the paper trains with), mixed with long ones,
    and an unquantised operand on either side -- including the paper's binary-weight networks with
    beta_w = 4 and 8 (Tables 2-3: beta_a = 1)."""
    A = synth.normal(900 + beta_a, (200, 1280))
    B = synth.normal(901 + beta_w, (300, 1280), std=0.05)
    split_case(A, B, beta_a, beta_w)


@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (130, 260, 96), (257, 513, 1024), (64, 64, 4608)])
def test_gemm_short_segments_shapes(M, N, K):
    split_case(synth.relu_normal(910 + M, (M, K)), synth.normal(911 + N, (N, K)), 4, 16)
    split_case(synth.normal(912 + M, (M, K)), synth.uniform_pm1(913 + N, (N, K)), 16, 2)
    split_case(synth.relu_normal(914 + M, (M, K)), synth.normal(915 + N, (N, K)), 1, 4)
    split_case(synth.normal(916 + M, (M, K)), synth.normal(917 + N, (N, K)), 8, 1)


@pytest.mark.parametrize("beta_a,beta_w", [(2, 2), (4, 4), (8, 8), (2, 8), (8, 2), (4, 2), (8, 4)])
def test_gemm_both_segments_short(beta_a, beta_w):
    """Both segments shorter than 16 (e.g. the paper's HadaNet with beta_w = beta_a = 4): both operands
    are rebuilt as fp32 values on the fly."""
    split_case(synth.normal(920 + beta_a, (200, 1280)), synth.normal(921 + beta_w, (300, 1280), std=0.05), beta_a, beta_w)
    split_case(synth.relu_normal(922 + beta_a, (129, 96)), synth.uniform_pm1(923 + beta_w, (1, 96)), beta_a, beta_w)


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    betas = [1, 2, 4, 8, 16, 32, 64, 128, 256]
    cases = []
    while len(cases) < n:
        beta_a, beta_w = int(rng.choice(betas)), int(rng.choice(betas))
        if beta_a == 1 and beta_w == 1:
            continue                      # a plain dense product: reported as unsupported (tested elsewhere)
        unit = max(32, beta_a, beta_w)
        K = unit * int(rng.integers(1, max(2, 1536 // unit) + 1))
        M, N = int(rng.integers(1, 420)), int(rng.integers(1, 420))
        cases.append((M, N, K, beta_a, beta_w, int(rng.choice([0, -1])), int(rng.integers(0, 3)), int(rng.integers(0, 3))))
    return cases


@pytest.mark.parametrize("M,N,K,beta_a,beta_w,algo,kind_a,kind_b", _random_cases(56, 20260101))
def test_gemm_seeded_random_sweep(M, N, K, beta_a, beta_w, algo, kind_a, kind_b):
    """Shapes, segment lengths, kernel choice and value distributions drawn from a fixed seed, against
    the dense double-precision definition."""
    make = [lambda s, sh: synth.normal(s, sh), lambda s, sh: synth.relu_normal(s, sh), lambda s, sh: synth.uniform_pm1(s, sh)]
    A, B = make[kind_a](4000 + M, (M, K)), make[kind_b](5000 + N, (N, K))
    At, Bt = oracle.materialize(A, beta_a), oracle.materialize(B, beta_w)
    ref, T = oracle.dense_f64_gemm(At, Bt), oracle.dense_f64_gemm(np.abs(At), np.abs(Bt))
    if beta_a >= 32 and beta_w >= 32:
        # the XNOR + popcount kernel (and its matrix-core twins) add one term per segment: its error scale
        # is the sum of the absolute segment terms, about sqrt(segment length) tighter than |A~| . |B~|^T
        _, T = oracle.hbmm_popcount(A, B, beta_a, beta_w, want_T=True)

    def operand(x, beta):
        if beta == 1:
            return None, dev(x)
        return dev(oracle.sign_pack(x).view(np.int32)), dev(oracle.block_scales(x, beta))

    (ab, as_), (bb, bs) = operand(A, beta_a), operand(B, beta_w)
    got = hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K, algo=algo)
    assert_close_to_oracle(got.cpu().numpy(), ref, T, f"sweep {M}x{N}x{K} b=({beta_a},{beta_w}) algo {algo}")


# ------------------------------------------------------------------------------ general beta and K
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("rows,K,beta", [(3, 19, 5), (7, 19, 3), (1, 1, 2), (33, 100, 7), (130, 1000, 48), (5, 257, 256),
                                          (9, 96, 6), (40, 333, 32), (17, 64, 3), (2, 4100, 255), (65, 31, 16)])
def test_pack_any_beta_and_ragged_k(rows, K, beta, layout):
    """Segment lengths that are not powers of two, K that beta does not divide (the last segment is the
    shorter remainder, averaged over its own length) and K that does not fill its last 32-bit word.
    Double-precision sequential sums rounded once: the scales are the oracle's bit for bit."""
    x = synth.normal(7000 + rows + K + beta, (rows, K))
    x[0, :min(K, 4)] = [0.0, -0.0, 1e-38, -1e-38][:min(K, 4)]
    src = dev(x) if layout == 0 else dev(np.ascontiguousarray(x.T))
    nb = -(-K // beta)
    scales = torch.full((rows, nb + 2), -7.0, dtype=torch.float32, device="cuda")
    bits, _ = hbmm.quantize_pack(src, beta, layout, None, scales[:, :nb])
    assert np.array_equal(words(bits), oracle.sign_pack(x))
    got = scales.cpu().numpy()
    assert np.array_equal(got[:, :nb], oracle.block_scales(x, beta))
    assert (got[:, nb:] == -7.0).all()


@pytest.mark.parametrize("M,N,K,beta_a,beta_w", [
    (4, 3, 19, 3, 5), (4, 3, 19, 5, 3), (130, 260, 19, 3, 5), (200, 300, 1000, 7, 6), (257, 129, 96, 3, 16),
    (64, 64, 1280, 5, 1), (70, 90, 333, 1, 7), (33, 40, 100, 32, 48), (129, 131, 4607, 255, 9), (50, 60, 31, 2, 4),
    (1, 1, 1, 2, 2), (150, 140, 1056, 12, 12), (90, 200, 2000, 64, 100), (300, 10, 65, 1, 64), (10, 300, 70, 64, 1)])
def test_gemm_any_beta_and_ragged_k(M, N, K, beta_a, beta_w):
    """General segment lengths and K against the dense double-precision definition: operands packed by the
    oracle, so this checks the product alone (the pack kernel has its own test above)."""
    split_case(synth.normal(7100 + M + K, (M, K)), synth.normal(7101 + N + K, (N, K), std=0.05), beta_a, beta_w)


@pytest.mark.parametrize("M,N,K,beta_a,beta_w", [
    (70, 90, 70, 32, 32), (130, 260, 4100, 64, 64), (200, 150, 1000, 128, 32), (300, 64, 523, 256, 64),
    (50, 40, 33, 32, 256), (64, 64, 31, 32, 32), (10, 10, 1, 32, 32), (9, 7, 255, 256, 256), (100, 80, 513, 128, 128),
    (2100, 2100, 1030, 64, 32), (20000, 2000, 600, 64, 64), (1500, 3000, 2047, 32, 32)])
def test_gemm_word_segments_with_a_shorter_last_one(M, N, K, beta_a, beta_w):
    """Power-of-two segments of 32 bits or more and a K that they, or a 32-bit word, do not divide: the XNOR +
    popcount kernel with the last, shorter segment counted over the elements that exist (Eq. 7 with the
    remainder as its last term).  Against the oracle's own popcount form and its per-segment error scale;
    grids of one workgroup, of a few (the small-grid forms) and of several rounds (the 128- and 256-row forms)."""
    A, B = synth.normal(7500 + M + K, (M, K)), synth.normal(7501 + N + K, (N, K), std=0.05)
    ab, as_, bb, bs = oracle.sign_pack(A), oracle.block_scales(A, beta_a), oracle.sign_pack(B), oracle.block_scales(B, beta_w)
    ref, T = oracle.popcount_gemm(ab, as_, beta_a, bb, bs, beta_w, K, want_T=True)
    got = hbmm.gemm(dev(ab.view(np.int32)), dev(as_), beta_a, dev(bb.view(np.int32)), dev(bs), beta_w, K, algo=0)
    assert_close_to_oracle(got.cpu().numpy(), ref, T, f"ragged K {M}x{N}x{K} b=({beta_a},{beta_w})")
    if M * N <= 70000:
        # and the same numbers from the definition on materialised operands
        dense = oracle.dense_f64_gemm(oracle.materialize(A, beta_a), oracle.materialize(B, beta_w))
        assert np.allclose(ref, dense, rtol=1e-12, atol=1e-12 * np.abs(dense).max())
    for algo in (1, 2, 3):
        with pytest.raises(hbmm.HbmmError) as ei:
            hbmm.gemm(dev(ab.view(np.int32)), dev(as_), beta_a, dev(bb.view(np.int32)), dev(bs), beta_w, K, algo=algo)
        assert ei.value.code == hbmm.EUNSUPPORTED


def _random_any_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        beta_a, beta_w = int(rng.integers(1, 257)), int(rng.integers(1, 257))
        if rng.integers(0, 3) == 0:
            beta_a = int(rng.integers(1, 17))
        if rng.integers(0, 3) == 0:
            beta_w = int(rng.integers(1, 17))
        if beta_a == 1 and beta_w == 1:
            continue
        cases.append((int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 1500)), beta_a, beta_w,
                      int(rng.integers(0, 3)), int(rng.integers(0, 3))))
    return cases


@pytest.mark.parametrize("M,N,K,beta_a,beta_w,kind_a,kind_b", _random_any_cases(40, 20260104))
def test_gemm_any_beta_seeded_random_sweep(M, N, K, beta_a, beta_w, kind_a, kind_b):
    """Any segment lengths in 1..256 and any K, packed on the GPU and multiplied there (algo -1), against the
    dense double-precision definition."""
    make = [synth.normal, synth.relu_normal, synth.uniform_pm1]
    A, B = make[kind_a](7300 + M, (M, K)), make[kind_b](7400 + N, (N, K))
    At, Bt = oracle.materialize(A, beta_a), oracle.materialize(B, beta_w)
    ref, T = oracle.dense_f64_gemm(At, Bt), oracle.dense_f64_gemm(np.abs(At), np.abs(Bt))

    def operand(x, beta):
        if beta == 1:
            return None, dev(x)
        bits, scales = hbmm.quantize_pack(dev(x), beta)
        assert np.array_equal(words(bits), oracle.sign_pack(x))
        # tuned kernels: pairwise fp32 sums; general kernel: the oracle's own rounding
        ref_s = oracle.block_scales(x, beta)
        assert np.all(np.abs(scales.cpu().numpy() - ref_s) <= scale_tol(beta) * ref_s + 1e-30)
        return bits, scales

    (ab, as_), (bb, bs) = operand(A, beta_a), operand(B, beta_w)
    got = hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K, algo=-1)
    assert_close_to_oracle(got.cpu().numpy(), ref, T, f"any-beta sweep {M}x{N}x{K} b=({beta_a},{beta_w})")


def test_gemm_any_beta_end_to_end_and_strided():
    """Pack on the GPU, multiply on the GPU; the unquantised operand with a leading dimension that is not
    a multiple of 4 and an output with a padded leading dimension."""
    M, N, K = 77, 130, 203
    A, B = synth.relu_normal(7200, (M, K)), synth.normal(7201, (N, K), std=0.05)
    At, Bt = oracle.materialize(A, 1), oracle.materialize(B, 7)
    ref, T = oracle.dense_f64_gemm(At, Bt), oracle.dense_f64_gemm(np.abs(At), np.abs(Bt))
    wide = torch.zeros((M, K + 3), dtype=torch.float32, device="cuda")
    wide[:, :K] = dev(A)
    bb, bs = hbmm.quantize_pack(dev(B), 7)
    out = torch.full((M, N + 5), -3.0, dtype=torch.float32, device="cuda")
    hbmm.gemm(None, wide[:, :K], 1, bb, bs, 7, K, out=out[:, :N])
    got = out.cpu().numpy()
    assert_close_to_oracle(got[:, :N], ref, T, "any-beta end to end")
    assert (got[:, N:] == -3.0).all()
    # and both sides packed on the GPU with different odd segment lengths
    ab, as_ = hbmm.quantize_pack(dev(A), 11)
    At = oracle.materialize(A, 11)
    ref, T = oracle.dense_f64_gemm(At, Bt), oracle.dense_f64_gemm(np.abs(At), np.abs(Bt))
    assert_close_to_oracle(hbmm.gemm(ab, as_, 11, bb, bs, 7, K).cpu().numpy(), ref, T, "any-beta (11, 7)")


def test_gemm_any_beta_limits():
    x = torch.zeros((4, 96), dtype=torch.float32, device="cuda")
    bits, scales = hbmm.quantize_pack(x, 6)
    for algo in (1, 2, 3):
        with pytest.raises(hbmm.HbmmError) as ei:
            hbmm.gemm(bits, scales, 6, bits, scales, 6, 96, algo=algo)
        assert ei.value.code == hbmm.EUNSUPPORTED
    with pytest.raises(hbmm.HbmmError) as ei:
        hbmm.quantize_pack(x, 257)
    assert ei.value.code == hbmm.EUNSUPPORTED


def test_gemm_two_unquantised_operands_are_reported_unsupported():
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(hbmm.HbmmError) as ei:
        hbmm.gemm(None, x, 1, None, x, 1, 64)
    assert ei.value.code == hbmm.EUNSUPPORTED


def test_gemm_empty_and_zero_k():
    e = torch.empty((0, 4), dtype=torch.int32, device="cuda")
    s = torch.empty((0, 1), dtype=torch.float32, device="cuda")
    b = torch.zeros((8, 4), dtype=torch.int32, device="cuda")
    sb = torch.ones((8, 1), dtype=torch.float32, device="cuda")
    assert hbmm.gemm(e, s, 32, b, sb, 32, 32).shape == (0, 8)
    assert hbmm.gemm_int(e, b, 32).shape == (0, 8)


def test_unsupported_is_reported_not_faked():
    x = torch.zeros((4, 96), dtype=torch.float32, device="cuda")
    with pytest.raises(hbmm.HbmmError) as ei:
        hbmm.quantize_pack(x, 512)
    assert ei.value.code == hbmm.EUNSUPPORTED


# -------------------------------------------------------------------------- dense comparison
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 130, 256), (64, 300, 1024), (257, 129, 4608)])
def test_dense_ref_gemm(dtype, M, N, K):
    """C = A . B^T on unquantised operands against a double-precision library product of the same
    (already rounded) operands; fp32 accumulation, so the error is taken relative to sum |a||b|."""
    A, B = synth.normal(800 + M, (M, K)), synth.normal(801 + N, (N, K))
    dA, dB = dev(A), dev(B)
    if dtype == "bf16":
        dA, dB = dA.to(torch.bfloat16), dB.to(torch.bfloat16)
        A, B = dA.float().cpu().numpy(), dB.float().cpu().numpy()
    got = hbmm.dense_ref_gemm(dA, dB).cpu().numpy()
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    T = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64)).T
    assert_close_to_oracle(got, ref, T, f"dense {dtype}")


# ------------------------------------------------------------------- backward of the binarisation
@pytest.mark.parametrize("beta", [1, 2, 4, 8, 16, 32, 64, 128, 256])
@pytest.mark.parametrize("rows,K", [(1, 256), (7, 768), (33, 4608), (130, 1280)])
def test_binarize_backward(beta, rows, K):
    x = synth.normal(1000 + beta + rows, (rows, K)) * 1.2
    x[0, :6] = [1.0, -1.0, 0.0, -0.0, 1.0000001, -0.99999994]
    g = synth.normal(1001 + beta + K, (rows, K))
    got = hbmm.binarize_backward(dev(x), dev(g), beta).cpu().numpy()
    ref, T = oracle.binarize_backward(x, g, beta, want_T=True)
    assert_close_to_oracle(got, ref, T, f"backward beta={beta}")


@pytest.mark.parametrize("rows,K,beta", [(3, 19, 5), (7, 19, 3), (1, 1, 2), (33, 100, 7), (40, 1000, 48), (5, 257, 256),
                                          (9, 96, 6), (17, 70, 64), (2, 4100, 255), (65, 31, 16), (8, 50, 1)])
def test_binarize_backward_any_beta_and_ragged_k(rows, K, beta):
    """Eq. 6 for segment lengths that are not powers of two and a K that beta does not divide: the last segment
    has delta averaged over its own length n and 1/n in place of 1/beta."""
    x = synth.normal(8700 + rows + K, (rows, K)) * 1.2
    x[0, :min(K, 4)] = [1.0, -1.0, 0.0, 1.0000001][:min(K, 4)]
    g = synth.normal(8701 + rows + beta, (rows, K))
    got = hbmm.binarize_backward(dev(x), dev(g), beta).cpu().numpy()
    ref, T = oracle.binarize_backward(x, g, beta, want_T=True)
    assert_close_to_oracle(got, ref, T, f"backward any beta={beta} K={K}")


def test_binarize_backward_ragged_and_strided():
    K, beta = 96, 8
    x, g = synth.normal(1010, (9, K)), synth.normal(1011, (9, K))
    wide_x = torch.zeros((9, K + 3), dtype=torch.float32, device="cuda")
    wide_x[:, :K] = dev(x)
    out = torch.full((9, K + 8), 5.0, dtype=torch.float32, device="cuda")
    hbmm.binarize_backward(wide_x[:, :K], dev(g), beta, out[:, :K])
    ref, T = oracle.binarize_backward(x, g, beta, want_T=True)
    assert_close_to_oracle(out[:, :K].cpu().numpy(), ref, T, "backward strided")
    assert (out[:, K:] == 5.0).all()


# ------------------------------------------------------------------------------ streams and graphs
def test_whole_path_in_a_hip_graph_replays_exactly():
    """pack(A), pack(B), gemm captured once into a HIP graph: every replay (with eager work and
    synchronisations of the program in between, and new input values written into the same buffers)
    must reproduce the eager result bit for bit.  The library allocates nothing, issues no memset and
    never synchronises, so it is capturable as is."""
    M, N, K, beta = 300, 200, 1024, 64
    A0, B0 = synth.normal(1100, (M, K)), synth.normal(1101, (N, K))
    A1, B1 = synth.uniform_pm1(1102, (M, K)), synth.normal(1103, (N, K))
    dA, dB = dev(A0), dev(B0)
    ldw, nb = hbmm.packed_ld_words(K), hbmm.num_blocks(K, beta)
    ab = torch.empty((M, ldw), dtype=torch.int32, device="cuda")
    bb = torch.empty((N, ldw), dtype=torch.int32, device="cuda")
    as_ = torch.empty((M, nb), dtype=torch.float32, device="cuda")
    bs = torch.empty((N, nb), dtype=torch.float32, device="cuda")
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")

    def step():
        hbmm.quantize_pack(dA, beta, 0, ab, as_)
        hbmm.quantize_pack(dB, beta, 0, bb, bs)
        hbmm.gemm(ab, as_, beta, bb, bs, beta, K, out=C)

    def eager(a, b):
        dA.copy_(dev(a)); dB.copy_(dev(b))
        step()
        torch.cuda.synchronize()
        return C.clone()

    want0, want1 = eager(A0, B0), eager(A1, B1)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for rep in range(4):
        a, b, want = (A0, B0, want0) if rep % 2 == 0 else (A1, B1, want1)
        dA.copy_(dev(a)); dB.copy_(dev(b))
        C.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        assert torch.equal(C, want), f"replay {rep} differs from the eager result"
        _ = (dA.sum() + dB.sum()).item()   # unrelated eager work between replays


def test_layer_pipeline_in_a_hip_graph_replays_exactly():
    """A layer as it would run in inference -- binarise the activation tensor, convolution from the
    packed tensors, and a matrix-core product of the flattened result -- captured once and replayed:
    none of these entry points allocates, clears memory with a memset or synchronises."""
    B, C, H, W, N, beta_a, beta_w = 2, 32, 8, 16, 64, 4, 32
    X0, X1 = synth.relu_normal(1200, (B, C, H, W)), synth.relu_normal(1201, (B, C, H, W))
    F = synth.normal(1202, (N, C, 3, 3), std=0.1)
    L = synth.normal(1203, (40, N * H * W // 16), std=0.1)     # a "linear layer" over 1/16 of the features per row
    dX = dev(X0)
    fb, fs = hbmm.quantize_pack(dev(F.reshape(N, -1)), beta_w)
    lb, ls = hbmm.quantize_pack(dev(L), 64)
    xb = torch.empty((dX.numel() // 32,), dtype=torch.int32, device="cuda")
    xs = torch.empty((dX.numel() // beta_a,), dtype=torch.float32, device="cuda")
    Y = torch.empty((B, N, H, W), dtype=torch.float32, device="cuda")
    rows, K2 = 16 * B, N * H * W // 16
    yb = torch.empty((rows, hbmm.packed_ld_words(K2)), dtype=torch.int32, device="cuda")
    ys = torch.empty((rows, K2 // 64), dtype=torch.float32, device="cuda")
    Z = torch.empty((rows, 40), dtype=torch.float32, device="cuda")

    def step():
        hbmm.quantize_pack_tensor(dX, beta_a, xb, xs)
        hbmm.conv2d(xb, xs, beta_a, dX.shape, fb, fs, beta_w, (3, 3), 1, 1, out=Y)
        hbmm.quantize_pack(Y.view(rows, K2), 64, 0, yb, ys)
        hbmm.gemm(yb, ys, 64, lb, ls, 64, K2, algo=hbmm.ALGO_MFMA_FP4, out=Z)

    def eager(x):
        dX.copy_(dev(x))
        step()
        torch.cuda.synchronize()
        return Z.clone()

    want0, want1 = eager(X0), eager(X1)
    assert not torch.equal(want0, want1)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for rep in range(4):
        x, want = (X0, want0) if rep % 2 == 0 else (X1, want1)
        dX.copy_(dev(x))
        Z.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        assert torch.equal(Z, want), f"replay {rep} differs from the eager result"
        _ = dX.sum().item()   # unrelated eager work between replays


@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
def test_prepared_layer_pipeline_in_a_hip_graph_replays_exactly(form):
    """The same with the entry points added for settings outside the paper's table: activations of a 7-wide
    map packed with a segment length that does not divide the width, the layer with prepared filters, the
    gradient through the binarisation and a product with segment lengths that are not powers of two --
    captured once and replayed."""
    B, C, H, W, N, beta_a, beta_w = 3, 48, 7, 7, 40, 4, 5
    X0, X1 = synth.relu_normal(1300, (B, C, H, W)), synth.relu_normal(1301, (B, C, H, W))
    F = synth.normal(1302, (N, C, 3, 3), std=0.1)
    L = synth.normal(1303, (30, N * H * W), std=0.1)
    dX = dev(X0)
    fb, fs = hbmm.quantize_pack(dev(F.reshape(N, -1)), beta_w)
    prepared = hbmm.conv_prepare_filters(fb, fs, beta_w, C, (3, 3), form=form)
    K2 = N * H * W
    lb, ls = hbmm.quantize_pack(dev(L), 6)
    xb, xs = hbmm.quantize_pack_activations(dX, beta_a)
    Y = torch.empty((B, N, H, W), dtype=torch.float32, device="cuda")
    yb = torch.empty((B, hbmm.packed_ld_words(K2)), dtype=torch.int32, device="cuda")
    ys = torch.empty((B, hbmm.num_blocks(K2, 7)), dtype=torch.float32, device="cuda")
    Z = torch.empty((B, 30), dtype=torch.float32, device="cuda")
    G = torch.empty((B * C * H, W), dtype=torch.float32, device="cuda")

    def step():
        hbmm.quantize_pack_activations(dX, beta_a, xb, xs)
        hbmm.conv2d_prepared(xb, xs, beta_a, dX.shape, prepared, N, (3, 3), 1, 1, out=Y, form=form)
        hbmm.quantize_pack(Y.view(B, K2), 7, 0, yb, ys)
        hbmm.gemm(yb, ys, 7, lb, ls, 6, K2, out=Z)
        hbmm.binarize_backward(dX.view(-1, W), dX.view(-1, W), beta_a, out=G)

    def eager(x):
        dX.copy_(dev(x))
        step()
        torch.cuda.synchronize()
        return Z.clone(), G.clone()

    want0, want1 = eager(X0), eager(X1)
    assert not torch.equal(want0[0], want1[0])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for rep in range(4):
        x, want = (X0, want0) if rep % 2 == 0 else (X1, want1)
        dX.copy_(dev(x))
        Z.zero_()
        G.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        side.synchronize()
        assert torch.equal(Z, want[0]) and torch.equal(G, want[1]), f"replay {rep} differs from the eager result"
        _ = dX.sum().item()   # unrelated eager work between replays


def test_calls_on_a_side_stream():
    """Kernels go to the stream that is current when the call is made."""
    M, N, K, beta = 130, 70, 512, 128
    A, B = synth.normal(1110, (M, K)), synth.normal(1111, (N, K))
    ref = None
    for stream in (None, torch.cuda.Stream()):
        ctx = torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream())
        with ctx:
            ab, as_ = hbmm.quantize_pack(dev(A), beta)
            bb, bs = hbmm.quantize_pack(dev(B), beta)
            C = hbmm.gemm(ab, as_, beta, bb, bs, beta, K)
            torch.cuda.current_stream().synchronize()
        got = C.cpu().numpy()
        if ref is None:
            ref = got
        assert np.array_equal(ref, got)


# ------------------------------------------------------------------------------------- fused
@pytest.mark.parametrize("beta_a,beta_w,M,N,K", [
    (ba, bw, M, N, K)
    for (ba, bw) in [(32, 32), (64, 64), (128, 128), (256, 256), (32, 128), (256, 64)]
    for (M, N, K) in [(3136, 64, 576), (300, 128, 1024), (257, 5, 256), (64, 64, 512), (1000, 100, 4608), (33000, 64, 768)]
    if K % ba == 0 and K % bw == 0])
def test_gemm_fused_equals_pack_then_gemm(beta_a, beta_w, M, N, K):
    """The fused call must give bit for bit what packing A first and multiplying gives, and both
    must be within the tolerance of the oracle.  (The shapes cover the 64-row and the 128-row form.)"""
    A, B = synth.relu_normal(1200 + M, (M, K)) - 0.3, synth.normal(1201 + N, (N, K), std=0.06)
    A = A.astype(np.float32)
    dA = dev(A)
    bb, bs = hbmm.quantize_pack(dev(B), beta_w)
    ab, as_ = hbmm.quantize_pack(dA, beta_a)
    two_step = hbmm.gemm(ab, as_, beta_a, bb, bs, beta_w, K)
    fused = hbmm.gemm_fused(dA, beta_a, bb, bs, beta_w)
    assert torch.equal(fused, two_step)
    ref, T = oracle.hbmm_popcount(A, B, beta_a, beta_w, want_T=True)
    assert_close_to_oracle(fused.cpu().numpy(), ref, T, "fused")


def test_gemm_fused_limits():
    A = torch.zeros((8, 64), dtype=torch.float32, device="cuda")
    bb = torch.zeros((200, 4), dtype=torch.int32, device="cuda")
    bs = torch.ones((200, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(hbmm.HbmmError) as ei:
        hbmm.gemm_fused(A, 32, bb, bs, 32)      # N > 128
    assert ei.value.code == hbmm.EUNSUPPORTED


# ------------------------------------------------------------------------------------- convolution
def _conv_inputs(seed, B, C, H, W, N, KH, KW):
    A = synth.relu_normal(seed, (B, C, H, W))
    Wf = synth.normal(seed + 1, (N, C, KH, KW)) * np.float32(np.sqrt(2.0 / (C * KH * KW)))
    return A, Wf.astype(np.float32)


@pytest.mark.parametrize("beta,shape", [(b, sh) for b in [2, 4, 8, 32, 256]
                                        for sh in [(1, 4, 8, 8), (2, 3, 16, 32), (1, 1, 4, 1024)] if sh[-1] % b == 0])
def test_quantize_pack_tensor(beta, shape):
    """Flat tensor packing: bit e of the tensor is bit (e mod 32) of word (e div 32); segment j covers
    elements [j beta, (j + 1) beta) -- for W a multiple of beta these are Eq. 3's width segments."""
    x = synth.normal(7 + beta, shape)
    x.reshape(-1)[:3] = [0.0, -0.0, -1e-30]
    bits, scales = hbmm.quantize_pack_tensor(dev(x), beta)
    flat = x.reshape(1, -1)
    np.testing.assert_array_equal(words(bits), oracle.sign_pack(flat, ldw=flat.shape[1] // 32).reshape(-1))
    ref = oracle.block_scales(x.reshape(-1, shape[-1]), beta).reshape(-1)
    np.testing.assert_allclose(scales.cpu().numpy(), ref, rtol=scale_tol(beta), atol=0)


CONV_CASES = [
    # B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w
    (2, 32, 8, 8, 40, 3, 3, 1, 1, 4, 32),       # one position tile, ragged filters
    (3, 32, 6, 8, 72, 3, 3, 1, 1, 2, 16),       # ragged positions (144), beta_w = 16
    (2, 32, 9, 16, 24, 3, 3, 2, 1, 8, 32),      # stride 2, odd height
    (1, 64, 12, 12, 300, 1, 1, 1, 0, 4, 64),    # 1x1 kernel, two filter tiles
    (2, 64, 10, 12, 16, 1, 1, 2, 0, 2, 32),     # 1x1, stride 2
    (1, 32, 10, 16, 33, 5, 3, 1, 2, 16, 32),    # tall window, padding larger than the kernel's half width
    (2, 32, 7, 8, 8, 2, 2, 2, 0, 8, 128),       # even window without padding
    (1, 128, 14, 16, 130, 3, 3, 1, 1, 4, 128),  # K = 1152, 9 segments of 128
    (5, 32, 12, 12, 20, 3, 3, 1, 1, 4, 32),     # several tiles of positions that cross images
    (1, 32, 12, 44, 20, 3, 3, 2, 1, 4, 32),     # stride 2 on a wide input: 506 patch elements, 4 staging items per thread
    (1, 32, 9, 60, 12, 3, 3, 2, 1, 4, 32),      # 558 patch elements: 6 staging items per thread
    (2, 32, 8, 8, 9, 2, 3, 1, 1, 8, 32),        # 2 x 3 window: up to 6 channels enter per stage
    (1, 32, 6, 132, 10, 3, 3, 1, 1, 4, 32),     # output rows wider than a position tile: per-tap gather kernel
    (2, 32, 8, 8, 40, 3, 3, 1, 1, 4, 4),        # the paper's HadaNet setting beta_a = beta_w = 4: filters rebuilt as values too
    (1, 64, 12, 12, 150, 3, 3, 1, 1, 2, 8),     # beta_w = 8, two filter tiles of 128
    (3, 32, 6, 8, 72, 3, 3, 2, 1, 8, 2),        # beta_w = 2, stride 2
    (1, 32, 10, 16, 33, 1, 1, 1, 0, 16, 4),     # 1x1 window, beta_w = 4
]


@pytest.mark.parametrize("algo", [0, 1])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d(case, algo):
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(31 + B + C + N, B, C, H, W, N, KH, KW)
    A[0, 0, 0, :2] = [0.0, -0.0]
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    ab, asc = hbmm.quantize_pack_tensor(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    out = hbmm.conv2d(ab, asc, beta_a, A.shape, wb, ws, beta_w, (KH, KW), stride, pad, algo=algo)
    assert tuple(out.shape) == ref.shape
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d {case} algo {algo}")
    # no atomics, no order that depends on timing: a second call gives the same bits
    assert torch.equal(out, hbmm.conv2d(ab, asc, beta_a, A.shape, wb, ws, beta_w, (KH, KW), stride, pad, algo=algo))


def _random_conv_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        C = int(rng.choice([32, 64, 96]))
        KH, KW = (int(v) for v in rng.choice([1, 2, 3], size=2))
        beta_w = int(rng.choice([2, 4, 8, 16, 32, 64, 128]))
        if (C * KH * KW) % beta_w:
            continue
        beta_a = int(rng.choice([2, 4, 8]))
        W = beta_a * int(rng.integers(1, 7)) * (2 if beta_a == 2 else 1)      # a multiple of beta_a and of 4
        H = int(rng.integers(3, 13))
        stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
        if H + 2 * pad < KH or W + 2 * pad < KW:
            continue
        cases.append((int(rng.integers(1, 4)), C, H, W, int(rng.integers(1, 90)), KH, KW, stride, pad, beta_a, beta_w))
    return cases


@pytest.mark.parametrize("case", _random_conv_cases(28, 20260102), ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d_seeded_random_sweep(case):
    """Layer geometries drawn from a fixed seed; the library picks the kernel."""
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(700 + H + W + N, B, C, H, W, N, KH, KW)
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    ab, asc = hbmm.quantize_pack_tensor(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    out = hbmm.conv2d(ab, asc, beta_a, A.shape, wb, ws, beta_w, (KH, KW), stride, pad)
    assert tuple(out.shape) == ref.shape
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d sweep {case}")


# ------------------------------------------------------------------ convolution with prepared filters
def _decode_filter_pieces(pieces: np.ndarray, N, C, KH, KW) -> np.ndarray:
    """The prepared form back to numbers: for each block of 32 filters, channel group of 32, tap, step of
    16 channels and piece, 64 lanes x 8 bf16 (lane l: filter l mod 32, channels 8 (l div 32) .. + 7).
    Returns hi + mid + lo as float64, shape (N rounded up to 32, C rounded up to 32, KH, KW)."""
    nb, G, KK = -(-N // 32), -(-C // 32), KH * KW
    raw = pieces.view(np.uint16).reshape(nb, G, KK, 2, 3, 64, 8)
    val = (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64).sum(axis=4)   # nb, G, KK, ks, lane, 8
    val = val.reshape(nb, G, KK, 2, 2, 32, 8)                    # lane = half * 32 + filter
    out = val.transpose(0, 5, 1, 3, 4, 6, 2)                     # nb, filter, G, ks, half, i, tap
    return out.reshape(nb * 32, G * 32, KH, KW)


@pytest.mark.parametrize("N,C,KH,KW,beta_w", [(40, 32, 3, 3, 32), (130, 64, 1, 1, 64), (7, 20, 3, 3, 4), (33, 48, 2, 3, 7),
                                              (64, 96, 3, 3, 1), (5, 3, 5, 5, 25), (96, 128, 3, 3, 128)])
def test_conv_prepare_filters_is_exact(N, C, KH, KW, beta_w):
    """The three pieces of every weight add up to delta_w * Sign(w) exactly (Eq. 1-2 on the flattened filter),
    each piece is a bf16 number, and the padding (filters past N, channels past C) is zero."""
    Wf = synth.normal(8100 + N + C, (N, C, KH, KW)).astype(np.float32)
    K = C * KH * KW
    if beta_w == 1:
        pieces = hbmm.conv_prepare_filters(None, dev(Wf.reshape(N, K)), 1, C, (KH, KW))
        want = Wf.astype(np.float64)
    else:
        # (words and scales from the oracle, so that the values are the oracle's bit for bit)
        flat = Wf.reshape(N, K)
        wb, ws = dev(oracle.sign_pack(flat).view(np.int32)), dev(oracle.block_scales(flat, beta_w))
        pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW))
        want = oracle.materialize_filters(Wf, beta_w)
    assert pieces.numel() == hbmm.conv_filter_pieces_bytes(N, C, KH, KW) == -(-N // 32) * 32 * -(-C // 32) * 32 * KH * KW * 6
    got = _decode_filter_pieces(pieces.cpu().numpy(), N, C, KH, KW)
    assert np.array_equal(got[:N, :C], want)
    assert not got[N:].any() and not got[:, C:].any()


def _decode_filter_pieces_f16(pieces: np.ndarray, N, C, KH, KW):
    """The two-piece form back to numbers: per block of 32 filters, channel group, tap, step and piece, 64 lanes x
    8 fp16, then one int32 exponent per filter.  Returns (hi + mid scaled back by the filter's power of two, as
    float64, shape (N rounded up to 32, C rounded up to 32, KH, KW); the pieces themselves; the exponents)."""
    nb, G, KK = -(-N // 32), -(-C // 32), KH * KW
    body = nb * G * KK * 2 * 2 * 64 * 16
    raw = pieces[:body].view(np.float16).reshape(nb, G, KK, 2, 2, 64, 8).astype(np.float64)
    exps = pieces[body:].view(np.int32)
    assert exps.size == nb * 32
    val = raw.sum(axis=4).reshape(nb, G, KK, 2, 2, 32, 8)        # lane = half * 32 + filter
    out = val.transpose(0, 5, 1, 3, 4, 6, 2).reshape(nb * 32, G * 32, KH, KW)
    return out * np.ldexp(1.0, exps - 141)[:, None, None, None], raw, exps


@pytest.mark.parametrize("N,C,KH,KW,beta_w", [(40, 32, 3, 3, 32), (130, 64, 1, 1, 64), (7, 20, 3, 3, 4), (33, 48, 2, 3, 7),
                                              (64, 96, 3, 3, 1), (5, 3, 5, 5, 25)])
def test_conv_prepare_filters_two_fp16_pieces(N, C, KH, KW, beta_w):
    """The two-piece form: every filter scaled by the power of two that brings its largest magnitude into
    [2^14, 2^15), the scaled value rounded to fp16 and the remainder rounded to fp16 again: 22 significant
    bits, i.e. within 2^-22 of delta_w * Sign(w) (Eq. 1-2), or within half of fp16's smallest subnormal of the
    scaled value."""
    Wf = synth.normal(8100 + N + C, (N, C, KH, KW)).astype(np.float32)
    Wf[0] *= np.float32(2.0 ** -60)
    Wf[N - 1] *= np.float32(2.0 ** 70)
    Wf[N // 2, 0] *= np.float32(2.0 ** -30)      # a channel far below the filter's largest: subnormal remainders
    K = C * KH * KW
    if beta_w == 1:
        pieces = hbmm.conv_prepare_filters(None, dev(Wf.reshape(N, K)), 1, C, (KH, KW), form=hbmm.PIECES_F16X2)
        want = Wf.astype(np.float64)
    else:
        flat = Wf.reshape(N, K)
        wb, ws = dev(oracle.sign_pack(flat).view(np.int32)), dev(oracle.block_scales(flat, beta_w))
        pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=hbmm.PIECES_F16X2)
        want = oracle.materialize_filters(Wf, beta_w)
    nb = -(-N // 32)
    assert pieces.numel() == hbmm.conv_filter_pieces_bytes(N, C, KH, KW, hbmm.PIECES_F16X2) \
        == nb * 32 * -(-C // 32) * 32 * KH * KW * 4 + nb * 32 * 4
    got, raw, exps = _decode_filter_pieces_f16(pieces.cpu().numpy(), N, C, KH, KW)
    top = np.abs(want).reshape(N, -1).max(axis=1)
    assert np.array_equal(exps[:N], np.frexp(top)[1] - 1 + 127)           # the biased exponent of the largest magnitude
    assert np.all(np.isfinite(raw)) and np.abs(raw).max() < 2.0 ** 15
    unit = np.ldexp(1.0, exps[:N] - 141)[:, None, None, None]              # one scaled unit in the filter's own units
    err = np.abs(got[:N, :C] - want)
    assert np.all(err <= np.maximum(2.0 ** -22 * np.abs(want), 2.0 ** -25 * unit))
    assert not got[N:].any() and not got[:, C:].any()


@pytest.mark.parametrize("beta_a", [1, 4])
def test_conv2d_two_piece_form_follows_the_largest_magnitude(beta_a):
    """The two-piece form scales the activations by the exponent of the largest magnitude staged so far.  Channel
    groups that differ by many orders of magnitude in both directions (the exponent rises in a later group: the
    partial sums are rescaled; it falls: the later group is written on the coarser grid), whole tensors near
    the ends of the fp32 range, and an image that is all zeros."""
    B, C, H, W, N, KH, KW = 3, 128, 10, 12, 40, 3, 3
    A, Wf = _conv_inputs(8700 + beta_a, B, C, H, W, N, KH, KW)
    A[0, 32:64] *= 2.0 ** 20      # image 0: the second group is far larger than the first
    A[0, 96:] *= 2.0 ** -20       #          and the last far smaller
    A[1] *= 2.0 ** -100           # image 1: tiny throughout ...
    Wf[:N // 2] *= 2.0 ** 80      #          ... against large filters
    A[2] = 0.0
    A, Wf = A.astype(np.float32), Wf.astype(np.float32)
    for beta_w in (4, 32):
        ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, 1, 1, want_T=True)
        ab, asc = (None, dev(A)) if beta_a == 1 else hbmm.quantize_pack_activations(dev(A), beta_a)
        wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
        for form in (hbmm.PIECES_BF16X3, hbmm.PIECES_F16X2):
            pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
            out = hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), 1, 1, form=form).cpu().numpy()
            assert np.all(np.isfinite(out)) and not out[2].any()
            assert_close_to_oracle(out, ref, T, f"dynamic range beta_a {beta_a} beta_w {beta_w} form {form}")


PREPARED_CONV_CASES = CONV_CASES + [
    # B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w
    (2, 20, 8, 8, 40, 3, 3, 1, 1, 4, 5),        # channels not a multiple of 32, K = 180 not a multiple of 32, beta_w = 5
    (1, 48, 8, 12, 70, 3, 3, 1, 1, 2, 7),       # one and a half channel groups; the last filter segment is shorter
    (3, 64, 28, 28, 64, 3, 3, 1, 1, 4, 64),     # 4 output rows per tile, 7 tiles per image, two staging items per thread
    (2, 32, 14, 14, 96, 3, 3, 1, 1, 2, 128),    # 9 rows per tile (126 positions), second tile of 5 rows
    (1, 3, 16, 16, 16, 5, 5, 1, 2, 4, 25),      # a first-layer shape: 3 channels, 5 x 5 window
    (2, 64, 56, 56, 64, 3, 3, 2, 1, 8, 64),     # stride 2: the patch of four output rows is 9 x 57 = 513 pixels, five staging items
    (1, 32, 56, 56, 96, 3, 3, 2, 1, 8, 32),     # the same patch with a 128-filter tile
    (1, 32, 8, 120, 8, 3, 3, 1, 1, 8, 32),      # one output row of 120 positions: 366 pixels, three staging items
    (1, 160, 6, 8, 200, 1, 1, 1, 0, 4, 160),    # five channel groups, two filter tiles of 128 (the second ragged)
]


@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
@pytest.mark.parametrize("case", PREPARED_CONV_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d_prepared(case, form):
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(8200 + B + C + N, B, C, H, W, N, KH, KW)
    A[0, 0, 0, :2] = [0.0, -0.0]
    ab, asc = hbmm.quantize_pack_tensor(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
    OW = (W + 2 * pad - KW) // stride + 1
    if OW > 128 or ((OW - 1) * stride + KW) * KH > 640:
        with pytest.raises(hbmm.HbmmError) as ei:
            hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
        assert ei.value.code == hbmm.EUNSUPPORTED
        return
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    out = hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
    assert tuple(out.shape) == ref.shape
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d_prepared {case} form {form}")
    # a fixed summation order: a second call gives the same bits
    assert torch.equal(out, hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form))


@pytest.mark.parametrize("case", [(2, 32, 8, 8, 40, 3, 3, 1, 1, 32), (1, 64, 12, 12, 70, 1, 1, 1, 0, 64),
                                  (2, 32, 9, 16, 24, 3, 3, 2, 1, 4), (1, 64, 12, 12, 140, 3, 3, 1, 1, 8),
                                  (2, 24, 10, 10, 30, 3, 3, 1, 1, 1)], ids=str)
@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
def test_conv2d_prepared_unquantised_operands(case, form):
    """beta_a = 1: activations stay fp32 (the paper's binary-weight layers, Tables 2-3); the last case also
    leaves the filters unquantised (beta_w = 1), i.e. a plain fp32 convolution through the same kernel."""
    B, C, H, W, N, KH, KW, stride, pad, beta_w = case
    A = synth.normal(8300 + C + N, (B, C, H, W))
    A[0, 0, 0, :3] = [0.0, -0.0, 1e-30]
    Wf = synth.normal(8301 + C, (N, C, KH, KW)).astype(np.float32)
    ref, T = oracle.hbmm_conv2d(A, Wf, 1, beta_w, stride, pad, want_T=True)
    if beta_w == 1:
        pieces = hbmm.conv_prepare_filters(None, dev(Wf.reshape(N, -1)), 1, C, (KH, KW), form=form)
    else:
        wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
        pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
    out = hbmm.conv2d_prepared(None, dev(A), 1, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d_prepared unquantised {case} form {form}")


@pytest.mark.parametrize("shape,beta", [((2, 3, 7, 7), 4), ((2, 3, 7, 7), 2), ((1, 5, 14, 14), 4), ((3, 2, 5, 9), 3), ((1, 1, 1, 1), 2),
                                        ((2, 4, 8, 8), 4), ((1, 16, 8, 28), 7), ((2, 3, 4, 130), 128), ((1, 2, 3, 300), 256)])
def test_quantize_pack_activations(shape, beta):
    """Segments along the width, anew in every row, for any segment length: flat sign bits, and scales that
    are the oracle's bit for bit where the general kernel runs (double-precision sums rounded once)."""
    x = synth.normal(8500 + sum(shape) + beta, shape)
    x.reshape(-1)[:3] = [0.0, -0.0, -1e-30][:min(3, x.size)]
    bits, scales = hbmm.quantize_pack_activations(dev(x), beta)
    count, W = x.size, shape[-1]
    flat = oracle.sign_pack(x.reshape(1, -1))[0, :(count + 31) // 32]
    assert np.array_equal(words(bits), flat)
    ref = oracle.block_scales(x.reshape(-1, W), beta).reshape(-1)
    got = scales.cpu().numpy()
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= scale_tol(beta) * ref)
    if W % beta:
        assert np.array_equal(got, ref)


RAGGED_WIDTH_CONV_CASES = [
    # B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w
    (2, 32, 7, 7, 40, 3, 3, 1, 1, 4, 4),        # 7 x 7 maps (the last stage of a ResNet) with the paper's beta = 4: segments 4 + 3
    (3, 48, 7, 7, 70, 3, 3, 1, 1, 2, 8),        # 2 + 2 + 2 + 1
    (1, 64, 7, 7, 130, 1, 1, 1, 0, 7, 64),      # one segment per row
    (2, 20, 14, 14, 33, 3, 3, 2, 1, 4, 5),      # 4 + 4 + 4 + 2, stride 2
    (1, 32, 9, 10, 16, 3, 3, 1, 1, 3, 32),      # 3 + 3 + 3 + 1
    (2, 16, 5, 13, 12, 2, 3, 1, 1, 16, 6),      # beta_a longer than the width: one short segment per row
    (5, 32, 7, 7, 40, 3, 3, 1, 1, 4, 4),        # two whole images per tile, the last tile with one
    (7, 32, 4, 4, 20, 3, 3, 1, 1, 2, 32),       # 16 positions per image: eight images per tile would fit, seven exist
    (9, 32, 6, 6, 70, 3, 3, 2, 1, 4, 16),       # 3 x 3 outputs per image, stride 2: fourteen images per tile would fit
    (3, 64, 8, 8, 16, 1, 1, 1, 0, 8, 64),       # 64 positions per image: two images per tile, 1 x 1 window
]


@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
@pytest.mark.parametrize("case", RAGGED_WIDTH_CONV_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d_prepared_width_not_a_multiple_of_beta_a(case, form):
    """Eq. 3 on widths that beta_a does not divide: hbmm_quantize_pack_activations + hbmm_conv2d_prepared against
    the oracle's layer."""
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(8600 + B + C + N, B, C, H, W, N, KH, KW)
    ab, asc = hbmm.quantize_pack_activations(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    out = hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
    assert tuple(out.shape) == ref.shape
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d_prepared ragged width {case} form {form}")


MANY_TILE_CONV_CASES = [
    # B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w: 3 x 3 layers with more tiles than the chip has compute units
    (40, 32, 56, 56, 64, 3, 3, 1, 1, 4, 32),     # 560 tiles of 64 filters, one channel group
    (9, 40, 56, 56, 130, 3, 3, 1, 1, 8, 5),      # 126 position tiles x 3 filter tiles; the second channel group partial
    (3, 64, 112, 112, 128, 3, 3, 1, 1, 4, 64),   # one output row per tile, three pixels per lane, 128-filter tiles
    (41, 96, 28, 28, 64, 3, 3, 1, 1, 1, 4),      # unquantised activations, three channel groups, 287 tiles
]


@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
@pytest.mark.parametrize("case", MANY_TILE_CONV_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d_prepared_many_tiles(case, form):
    """Layers of several hundred tiles (several rounds of workgroups, all XCD slots in use), with the images scaled
    differently and one half image of zeros, so that neighbouring tiles of the two-piece form work in different
    units."""
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(8800 + B + C + N, B, C, H, W, N, KH, KW)
    A *= (2.0 ** (np.arange(B) % 5 * 3 - 6)).astype(np.float32)[:, None, None, None]
    if B > 2:
        A[2, :, : H // 2] = 0.0          # tiles that are all zeros between ordinary ones
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    ab, asc = (None, dev(A)) if beta_a == 1 else hbmm.quantize_pack_activations(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
    out = hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d_prepared many tiles {case} form {form}")
    assert torch.equal(out, hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form))


def _random_prepared_conv_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        C = int(rng.integers(1, 100))
        KH, KW = (int(v) for v in rng.integers(1, 4, size=2))
        beta_w = int(rng.integers(1, 65))
        beta_a = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
        W = int(rng.integers(3, 60))
        H = int(rng.integers(3, 20))
        stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
        B = int(rng.integers(1, 4))
        if H + 2 * pad < KH or W + 2 * pad < KW:
            continue
        cases.append((B, C, H, W, int(rng.integers(1, 150)), KH, KW, stride, pad, beta_a, beta_w))
    return cases


@pytest.mark.parametrize("form", [0, 1], ids=["bf16x3", "f16x2"])
@pytest.mark.parametrize("case", _random_prepared_conv_cases(32, 20260105), ids=lambda c: "x".join(str(v) for v in c))
def test_conv2d_prepared_seeded_random_sweep(case, form):
    """Layer geometries, channel counts, widths and segment lengths (any beta_w in 1..64, beta_a from 1 to 16,
    dividing the width or not) drawn from a fixed seed."""
    B, C, H, W, N, KH, KW, stride, pad, beta_a, beta_w = case
    A, Wf = _conv_inputs(8400 + H + W + N, B, C, H, W, N, KH, KW)
    ref, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    ab, asc = (None, dev(A)) if beta_a == 1 else hbmm.quantize_pack_activations(dev(A), beta_a)
    if beta_w == 1:
        pieces = hbmm.conv_prepare_filters(None, dev(Wf.reshape(N, -1)), 1, C, (KH, KW), form=form)
    else:
        wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
        pieces = hbmm.conv_prepare_filters(wb, ws, beta_w, C, (KH, KW), form=form)
    out = hbmm.conv2d_prepared(ab, asc, beta_a, A.shape, pieces, N, (KH, KW), stride, pad, form=form)
    assert tuple(out.shape) == ref.shape
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d_prepared sweep {case} form {form}")


def test_conv2d_equals_gemm_on_im2col():
    """For a 1x1 window with stride 1 the convolution is the matrix product of the positions x channels
    matrix of materialised activations with the filters: the same kernel family must agree with
    hbmm_gemm's unquantised-activation path on that matrix (each within 1e-5 T of the exact value), a check that does not go
    through the oracle's convolution loops."""
    B, C, H, W, N, beta_a, beta_w = 2, 64, 8, 8, 48, 4, 32
    A, Wf = _conv_inputs(77, B, C, H, W, N, 1, 1)
    ab, asc = hbmm.quantize_pack_tensor(dev(A), beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    out = hbmm.conv2d(ab, asc, beta_a, A.shape, wb, ws, beta_w, (1, 1), 1, 0)
    At = oracle.materialize_activations(A, beta_a).astype(np.float32)          # exact: +-fp32 scale
    X = np.ascontiguousarray(At.transpose(0, 2, 3, 1).reshape(B * H * W, C))
    via_gemm = hbmm.gemm(None, dev(X), 1, wb, ws, beta_w, C)
    got = out.permute(0, 2, 3, 1).reshape(B * H * W, N).cpu().numpy().astype(np.float64)
    T = np.abs(X.astype(np.float64)) @ np.abs(oracle.materialize_filters(Wf, beta_w).reshape(N, C)).T
    assert np.all(np.abs(got - via_gemm.cpu().numpy()) <= 2e-5 * T)


def test_conv2d_unsupported():
    A, Wf = _conv_inputs(5, 1, 32, 8, 8, 8, 3, 3)
    ab, asc = hbmm.quantize_pack_tensor(dev(A), 4)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(8, -1)), 32)
    with pytest.raises(hbmm.HbmmError):
        hbmm.conv2d(ab, asc, 16, A.shape, wb, ws, 32, (3, 3), 1, 1)     # beta_a does not divide W
    with pytest.raises(hbmm.HbmmError):
        hbmm.quantize_pack_tensor(dev(synth.normal(1, (3, 5, 8))), 4)   # 120 elements: not a multiple of 128


@pytest.mark.parametrize("algo", [0, 1])
@pytest.mark.parametrize("case", [(2, 32, 8, 8, 40, 3, 3, 1, 1, 32), (1, 64, 12, 12, 70, 1, 1, 1, 0, 64),
                                  (2, 32, 9, 16, 24, 3, 3, 2, 1, 32), (2, 32, 8, 8, 40, 3, 3, 1, 1, 4),
                                  (1, 64, 12, 12, 140, 3, 3, 1, 1, 8)], ids=str)
def test_conv2d_unquantised_activations(case, algo):
    """beta_a = 1 (binary-weight layer): activations stay fp32, filters are binarised -- with
    beta_w = 4 and 8 this is a layer of the paper's binary-weight networks (Tables 2-3)."""
    B, C, H, W, N, KH, KW, stride, pad, beta_w = case
    A = synth.normal(91 + C + N, (B, C, H, W))
    A[0, 0, 0, :3] = [0.0, -0.0, 1e-30]
    Wf = synth.normal(92 + C, (N, C, KH, KW)).astype(np.float32)
    ref, T = oracle.hbmm_conv2d(A, Wf, 1, beta_w, stride, pad, want_T=True)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(N, -1)), beta_w)
    out = hbmm.conv2d(None, dev(A), 1, A.shape, wb, ws, beta_w, (KH, KW), stride, pad, algo=algo)
    assert_close_to_oracle(out.cpu().numpy(), ref, T, f"conv2d beta_a=1 {case} algo {algo}")


@pytest.mark.parametrize("beta", [2, 8, 16])
def test_binarize_backward_tensor(beta):
    """Gradient through Eq. 3-4 for an activation tensor (segments along the width)."""
    shape = (2, 3, 8, 32)
    x, g = synth.normal(95, shape, std=0.8), synth.normal(96, shape)
    ref, T = oracle.binarize_backward(x.reshape(-1, shape[-1]), g.reshape(-1, shape[-1]), beta, want_T=True)
    got = hbmm.binarize_backward_tensor(dev(x), dev(g), beta).cpu().numpy().reshape(-1, shape[-1])
    err = np.abs(got.astype(np.float64) - ref)
    assert np.all(err <= (np.log2(beta) + 3) * 2.0 ** -24 * T + 1e-30)


@pytest.mark.parametrize("beta", [32, 64, 128, 256])
def test_gemm_short_k_on_a_large_grid(beta):
    """A K of at most two chunks on a grid that fills the chip takes the 256-row workgroups (except for
    32-bit segments): ragged in both dimensions, against the oracle's integer path."""
    M, N, K = 33000, 1000, 768
    A, B = synth.normal(8100 + beta, (M, K)), synth.uniform_pm1(8101 + beta, (N, K))
    run_gemm_case(A, B, beta, beta)
