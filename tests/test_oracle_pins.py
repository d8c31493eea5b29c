"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself and never against the GPU path.

Each test names the mistake it is meant to catch.  Brute-force helpers below are written
per element in pure Python (fractions / ints) and share nothing with ``oracle/``.
"""
from __future__ import annotations

import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_1905_10759_amd import synth


# ----------------------------------------------------------------------------- helpers
def _sgn(v: float) -> int:
    return 1 if v >= 0 else -1


def brute_scales(x: np.ndarray, beta: int):
    """Exact mean |x| per segment with rationals, then one rounding to fp32."""
    rows, K = x.shape
    out = []
    for r in range(rows):
        row = []
        for k0 in range(0, K, beta):
            seg = [Fraction(float(abs(v))) for v in x[r, k0:k0 + beta]]
            row.append(np.float32(float(sum(seg) / len(seg))))
        out.append(row)
    return np.array(out, dtype=np.float32)


def brute_hbmm(A: np.ndarray, B: np.ndarray, beta_a: int, beta_w: int):
    """sum_k (sA * sgn a)(sB * sgn b) with exact rationals (scales are the fp32 ones)."""
    sa, sb = brute_scales(A, beta_a), brute_scales(B, beta_w)
    M, K = A.shape
    N = B.shape[0]
    C = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                av = Fraction(float(A[m, k])) if beta_a == 1 else Fraction(float(sa[m, k // beta_a])) * _sgn(A[m, k])
                bv = Fraction(float(B[n, k])) if beta_w == 1 else Fraction(float(sb[n, k // beta_w])) * _sgn(B[n, k])
                acc += av * bv
            C[m, n] = float(acc)
    return C


def unpack(bits: np.ndarray, K: int) -> np.ndarray:
    rows = bits.shape[0]
    out = np.zeros((rows, K), dtype=np.int64)
    for r in range(rows):
        for k in range(K):
            out[r, k] = (int(bits[r, k // 32]) >> (k % 32)) & 1
    return out


# ------------------------------------------------------------------------ sign + pack
def test_pack_matches_paper_example(golden_dir):
    """Catches: inverted value mapping (-1 -> 1), reversed element order inside a word."""
    txt = (golden_dir / "bitpack_example.txt").read_text().splitlines()
    signs = [int(t) for t in next(l for l in txt if l.startswith("signs:")).split(":")[1].split()]
    want = next(l for l in txt if l.startswith("bits:")).split(":")[1].strip()
    x = np.array([signs], dtype=np.float32) * 0.37
    bits = oracle.sign_pack(x)
    got = "".join(str((int(bits[0, 0]) >> k) & 1) for k in range(len(signs)))
    assert got == want
    assert int(bits[0, 0]) == 0b100110  # element k is bit k: value 38
    assert not bits[0, 1:].any()


def test_pack_roundtrip_ragged_and_pad_zero():
    """Catches: wrong word index / bit index, dirty pad bits, sign(0) != +1."""
    K = 77
    x = synth.normal(11, (9, K))
    x[0, :5] = [0.0, -0.0, 1.0, -1.0, np.float32(1e-30)]
    bits = oracle.sign_pack(x)
    assert bits.shape == (9, 4) and bits.dtype == np.uint32
    assert np.array_equal(unpack(bits, K), (x >= 0).astype(np.int64))
    assert unpack(bits, K)[0, :5].tolist() == [1, 1, 1, 0, 1]
    full = unpack(bits, 128)
    assert not full[:, K:].any()


def test_pack_non_finite_inputs_follow_the_comparison():
    """Sign is the comparison x >= 0: +inf gives 1, -inf and NaN give 0 (outside the method's
    domain, but the reading is fixed so that both sides of the parity tests agree on it)."""
    x = np.array([[np.inf, -np.inf, np.nan, -np.nan, 1.0, -1.0, 0.0, 2.0]], dtype=np.float32)
    assert unpack(oracle.sign_pack(x), 8)[0].tolist() == [1, 0, 0, 0, 1, 0, 1, 1]
    s = oracle.block_scales(x, 4)
    assert np.isnan(s[0, 0]) and s[0, 1] == np.float32(1.0)


def test_pack_word_boundaries():
    """Catches: off-by-one at bit 31/32 and between words."""
    K = 96
    for hot in (0, 31, 32, 63, 64, 95):
        x = -np.ones((1, K), dtype=np.float32)
        x[0, hot] = 2.0
        bits = oracle.sign_pack(x)
        want = np.zeros(4, dtype=np.uint32)
        want[hot // 32] = np.uint32(1) << np.uint32(hot % 32)
        assert np.array_equal(bits[0], want), hot


# ------------------------------------------------------------------------------ scales
@pytest.mark.parametrize("K,beta", [(12, 1), (12, 4), (12, 12), (13, 4), (64, 32), (70, 32)])
def test_scales_brute_force(K, beta):
    """Catches: beta+1 terms in the sum, wrong divisor on a short last segment, abs dropped."""
    x = synth.normal(21, (3, K))
    got = oracle.block_scales(x, beta)
    assert got.dtype == np.float32 and got.shape == (3, -(-K // beta))
    assert np.array_equal(got, brute_scales(x, beta))


def test_scales_special_cases():
    """beta = 1 keeps |x|; beta = K is the per-row (1/n)||W||_1 of XNOR-Net (section 3.1.2)."""
    x = synth.normal(22, (4, 48))
    assert np.array_equal(oracle.block_scales(x, 1), np.abs(x))
    l1 = np.abs(x.astype(np.float64)).sum(axis=1) / 48
    assert np.allclose(oracle.block_scales(x, 48)[:, 0], l1, rtol=1e-7, atol=0)


def test_scales_expectations():
    """Textbook first absolute moments of the three input distributions (statistical sanity)."""
    n = 1 << 18
    assert abs(oracle.block_scales(synth.normal(23, (1, n)), 64).mean() - math.sqrt(2 / math.pi)) < 5e-3
    assert abs(oracle.block_scales(synth.uniform_pm1(24, (1, n)), 64).mean() - 0.5) < 5e-3
    assert abs(oracle.block_scales(synth.relu_normal(25, (1, n)), 64).mean() - 1 / math.sqrt(2 * math.pi)) < 5e-3


def test_compression_ratio_formula(golden_dir):
    """Packed bits + fp32 scales are beta*X/(beta+X) times smaller than fp32 (X = 32)."""
    X = 32
    rows, K = 8, 1024
    x = synth.normal(26, (rows, K))
    for beta, printed in ((16, 10.67), (64, 21.33), (128, 25.6), (256, 28.44)):
        nbytes = rows * K // 8 + oracle.block_scales(x, beta).nbytes
        assert oracle.sign_pack(x, ldw=K // 32).nbytes == rows * K // 8
        ratio = x.nbytes / nbytes
        assert ratio == pytest.approx(beta * X / (beta + X), rel=1e-12)
        assert ratio == pytest.approx(printed, abs=0.01)


# ----------------------------------------------------------- Hadamard binarisation whole
def test_materialize_brute_force():
    """Catches: scale of the wrong segment, sign flipped, beta = 1 not the identity."""
    x = synth.normal(31, (3, 14))
    x[1, 3] = 0.0
    for beta in (1, 2, 4, 7, 14, 5):
        s = brute_scales(x, beta)
        want = np.array([[float(x[r, k]) if beta == 1 else float(s[r, k // beta]) * _sgn(x[r, k])
                          for k in range(14)] for r in range(3)])
        assert np.array_equal(oracle.materialize(x, beta), want), beta


@pytest.mark.parametrize("beta", [1, 2, 8, 64, 1024])
def test_angle_closed_form(beta, golden_dir):
    """For i.i.d. N(0,1) entries cos^2(angle) -> 2/pi + (1 - 2/pi)/beta (follows from Eq. 2:
    <x, x~> = |x~|^2 = sum_j beta s_j^2 and E s^2 = Var|x|/beta + (E|x|)^2); large beta gives
    arccos sqrt(2/pi) = 37.07 deg, the saturation value the paper prints (section 3.2)."""
    n = 1 << 20
    x = synth.normal(32, (1, n))
    xt = oracle.materialize(x, beta)[0]
    xd = x[0].astype(np.float64)
    cosang = xd @ xt / (np.linalg.norm(xd) * np.linalg.norm(xt))
    ang = math.degrees(math.acos(min(1.0, cosang)))
    want = math.degrees(math.acos(math.sqrt(2 / math.pi + (1 - 2 / math.pi) / beta)))
    assert abs(ang - want) < 0.2
    if beta == 1:
        assert ang < 1e-3
    if beta >= 64:
        printed = float(next(l for l in (golden_dir / "paper_constants.txt").read_text().splitlines()
                             if l.startswith("angle_saturation_deg")).split(":")[1])
        assert abs(ang - printed) < 0.5


# ------------------------------------------------------------------------- integer dot
def test_int_dot_brute_force_and_identities():
    """Catches: popcount of xnor over pad bits, dot = popcount instead of n - 2*hamming."""
    K = 45
    A, B = synth.normal(41, (6, K)), synth.normal(42, (5, K))
    a, b = oracle.sign_pack(A), oracle.sign_pack(B)
    D = oracle.int_dot(a, b, K)
    want = np.array([[sum(_sgn(A[m, k]) * _sgn(B[n, k]) for k in range(K)) for n in range(5)] for m in range(6)])
    assert D.dtype == np.int32 and np.array_equal(D, want)
    # xnor identity on the K valid bits: dot = 2 * matches - K
    ua, ub = unpack(a, K), unpack(b, K)
    matches = (ua[:, None, :] == ub[None, :, :]).sum(-1)
    assert np.array_equal(D, 2 * matches - K)
    S = oracle.int_dot(a, a, K)
    assert np.array_equal(np.diag(S), np.full(6, K)) and np.array_equal(S, S.T)
    assert np.array_equal(oracle.int_dot(a, oracle.sign_pack(-np.abs(A) * np.sign(A + 1e-30)), K).diagonal(), np.full(6, -K))


# -------------------------------------------------------------------------- full HBMM
@pytest.mark.parametrize("beta_a,beta_w", [(1, 1), (2, 2), (4, 4), (4, 2), (2, 8), (16, 16), (3, 5), (1, 4), (16, 1)])
def test_hbmm_brute_force(beta_a, beta_w):
    """Both oracle paths against exact rational arithmetic on a tiny ragged problem."""
    A, B = synth.normal(51, (3, 19)), synth.normal(52, (4, 19))
    want = brute_hbmm(A, B, beta_a, beta_w)
    dense = oracle.hbmm_dense(A, B, beta_a, beta_w)
    assert np.allclose(dense, want, rtol=0, atol=1e-13)
    pop = oracle.hbmm_popcount(A, B, beta_a, beta_w)
    assert np.allclose(pop, want, rtol=0, atol=1e-13)


def test_hbmm_all_sign_patterns_one_block():
    """Every sign pattern of one beta = 4 segment: contribution = sA*sB*(4 - 2*hamming).
    Catches the literal reading of Eq. 7 (count of agreeing bits instead of 2p - n)."""
    mags = np.array([0.5, 1.5, 0.25, 2.0], dtype=np.float32)
    b = (mags * np.array([1, -1, 1, 1], dtype=np.float32))[None, :]
    sb = float(np.float32(np.abs(b).mean()))
    for pattern in itertools.product((1, -1), repeat=4):
        a = (mags[::-1] * np.array(pattern, dtype=np.float32))[None, :]
        sa = float(np.float32(np.abs(a).mean()))
        ham = sum(1 for p, q in zip(pattern, (1, -1, 1, 1)) if p != q)
        want = sa * sb * (4 - 2 * ham)
        assert oracle.hbmm_popcount(a, b, 4, 4)[0, 0] == pytest.approx(want, abs=1e-14)
        assert oracle.hbmm_dense(a, b, 4, 4)[0, 0] == pytest.approx(want, abs=1e-14)
        literal = sa * sb * (4 - ham)  # Eq. 7 as printed: popcount(xnor) = agreeing bits
        if ham != 0:
            assert abs(oracle.hbmm_dense(a, b, 4, 4)[0, 0] - literal) > 1e-3


def test_beta_one_is_plain_matmul():
    """beta_a = beta_w = 1 is the unquantised product (library matmul in double)."""
    A, B = synth.normal(53, (17, 96)), synth.normal(54, (13, 96))
    want = A.astype(np.float64) @ B.astype(np.float64).T
    assert np.allclose(oracle.hbmm_dense(A, B, 1, 1), want, rtol=0, atol=1e-12)


def test_whole_row_blocks_reduce_to_xnor_net():
    """beta = K for both operands: C = sA[m] * sB[n] * D[m, n], XNOR-Net's per-row scaling
    (section 5: beta = nElement is essentially the XNOR-Net)."""
    K = 160
    A, B = synth.normal(55, (9, K)), synth.normal(56, (7, K))
    D = oracle.int_dot(oracle.sign_pack(A), oracle.sign_pack(B), K).astype(np.float64)
    sa = np.abs(A.astype(np.float64)).mean(1).astype(np.float32).astype(np.float64)
    sb = np.abs(B.astype(np.float64)).mean(1).astype(np.float32).astype(np.float64)
    want = sa[:, None] * sb[None, :] * D
    assert np.allclose(oracle.hbmm_popcount(A, B, K, K), want, rtol=1e-14, atol=0)
    assert np.allclose(oracle.hbmm_dense(A, B, K, K), want, rtol=1e-12, atol=1e-12)


def test_binary_weight_form():
    """beta_a = 1 (HBWN): C = A . (delta (.) Sign(B))^T with A untouched; the segmented
    add/subtract form, the dense path and a library matmul agree."""
    K = 96
    B = synth.normal(58, (6, K))
    # rectified activations (the benchmark's kind) and signed ones (a lost sign of A shows only there)
    for A in (synth.relu_normal(57, (11, K)), synth.normal(157, (11, K))):
        for beta_w in (4, 32, 96, 40):
            sb = oracle.block_scales(B, beta_w)
            Bt = oracle.materialize(B, beta_w, sb)
            want = A.astype(np.float64) @ Bt.T
            got, T = oracle.binary_weight_gemm(A, oracle.sign_pack(B), sb, beta_w, want_T=True)
            assert np.allclose(got, want, rtol=0, atol=1e-12)
            assert np.allclose(oracle.hbmm_dense(A, B, 1, beta_w), want, rtol=0, atol=1e-12)
            assert np.allclose(T, np.abs(A.astype(np.float64)) @ np.abs(Bt).T, rtol=1e-12)


def test_paths_agree_and_T_bounds():
    """Integer path == dense path on a multi-block problem; T = sum |terms| >= |C|."""
    A, B = synth.normal(59, (33, 320)), synth.uniform_pm1(60, (21, 320))
    for ba, bw in ((32, 32), (64, 32), (32, 160), (320, 64)):
        dense = oracle.hbmm_dense(A, B, ba, bw)
        pop, T = oracle.hbmm_popcount(A, B, ba, bw, want_T=True)
        assert np.abs(dense - pop).max() <= 1e-12 * np.abs(dense).max()
        assert (T >= np.abs(pop) - 1e-12).all()


def test_error_scale_T_of_the_product_is_the_sum_of_absolute_terms():
    """T, the scale every fp32 parity bar is taken relative to, recomputed with exact rationals for
    equal, mixed and ragged segment lengths: T[m, n] = sum over the pieces between consecutive
    segment ends of either operand of |sA * sB * d| (Eq. 7's terms).  An inflated T would loosen
    every GPU tolerance without any other test noticing."""
    A, B = synth.normal(63, (3, 19)), synth.uniform_pm1(64, (2, 19))
    for ba, bw in ((4, 4), (2, 8), (8, 2), (3, 5), (19, 4), (6, 19)):
        sa, sb = oracle.block_scales(A, ba), oracle.block_scales(B, bw)
        _, T = oracle.popcount_gemm(oracle.sign_pack(A), sa, ba, oracle.sign_pack(B), sb, bw, 19, want_T=True)
        cuts = sorted(set(range(0, 19, ba)) | set(range(0, 19, bw)) | {19})
        for m in range(3):
            for n in range(2):
                want = Fraction(0)
                for k0, k1 in zip(cuts[:-1], cuts[1:]):
                    d = sum(int(_sgn(A[m, k]) * _sgn(B[n, k])) for k in range(k0, k1))
                    want += abs(Fraction(float(sa[m, k0 // ba])) * Fraction(float(sb[n, k0 // bw])) * d)
                assert T[m, n] == pytest.approx(float(want), rel=1e-13), (ba, bw, m, n)


def test_positive_scaling_invariance():
    """Scaling an operand by c > 0 (a power of two, so exact) scales C and leaves bits alone."""
    A, B = synth.normal(61, (8, 128)), synth.normal(62, (8, 128))
    assert np.array_equal(oracle.sign_pack(A), oracle.sign_pack(4 * A))
    assert np.array_equal(oracle.hbmm_popcount(4 * A, B, 32, 64), 4 * oracle.hbmm_popcount(A, B, 32, 64))


def test_layout_one_is_transpose():
    """A K x N right-hand operand is binarised along K: identical to its N x K transpose."""
    Bkn = synth.normal(63, (64, 5))
    assert np.array_equal(oracle.as_rows_by_k(Bkn, 1), Bkn.T)
    assert np.array_equal(oracle.block_scales(oracle.as_rows_by_k(Bkn, 1), 32),
                          brute_scales(np.ascontiguousarray(Bkn.T), 32))


# ------------------------------------------------------------ backward of the binarisation
def _torch_binarize(x, beta):
    """delta (.) Sign(x) written with library autograd pieces: mean |x| per segment, and Sign with the
    straight-through derivative 1[|x| <= 1] (forward value sign, backward value of hardtanh)."""
    import torch
    rows, K = x.shape
    seg = x.reshape(rows, K // beta, beta)
    delta = seg.abs().mean(dim=2, keepdim=True)
    hard = torch.nn.functional.hardtanh(seg)
    sign = torch.where(seg >= 0, torch.ones_like(seg), -torch.ones_like(seg))
    ste = hard + (sign - hard).detach()
    return (delta * ste).reshape(rows, K)


@pytest.mark.parametrize("beta", [1, 2, 4, 8, 32])
def test_backward_matches_library_autograd(beta):
    """Eq. 6 against torch autograd of the same function in float64 (catches: missing 1/beta, the sum
    taken over the wrong segment, a dropped Sign(W_i), the STE mask on the wrong term)."""
    import torch
    x = synth.normal(71, (5, 64)) * 1.3          # some |x| > 1 so the mask matters
    g = synth.normal(72, (5, 64))
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    _torch_binarize(xt, beta).backward(torch.tensor(g, dtype=torch.float64))
    want = xt.grad.numpy()
    got = oracle.binarize_backward(x, g, beta)
    # the oracle uses the stored fp32 delta: allow that rounding (2^-24 relative on the second term)
    assert np.allclose(got, want, rtol=0, atol=2e-7 * (np.abs(g).max() * np.abs(x).max() + 1))
    assert ((np.abs(x) > 1).sum() > 10) and ((np.abs(x) <= 1).sum() > 10)


def test_backward_scale_path_is_the_true_derivative():
    """With the signs frozen, the first term of Eq. 6 is the exact derivative of sum_j g_j delta s_j:
    central differences in double."""
    beta, K = 4, 16
    z = synth.normal(73, (1, K)).astype(np.float64)
    x = np.sign(z) * (1.5 + np.abs(z))                            # |x| > 1 everywhere (the STE term vanishes), mixed signs
    g = synth.normal(74, (1, K)).astype(np.float64)
    s = np.sign(x)

    def f(xx):
        delta = np.abs(xx).reshape(-1, beta).mean(1).repeat(beta)
        return float((g[0] * delta * s[0]).sum())

    num = np.zeros(K)
    for i in range(K):
        e = np.zeros(K)
        e[i] = 1e-4
        num[i] = (f(x[0] + e) - f(x[0] - e)) / 2e-4
    got = oracle.binarize_backward(x.astype(np.float32), g.astype(np.float32), beta)[0]
    assert np.allclose(got, num, rtol=1e-5, atol=1e-6)


def test_backward_brute_force_ragged_and_mask_edges():
    """Exact rationals on a ragged row; |x| = 1 is inside the straight-through window (Eq. 5: <=)."""
    beta = 4
    x = np.array([[0.5, -1.0, 1.0, -2.5, 0.0, -0.25, 3.0, 1.5, -0.75, 2.0]], dtype=np.float32)
    g = np.array([[1.0, -2.0, 0.5, 4.0, -1.0, 0.25, 2.0, -3.0, 1.5, -0.5]], dtype=np.float32)
    got, T = oracle.binarize_backward(x, g, beta, want_T=True)
    K = x.shape[1]
    for i in range(K):
        k0 = (i // beta) * beta
        k1 = min(k0 + beta, K)
        n = k1 - k0
        delta = Fraction(float(np.float32(float(sum(Fraction(float(abs(v))) for v in x[0, k0:k1]) / n))))
        sdot = sum(Fraction(float(g[0, j])) * _sgn(x[0, j]) for j in range(k0, k1))
        want = _sgn(x[0, i]) * sdot / n + (delta * Fraction(float(g[0, i])) if abs(x[0, i]) <= 1 else 0)
        assert got[0, i] == pytest.approx(float(want), abs=1e-14), i
        # the error scale: (1/n) sum_j |g_j| + delta |g_i| [|x_i| <= 1], exactly
        want_T = sum(abs(Fraction(float(g[0, j]))) for j in range(k0, k1)) / n + (
            delta * abs(Fraction(float(g[0, i]))) if abs(x[0, i]) <= 1 else 0)
        assert T[0, i] == pytest.approx(float(want_T), rel=1e-13), i


# ----------------------------------------------------------------------------- convolution (Eq. 1-4 on tensors)
def _np_materialize_act(A: np.ndarray, beta: int) -> np.ndarray:
    """delta (.) Sign(A) with segments along the last (width) axis, in numpy, independent of oracle/."""
    B, C, H, W = A.shape
    seg = np.abs(A.astype(np.float64)).reshape(B, C, H, W // beta, beta).mean(axis=-1).astype(np.float32)
    return np.where(A >= 0, 1.0, -1.0) * np.repeat(seg.astype(np.float64), beta, axis=-1)


def _np_materialize_filt(Wf: np.ndarray, beta: int) -> np.ndarray:
    N = Wf.shape[0]
    flat = Wf.reshape(N, -1)
    seg = np.abs(flat.astype(np.float64)).reshape(N, -1, beta).mean(axis=-1).astype(np.float32)
    return (np.where(flat >= 0, 1.0, -1.0) * np.repeat(seg.astype(np.float64), beta, axis=-1)).reshape(Wf.shape)


@pytest.mark.parametrize("stride,pad,KH,KW", [(1, 1, 3, 3), (2, 1, 3, 3), (1, 0, 1, 1), (2, 0, 1, 1), (1, 2, 5, 3), (2, 0, 2, 2)])
def test_conv_matches_library_convolution(stride, pad, KH, KW):
    """Catches: swapped height/width, wrong stride/padding arithmetic, a flipped kernel (true
    convolution instead of cross-correlation), wrong output size, segments along the wrong axis."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11 * stride + pad + KH)
    B, C, H, W, N = 2, 4, 7, 8, 3
    A = rng.standard_normal((B, C, H, W)).astype(np.float32)
    Wf = rng.standard_normal((N, C, KH, KW)).astype(np.float32)
    beta_a, beta_w = 4, 2
    At, Wt = _np_materialize_act(A, beta_a), _np_materialize_filt(Wf, beta_w)
    ref = torch.nn.functional.conv2d(torch.from_numpy(At), torch.from_numpy(Wt), stride=stride, padding=pad).numpy()
    got, T = oracle.hbmm_conv2d(A, Wf, beta_a, beta_w, stride, pad, want_T=True)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12 * max(1.0, float(np.abs(ref).max())))
    assert np.all(T >= np.abs(got) - 1e-12)


def test_conv_activation_segments_run_along_the_width():
    """|A| depends on the width index only, so segment means along the width differ from |A| while
    means along the height (the wrong axis) would reproduce |A| itself.  Eq. 3: the segment index
    is floor(y / beta_a) with y the width."""
    B, C, H, W = 1, 2, 4, 8
    A = np.broadcast_to(np.arange(1, W + 1, dtype=np.float32), (B, C, H, W)).copy()
    A[:, :, 1::2, :] *= -1.0
    At = oracle.materialize_activations(A, 4)
    np.testing.assert_array_equal(np.abs(At[0, 0, 0]), [2.5] * 4 + [6.5] * 4)
    np.testing.assert_array_equal(np.sign(At), np.sign(A))
    # a 1x1 filter with a single +1 weight reads the materialised activations back
    Wf = np.zeros((1, C, 1, 1), dtype=np.float32)
    Wf[0, 0, 0, 0] = 3.0
    out = oracle.hbmm_conv2d(A, Wf, 4, 1, 1, 0)
    np.testing.assert_array_equal(out[0, 0], 3.0 * At[0, 0])


def test_conv_activation_segments_with_a_shorter_last_one():
    """Widths that beta_a does not divide (7 x 7 feature maps with beta_a = 4 or 2; the paper asks only
    beta_a <= w_in): every row's last segment is the remainder, averaged over its own length -- means
    written out by hand here -- and segments never run on into the next row."""
    A = np.array([1, -2, 3, -4, 5, -6, 7], dtype=np.float32) * np.ones((1, 2, 3, 1), dtype=np.float32)
    A[0, 1] *= 2.0
    At = oracle.materialize_activations(A, 4)
    np.testing.assert_array_equal(At[0, 0, 1], [2.5, -2.5, 2.5, -2.5, 6.0, -6.0, 6.0])      # (1+2+3+4)/4, (5+6+7)/3
    np.testing.assert_array_equal(At[0, 1, 2], [5.0, -5.0, 5.0, -5.0, 12.0, -12.0, 12.0])
    At2 = oracle.materialize_activations(A, 2)
    np.testing.assert_array_equal(np.abs(At2[0, 0, 0]), [1.5, 1.5, 3.5, 3.5, 5.5, 5.5, 7.0])   # the last one alone
    # through the layer: a 1 x 1 filter with one weight reads the materialised tensor back, and with exact
    # rationals a 3 x 3 window over it gives the same sums as the oracle
    Wf = np.zeros((1, 2, 3, 3), dtype=np.float32)
    Wf[0, :, :, :] = np.arange(1, 19, dtype=np.float32).reshape(2, 3, 3) - 9.0
    got = oracle.hbmm_conv2d(A, Wf, 4, 1, 1, 1)
    for oz in range(3):
        for oy in range(7):
            acc = Fraction(0)
            for c in range(2):
                for dz in range(3):
                    for dy in range(3):
                        z, y = oz - 1 + dz, oy - 1 + dy
                        if 0 <= z < 3 and 0 <= y < 7:
                            acc += Fraction(float(At[0, c, z, y])) * Fraction(float(Wf[0, c, dz, dy]))
            assert got[0, 0, oz, oy] == float(acc)


def test_conv_filter_segments_run_over_the_flattened_filter():
    """Eq. 1: the filter is reshaped to (filters, C*KH*KW) before it is cut into segments, so a
    segment may cross kernel rows and channels.  With beta_w = C*KH*KW the scale is one per filter."""
    rng = np.random.default_rng(5)
    Wf = rng.standard_normal((2, 2, 3, 3)).astype(np.float32)
    Wt = oracle.materialize_filters(Wf, 6)
    flat = np.abs(Wf.reshape(2, 18).astype(np.float64))
    for n in range(2):
        for j in range(3):
            np.testing.assert_allclose(np.abs(Wt.reshape(2, 18)[n, 6 * j:6 * j + 6]),
                                       np.float32(flat[n, 6 * j:6 * j + 6].mean()), rtol=0, atol=0)
    Wt_all = oracle.materialize_filters(Wf, 18)
    for n in range(2):
        assert np.unique(np.abs(Wt_all[n])).size == 1


def test_conv_beta_one_is_plain_convolution_and_brute_force():
    """beta = 1 on both sides leaves both tensors as they are; the result must equal a convolution
    evaluated term by term with exact rationals (catches index or padding slips the library pin
    could share, and dropped boundary terms)."""
    rng = np.random.default_rng(9)
    B, C, H, W, N, KH, KW, stride, pad = 1, 2, 4, 4, 2, 3, 3, 1, 1
    A = rng.integers(-3, 4, (B, C, H, W)).astype(np.float32)
    Wf = rng.integers(-2, 3, (N, C, KH, KW)).astype(np.float32)
    got, T = oracle.hbmm_conv2d(A, Wf, 1, 1, stride, pad, want_T=True)
    for n in range(N):
        for oz in range(H):
            for oy in range(W):
                acc, tabs = Fraction(0), Fraction(0)
                for c in range(C):
                    for dz in range(KH):
                        for dy in range(KW):
                            z, y = oz - pad + dz, oy - pad + dy
                            if 0 <= z < H and 0 <= y < W:
                                term = Fraction(float(A[0, c, z, y])) * Fraction(float(Wf[n, c, dz, dy]))
                                acc += term
                                tabs += abs(term)
                assert got[0, n, oz, oy] == float(acc)
                assert T[0, n, oz, oy] == float(tabs)      # the error scale is the sum of the absolute terms, exactly
