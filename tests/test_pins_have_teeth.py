"""The pins of the oracle must fail when the oracle is wrong.  Each case below plants one plausible
mistake into the oracle (on the CPU, by wrapping one of its functions), runs the pins that are
meant to catch it and requires at least one of them to fail.  With no mistake planted the same
pins pass (that is the ordinary run of test_oracle_pins.py)."""
from __future__ import annotations

import inspect
import itertools

import numpy as np
import pytest

import oracle
import oracle.hbmm_oracle as impl

import test_oracle_pins as pins

REAL = {name: getattr(impl, name) for name in impl.__all__ if callable(getattr(impl, name))}


# ------------------------------------------------------------------------------ mistakes
def bits_msb_first(x, ldw=None):
    w = REAL["sign_pack"](x, ldw)
    rev = np.zeros_like(w)
    for b in range(32):
        rev |= ((w >> np.uint32(b)) & np.uint32(1)) << np.uint32(31 - b)
    return rev


def sign_of_zero_is_minus(x, ldw=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return REAL["sign_pack"](np.where(x == 0, np.float32(-1), x), ldw)


def pad_bits_set(x, ldw=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = REAL["sign_pack"](x, ldw).copy()
    K = x.shape[1]
    if K % 32:
        w[:, K // 32] |= np.uint32((0xFFFFFFFF << (K % 32)) & 0xFFFFFFFF)
    return w


def mean_over_beta_plus_one(x, beta):
    s = REAL["block_scales"](x, beta)
    return (s.astype(np.float64) * beta / (beta + 1)).astype(np.float32)


def short_segment_divided_by_beta(x, beta):
    x = np.ascontiguousarray(x, dtype=np.float32)
    s = REAL["block_scales"](x, beta).copy()
    tail = x.shape[1] % beta
    if tail:
        s[:, -1] = (s[:, -1].astype(np.float64) * tail / beta).astype(np.float32)
    return s


def scale_without_abs(x, beta):
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, K = x.shape
    nb = (K + beta - 1) // beta
    s = np.zeros((rows, nb), dtype=np.float32)
    for j in range(nb):
        s[:, j] = x[:, j * beta:(j + 1) * beta].astype(np.float64).mean(axis=1)
    return s


def int_dot_counts_matches(a_bits, b_bits, K):
    return ((REAL["int_dot"](a_bits, b_bits, K).astype(np.int64) + K) // 2).astype(np.int32)


def int_dot_counts_pad_bits(a_bits, b_bits, K):
    a_bits = np.ascontiguousarray(a_bits, dtype=np.uint32)
    Kpad = a_bits.shape[1] * 32
    return REAL["int_dot"](a_bits, b_bits, K) + np.int32(Kpad - K)


def _signs(bits, K):
    by = np.ascontiguousarray(bits, dtype=np.uint32).view(np.uint8)
    return np.unpackbits(by, axis=1, bitorder="little")[:, :K].astype(np.float64) * 2 - 1


def product_with_matching_bit_count(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T=False):
    """Eq. 7 taken literally: the scale product times the number of matching bits."""
    sa, sb = _signs(a_bits, K), _signs(b_bits, K)
    a_s, b_s = np.asarray(a_s, dtype=np.float64), np.asarray(b_s, dtype=np.float64)
    out = np.zeros((sa.shape[0], sb.shape[0]))
    for k in range(K):
        match = (sa[:, k, None] == sb[None, :, k]).astype(np.float64)
        out += a_s[:, k // beta_a, None] * b_s[None, :, k // beta_w] * match
    return (out, np.abs(out)) if want_T else out


def product_sign_flipped(*args, **kw):
    r = REAL["popcount_gemm"](*args, **kw)
    return (-r[0], r[1]) if isinstance(r, tuple) else -r


def product_drops_last_segment(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T=False):
    g = min(beta_a, beta_w)
    return REAL["popcount_gemm"](a_bits, a_s, beta_a, b_bits, b_s, beta_w, K - g if K > g else K, want_T)


def product_forgets_weight_scale(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T=False):
    return REAL["popcount_gemm"](a_bits, a_s, beta_a, b_bits, np.ones_like(b_s), beta_w, K, want_T)


def product_uses_one_scale_index_for_both(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T=False):
    """Mixed segment lengths: the weight's scale looked up with the activation's segment index."""
    b_s = np.asarray(b_s, dtype=np.float32)
    idx = np.minimum((np.arange(b_s.shape[1]) * beta_w) // beta_a, b_s.shape[1] - 1)
    return REAL["popcount_gemm"](a_bits, a_s, beta_a, b_bits, b_s[:, idx], beta_w, K, want_T)


def materialize_next_segments_scale(x, beta, scales=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if scales is None:
        scales = REAL["block_scales"](x, beta)
    return REAL["materialize"](x, beta, np.roll(scales, -1, axis=1))


def dense_product_skips_last_k(At, Bt):
    At, Bt = np.asarray(At, dtype=np.float64), np.asarray(Bt, dtype=np.float64)
    return REAL["dense_f64_gemm"](At[:, :-1], Bt[:, :-1]) if At.shape[1] > 1 else REAL["dense_f64_gemm"](At, Bt)


def binary_weight_ignores_activation_sign(A, b_bits, b_s, beta_w, want_T=False):
    return REAL["binary_weight_gemm"](np.abs(np.asarray(A, dtype=np.float32)), b_bits, b_s, beta_w, want_T)


def layout_one_not_transposed(x, layout):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def backward_plain_ste(x, g, beta, want_T=False):
    """Only the straight-through term: the derivative of the scale is forgotten."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    delta = np.repeat(REAL["block_scales"](x, beta).astype(np.float64), beta, axis=1)[:, :x.shape[1]]
    gx = delta * g * (np.abs(x) <= 1)
    return (gx, np.abs(gx) + 1e-300) if want_T else gx


def backward_strict_mask(x, g, beta, want_T=False):
    x = np.ascontiguousarray(x, dtype=np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    r = REAL["binarize_backward"](x, g, beta, want_T)
    gx = (r[0] if want_T else r).copy()
    delta = np.repeat(REAL["block_scales"](x, beta).astype(np.float64), beta, axis=1)[:, :x.shape[1]]
    edge = np.abs(x) == 1
    gx[edge] -= (delta * g)[edge]
    return (gx, r[1]) if want_T else gx


def backward_segment_sum_without_signs(x, g, beta, want_T=False):
    """sum_j g_j instead of sum_j g_j Sign(x_j) in the scale term."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    rows, K = x.shape
    gx = np.zeros((rows, K))
    s = REAL["block_scales"](x, beta).astype(np.float64)
    for k0 in range(0, K, beta):
        k1 = min(K, k0 + beta)
        seg = g[:, k0:k1].astype(np.float64).sum(axis=1, keepdims=True) / (k1 - k0)
        sign = np.where(x[:, k0:k1] >= 0, 1.0, -1.0)
        gx[:, k0:k1] = sign * seg + s[:, k0 // beta, None] * g[:, k0:k1] * (np.abs(x[:, k0:k1]) <= 1)
    return (gx, np.abs(gx) + 1e-300) if want_T else gx


def activation_segments_along_height(A, beta_a):
    A = np.ascontiguousarray(A, dtype=np.float32)
    if A.shape[2] % beta_a:
        return REAL["materialize_activations"](A, beta_a)
    At = REAL["materialize_activations"](np.ascontiguousarray(A.transpose(0, 1, 3, 2)), beta_a)
    return np.ascontiguousarray(At.transpose(0, 1, 3, 2))


def activation_segments_run_on_into_the_next_row(A, beta_a):
    """A width that beta_a does not divide, cut as one flat run of elements instead of row by row."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B, C, H, W = A.shape
    if W % beta_a == 0 or (B * C * H * W) % beta_a:
        return REAL["materialize_activations"](A, beta_a)
    return REAL["materialize"](A.reshape(1, -1), beta_a).reshape(A.shape)


def activation_short_segment_divided_by_beta(A, beta_a):
    A = np.ascontiguousarray(A, dtype=np.float32)
    At = REAL["materialize_activations"](A, beta_a)
    r = A.shape[3] % beta_a
    if r:
        At[..., -r:] *= r / beta_a
    return At


def filter_segments_restart_per_channel(Wf, beta_w):
    Wf = np.ascontiguousarray(Wf, dtype=np.float32)
    N, C, KH, KW = Wf.shape
    return REAL["materialize"](Wf.reshape(N * C, KH * KW), beta_w).reshape(Wf.shape)


def convolution_flips_the_filter(At, Wt, stride, pad, want_T=False):
    return REAL["conv2d_f64"](At, np.ascontiguousarray(np.asarray(Wt)[:, :, ::-1, ::-1]), stride, pad, want_T)


def convolution_pads_with_ones(At, Wt, stride, pad, want_T=False):
    """Padding that contributes (+1 times the filter) instead of nothing."""
    At = np.asarray(At, dtype=np.float64)
    if pad == 0:
        return REAL["conv2d_f64"](At, Wt, stride, pad, want_T)
    padded = np.pad(At, ((0, 0), (0, 0), (pad, pad), (pad, pad)), constant_values=1.0)
    return REAL["conv2d_f64"](padded, Wt, stride, 0, want_T)


def product_error_scale_doubled(*args, **kw):
    """An inflated T would silently loosen every fp32 parity bar."""
    out = REAL["popcount_gemm"](*args, **kw)
    return (out[0], 2.0 * out[1]) if kw.get("want_T") else out


def product_error_scale_without_abs(*args, **kw):
    out = REAL["popcount_gemm"](*args, **kw)
    return (out[0], np.abs(out[0])) if kw.get("want_T") else out


def backward_error_scale_doubled(x, g, beta, want_T=False):
    out = REAL["binarize_backward"](x, g, beta, want_T)
    return (out[0], 2.0 * out[1]) if want_T else out


def convolution_error_scale_doubled(At, Wt, stride, pad, want_T=False):
    out = REAL["conv2d_f64"](At, Wt, stride, pad, want_T)
    return (out[0], 2.0 * out[1]) if want_T else out


def binary_weight_error_scale_doubled(A, b_bits, b_s, beta_w, want_T=False):
    out = REAL["binary_weight_gemm"](A, b_bits, b_s, beta_w, want_T)
    return (out[0], 2.0 * out[1]) if want_T else out


# mistake -> (oracle function it lives in, pins that must notice)
CASES = [
    (bits_msb_first, "sign_pack", ["test_pack_matches_paper_example", "test_pack_roundtrip_ragged_and_pad_zero",
                                   "test_pack_word_boundaries"]),
    (sign_of_zero_is_minus, "sign_pack", ["test_pack_roundtrip_ragged_and_pad_zero", "test_pack_word_boundaries",
                                          "test_pack_matches_paper_example"]),
    (pad_bits_set, "sign_pack", ["test_pack_roundtrip_ragged_and_pad_zero"]),
    (mean_over_beta_plus_one, "block_scales", ["test_scales_brute_force", "test_scales_special_cases",
                                               "test_scales_expectations"]),
    (short_segment_divided_by_beta, "block_scales", ["test_scales_brute_force"]),
    (scale_without_abs, "block_scales", ["test_scales_brute_force", "test_scales_expectations"]),
    (int_dot_counts_matches, "int_dot", ["test_int_dot_brute_force_and_identities"]),
    (int_dot_counts_pad_bits, "int_dot", ["test_int_dot_brute_force_and_identities"]),
    (product_with_matching_bit_count, "popcount_gemm", ["test_hbmm_brute_force", "test_paths_agree_and_T_bounds"]),
    (product_sign_flipped, "popcount_gemm", ["test_hbmm_brute_force", "test_hbmm_all_sign_patterns_one_block"]),
    (product_drops_last_segment, "popcount_gemm", ["test_hbmm_brute_force"]),
    (product_forgets_weight_scale, "popcount_gemm", ["test_hbmm_brute_force", "test_whole_row_blocks_reduce_to_xnor_net"]),
    (product_uses_one_scale_index_for_both, "popcount_gemm", ["test_hbmm_brute_force"]),
    (materialize_next_segments_scale, "materialize", ["test_materialize_brute_force", "test_hbmm_brute_force"]),
    (dense_product_skips_last_k, "dense_f64_gemm", ["test_hbmm_brute_force", "test_beta_one_is_plain_matmul"]),
    (binary_weight_ignores_activation_sign, "binary_weight_gemm", ["test_binary_weight_form", "test_hbmm_brute_force"]),
    (layout_one_not_transposed, "as_rows_by_k", ["test_layout_one_is_transpose"]),
    (backward_plain_ste, "binarize_backward", ["test_backward_matches_library_autograd",
                                               "test_backward_scale_path_is_the_true_derivative"]),
    (backward_strict_mask, "binarize_backward", ["test_backward_brute_force_ragged_and_mask_edges"]),
    (backward_segment_sum_without_signs, "binarize_backward", ["test_backward_matches_library_autograd",
                                                               "test_backward_brute_force_ragged_and_mask_edges"]),
    (activation_segments_along_height, "materialize_activations", ["test_conv_activation_segments_run_along_the_width",
                                                                   "test_conv_matches_library_convolution"]),
    (activation_segments_run_on_into_the_next_row, "materialize_activations", ["test_conv_activation_segments_with_a_shorter_last_one"]),
    (activation_short_segment_divided_by_beta, "materialize_activations", ["test_conv_activation_segments_with_a_shorter_last_one"]),
    (filter_segments_restart_per_channel, "materialize_filters", ["test_conv_filter_segments_run_over_the_flattened_filter",
                                                                  "test_conv_matches_library_convolution"]),
    (convolution_flips_the_filter, "conv2d_f64", ["test_conv_matches_library_convolution",
                                                  "test_conv_beta_one_is_plain_convolution_and_brute_force"]),
    (convolution_pads_with_ones, "conv2d_f64", ["test_conv_matches_library_convolution",
                                                "test_conv_beta_one_is_plain_convolution_and_brute_force"]),
    (product_error_scale_doubled, "popcount_gemm", ["test_error_scale_T_of_the_product_is_the_sum_of_absolute_terms"]),
    (product_error_scale_without_abs, "popcount_gemm", ["test_error_scale_T_of_the_product_is_the_sum_of_absolute_terms"]),
    (backward_error_scale_doubled, "binarize_backward", ["test_backward_brute_force_ragged_and_mask_edges"]),
    (convolution_error_scale_doubled, "conv2d_f64", ["test_conv_beta_one_is_plain_convolution_and_brute_force"]),
    (binary_weight_error_scale_doubled, "binary_weight_gemm", ["test_binary_weight_form"]),
]


# ------------------------------------------------------------------------------ runner
def pin_invocations(name: str, golden_dir):
    """(label, callable) for every parameter set of one pin."""
    fn = getattr(pins, name)
    axes = []
    for mark in getattr(fn, "pytestmark", []):
        if mark.name != "parametrize":
            continue
        names = [n.strip() for n in mark.args[0].split(",")]
        axes.append([dict(zip(names, v if len(names) > 1 else (v,))) for v in mark.args[1]])
    for combo in itertools.product(*axes) if axes else [()]:
        kwargs = {}
        for part in combo:
            kwargs.update(part)
        if "golden_dir" in inspect.signature(fn).parameters:
            kwargs["golden_dir"] = golden_dir
        yield f"{name}{sorted(kwargs.items()) if combo else ''}", (lambda f=fn, k=kwargs: f(**k))


def failing_pins(names, golden_dir):
    failed = []
    for name in names:
        for label, call in pin_invocations(name, golden_dir):
            try:
                call()
            except AssertionError:
                failed.append(label)
    return failed


@pytest.mark.parametrize("mistake,where,catchers", CASES, ids=[c[0].__name__ for c in CASES])
def test_planted_mistake_is_caught(monkeypatch, golden_dir, mistake, where, catchers):
    assert where in REAL
    monkeypatch.setattr(impl, where, mistake)      # callers inside the oracle module
    monkeypatch.setattr(oracle, where, mistake)    # callers that go through the package
    failed = failing_pins(catchers, golden_dir)
    assert failed, f"no pin noticed '{mistake.__name__}' planted in oracle.{where}"


def test_the_runner_itself_reports_clean_pins_as_passing(golden_dir):
    names = sorted({n for _, _, catchers in CASES for n in catchers})
    assert failing_pins(names, golden_dir) == []
