"""Randomised pins for the oracle (hypothesis): shapes, segment lengths and values are drawn at
random, the expected value always comes from the exact-rational brute force of test_oracle_pins.py
or from an identity -- never from the oracle itself and never from the GPU path."""
from __future__ import annotations

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_pins import brute_hbmm, brute_scales, unpack

SETTINGS = dict(max_examples=60, deadline=None)


def matrix(draw, rows, K, kind):
    """fp32 values with exact zeros, negative zeros and ties mixed in."""
    seed = draw(st.integers(0, 2 ** 31 - 1))
    rng = np.random.default_rng(seed)
    if kind == 0:
        x = rng.standard_normal((rows, K)).astype(np.float32)
    elif kind == 1:
        x = np.maximum(rng.standard_normal((rows, K)), 0).astype(np.float32)          # rectified: many +0.0
    else:
        x = rng.integers(-2, 3, size=(rows, K)).astype(np.float32) * np.float32(0.5)  # few distinct values, zeros, ties
        x[rng.random((rows, K)) < 0.1] = np.float32(-0.0)
    return x


@st.composite
def problem(draw):
    M, N, K = draw(st.integers(1, 5)), draw(st.integers(1, 5)), draw(st.integers(1, 70))
    betas = [1, 2, 3, 4, 5, 8, 16, 32, K]
    beta_a, beta_w = draw(st.sampled_from(betas)), draw(st.sampled_from(betas))
    A = matrix(draw, M, K, draw(st.integers(0, 2)))
    B = matrix(draw, N, K, draw(st.integers(0, 2)))
    return A, B, beta_a, beta_w


@settings(**SETTINGS)
@given(problem())
def test_dense_path_equals_exact_rational_product(p):
    A, B, beta_a, beta_w = p
    want = brute_hbmm(A, B, beta_a, beta_w)
    got = oracle.hbmm_dense(A, B, beta_a, beta_w)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * max(1.0, np.abs(want).max()))


@settings(**SETTINGS)
@given(problem())
def test_integer_path_equals_exact_rational_product(p):
    A, B, beta_a, beta_w = p
    if beta_a == 1 or beta_w == 1:
        beta_a, beta_w = max(beta_a, 2), max(beta_w, 2)
    want = brute_hbmm(A, B, beta_a, beta_w)
    got, T = oracle.hbmm_popcount(A, B, beta_a, beta_w, want_T=True)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * max(1.0, np.abs(want).max()))
    assert np.all(T >= np.abs(got) - 1e-12 * max(1.0, np.abs(want).max()))


@settings(**SETTINGS)
@given(problem())
def test_pack_scales_and_integer_dots(p):
    A, B, beta_a, _ = p
    K = A.shape[1]
    a, b = oracle.sign_pack(A), oracle.sign_pack(B)
    ua, ub = unpack(a, K), unpack(b, K)
    assert np.array_equal(ua, (A >= 0).astype(np.int64))
    assert not unpack(a, a.shape[1] * 32)[:, K:].any()
    assert np.array_equal(oracle.block_scales(A, beta_a), brute_scales(A, beta_a))
    want = (2 * ua - 1) @ (2 * ub - 1).T
    assert np.array_equal(oracle.int_dot(a, b, K), want)


@settings(**SETTINGS)
@given(problem())
def test_binary_weight_form_equals_exact_rational_product(p):
    A, B, _, beta_w = p
    beta_w = max(beta_w, 2)
    want = brute_hbmm(A, B, 1, beta_w)
    got = oracle.binary_weight_gemm(A, oracle.sign_pack(B), oracle.block_scales(B, beta_w), beta_w)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * max(1.0, np.abs(want).max()))
