"""The five benchmark workloads (and the binary-weight variant of the third) at FULL size, in the
launch configuration bench.py times: packed words and integer dots are checked bit-exactly in
full against the oracle's integer path; fp32 outputs in full against the oracle's integer path
and, on sampled rows, against its dense double-precision path."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_1905_10759_amd import synth

from gpu_common import assert_close_to_oracle, dev, plain_relative_error, words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hbmm():
    assert torch.cuda.is_available()
    from paper_1905_10759_amd import hbmm as mod
    return mod


def scale_tol(beta):
    return (np.log2(beta) + 1) * 2.0 ** -24


@pytest.mark.parametrize("name", ["tiny", "c2x", "c5x", "sq4k", "sq8k"])
def test_workload_full_size(hbmm, name):
    w = synth.WORKLOADS[name]
    A, Bsrc = w.make_a(), w.make_b()
    B = oracle.as_rows_by_k(Bsrc, w.b_layout)
    print(f"[{name}] inputs ready", flush=True)

    a_bits, a_s = hbmm.quantize_pack(dev(A), w.beta_a)
    b_bits, b_s = hbmm.quantize_pack(dev(Bsrc), w.beta_w, layout=w.b_layout)
    torch.cuda.synchronize()

    # --- pack: words bit-exact, scales to the fp32 pairwise-sum bound
    ra, rb = oracle.sign_pack(A), oracle.sign_pack(B)
    assert np.array_equal(words(a_bits), ra)
    assert np.array_equal(words(b_bits), rb)
    sa, sb = oracle.block_scales(A, w.beta_a), oracle.block_scales(B, w.beta_w)
    assert np.all(np.abs(a_s.cpu().numpy() - sa) <= scale_tol(w.beta_a) * sa + 1e-30)
    assert np.all(np.abs(b_s.cpu().numpy() - sb) <= scale_tol(w.beta_w) * sb + 1e-30)
    print(f"[{name}] pack ok", flush=True)

    # --- integer contraction, every output
    D = hbmm.gemm_int(a_bits, b_bits, w.K).cpu().numpy()
    assert np.array_equal(D, oracle.int_dot(ra, rb, w.K))
    del D
    print(f"[{name}] int dots ok", flush=True)

    # --- scaled outputs, every output, same scales on both sides
    ref, T = oracle.popcount_gemm(ra, sa, w.beta_a, rb, sb, w.beta_w, w.K, want_T=True)
    got = hbmm.gemm(a_bits, dev(sa), w.beta_a, b_bits, dev(sb), w.beta_w, w.K).cpu().numpy()
    worst = assert_close_to_oracle(got, ref, T, name)
    print(f"[{name}] gemm ok, worst err/(1e-5 T) = {worst:.3f}, worst plain relative error = {plain_relative_error(got, ref):.2e}", flush=True)

    # --- the matrix-core variants reach the same segment sums and round in the same places
    same = torch.from_numpy(got).cuda()
    assert torch.equal(hbmm.gemm(a_bits, dev(sa), w.beta_a, b_bits, dev(sb), w.beta_w, w.K, algo=1), same)
    if min(w.beta_a, w.beta_w) >= 64:
        assert torch.equal(hbmm.gemm(a_bits, dev(sa), w.beta_a, b_bits, dev(sb), w.beta_w, w.K, algo=2), same)
    del same
    print(f"[{name}] matrix-core variants identical", flush=True)

    # --- whole path with the GPU's own scales against the dense f64 definition, sampled rows
    got2 = hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K).cpu().numpy()
    rows = np.unique(np.linspace(0, w.M - 1, 24).astype(np.int64))
    dense = oracle.dense_f64_gemm(oracle.materialize(A[rows], w.beta_a), oracle.materialize(B, w.beta_w))
    assert_close_to_oracle(got2[rows], dense, T[rows], name + " (dense f64, sampled rows)")


def test_workload_paper_setting_beta16(hbmm):
    """Square 4096^3 with beta = 16 on both sides (the paper's own benchmark setting): whole path on
    the GPU; every output against the oracle's integer path, sampled rows against the dense path."""
    w = synth.WORKLOADS["sq4k16"]
    A, B = w.make_a(), w.make_b()
    a_bits, a_s = hbmm.quantize_pack(dev(A), w.beta_a)
    b_bits, b_s = hbmm.quantize_pack(dev(B), w.beta_w)
    ra, rb = oracle.sign_pack(A), oracle.sign_pack(B)
    sa, sb = oracle.block_scales(A, w.beta_a), oracle.block_scales(B, w.beta_w)
    assert np.array_equal(words(a_bits), ra) and np.array_equal(words(b_bits), rb)
    assert np.all(np.abs(a_s.cpu().numpy() - sa) <= scale_tol(16) * sa)
    got = hbmm.gemm(a_bits, dev(sa), 16, b_bits, dev(sb), 16, w.K).cpu().numpy()
    ref, T = oracle.popcount_gemm(ra, sa, 16, rb, sb, 16, w.K, want_T=True)
    worst = assert_close_to_oracle(got, ref, T, "sq4k16")
    print(f"[sq4k16] ok, worst err/(1e-5 T) = {worst:.3f}, worst plain relative error = {plain_relative_error(got, ref):.2e}", flush=True)
    rows = np.unique(np.linspace(0, w.M - 1, 16).astype(np.int64))
    dense = oracle.dense_f64_gemm(oracle.materialize(A[rows], 16, sa[rows]), oracle.materialize(B, 16, sb))
    assert_close_to_oracle(got[rows], dense, T[rows], "sq4k16 (dense f64, sampled rows)")


@pytest.mark.parametrize("name", ["c5xw", "c5xw4"])
def test_workload_binary_weight_full_size(hbmm, name):
    """beta_a = 1 at full size: with beta_w = 128, and with the paper's own beta_w = 4 (Table 3)."""
    w = synth.WORKLOADS[name]
    A, B = w.make_a(), w.make_b()
    b_bits, b_s = hbmm.quantize_pack(dev(B), w.beta_w)
    rb, sb = oracle.sign_pack(B), oracle.block_scales(B, w.beta_w)
    assert np.array_equal(words(b_bits), rb)
    got = hbmm.gemm(None, dev(A), 1, b_bits, dev(sb), w.beta_w, w.K).cpu().numpy()
    print(f"[{name}] gpu done", flush=True)
    ref, T = oracle.binary_weight_gemm(A, rb, sb, w.beta_w, want_T=True)
    worst = assert_close_to_oracle(got, ref, T, name)
    print(f"[{name}] ok, worst err/(1e-5 T) = {worst:.3f}, worst plain relative error = {plain_relative_error(got, ref):.2e}", flush=True)
    rows = np.unique(np.linspace(0, w.M - 1, 16).astype(np.int64))
    dense = oracle.dense_f64_gemm(oracle.materialize(A[rows], 1), oracle.materialize(B, w.beta_w, sb))
    assert_close_to_oracle(got[rows], dense, T[rows], name + " (dense f64, sampled rows)")


@pytest.mark.parametrize("name,batch", [("conv2x_b1", 1), ("conv3x_b64", 4), ("conv4x_b64", 8), ("conv3x_down_b64", 2),
                                        ("conv3x_hadanet44_b64", 4), ("conv3x_hbwn41_b64", 4), ("conv5x_hadanet44_b64", 8)])
def test_conv_workload(hbmm, name, batch):
    """ResNet-18 convolution layers at their real geometry (batch cut to what the oracle's loops
    finish in seconds): every output against the oracle's plain convolution."""
    import dataclasses
    w = dataclasses.replace(synth.CONV_WORKLOADS[name], batch=batch)
    A, Wf = w.make_a(), w.make_w()
    # beta_a = 1: the activations are not binarised and go in as they are
    ragged = w.W % w.beta_a != 0     # (7 x 7 maps with beta_a = 4: the prepared-filter form only)
    ab, asc = (None, dev(A)) if w.beta_a == 1 else (hbmm.quantize_pack_activations if ragged else hbmm.quantize_pack_tensor)(dev(A), w.beta_a)
    wb, ws = hbmm.quantize_pack(dev(Wf.reshape(w.N, -1)), w.beta_w)
    # the oracle computes its own scales from the same inputs; the GPU's differ by their fp32
    # summation order, (log2 beta + 1) * 2^-24 relative at most, far inside the bound
    ref, T = oracle.hbmm_conv2d(A, Wf, w.beta_a, w.beta_w, w.stride, w.pad, want_T=True)
    if not ragged:
        got = hbmm.conv2d(ab, asc, w.beta_a, A.shape, wb, ws, w.beta_w, (w.KH, w.KW), w.stride, w.pad).cpu().numpy()
        print(f"[{name}] gpu done", flush=True)
        worst = assert_close_to_oracle(got, ref, T, name)
        print(f"[{name}] ok, worst err/(1e-5 T) = {worst:.3f}, worst plain relative error = {plain_relative_error(got, ref):.2e}", flush=True)
    # the same layer with the filters prepared ahead of time
    prepared = hbmm.conv_prepare_filters(wb, ws, w.beta_w, w.C, (w.KH, w.KW))
    got_p = hbmm.conv2d_prepared(ab, asc, w.beta_a, A.shape, prepared, w.N, (w.KH, w.KW), w.stride, w.pad).cpu().numpy()
    worst_p = assert_close_to_oracle(got_p, ref, T, name + " (prepared filters)")
    print(f"[{name}] prepared filters ok, worst err/(1e-5 T) = {worst_p:.3f}, worst plain relative error = "
          f"{plain_relative_error(got_p, ref):.2e}", flush=True)
    # ... and in the two-piece form (two fp16 pieces per number, 22 significant bits): the same bar
    prepared = hbmm.conv_prepare_filters(wb, ws, w.beta_w, w.C, (w.KH, w.KW), form=hbmm.PIECES_F16X2)
    got_2 = hbmm.conv2d_prepared(ab, asc, w.beta_a, A.shape, prepared, w.N, (w.KH, w.KW), w.stride, w.pad,
                                 form=hbmm.PIECES_F16X2).cpu().numpy()
    worst_2 = assert_close_to_oracle(got_2, ref, T, name + " (prepared filters, two fp16 pieces)")
    print(f"[{name}] two fp16 pieces ok, worst err/(1e-5 T) = {worst_2:.3f}, worst plain relative error = "
          f"{plain_relative_error(got_2, ref):.2e}", flush=True)
