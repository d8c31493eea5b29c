"""Buffers whose element offsets pass 2^31: the kernels index rows with 64-bit arithmetic, and these
cases put sampled rows on both sides of that boundary.  The oracle sees the sampled rows only
(whole rows, copied back from the device); the other rows are covered by properties that hold at
any size (bit counts, segment sums) and by the agreement of two differently tiled kernels."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
from paper_1905_10759_amd import synth

from gpu_common import assert_close_to_oracle, dev, words

pytestmark = pytest.mark.gpu

TWO31 = 1 << 31


@pytest.fixture(scope="module")
def hbmm():
    assert torch.cuda.is_available()
    from paper_1905_10759_amd import hbmm as mod
    return mod


def sample_rows(n_rows: int, row_len: int) -> np.ndarray:
    """First and last rows, and the rows around the one whose first element has offset 2^31."""
    edge = TWO31 // row_len
    rows = [0, 1, n_rows // 3, edge - 1, edge, edge + 1, n_rows - 2, n_rows - 1]
    return np.unique(np.clip(np.array(rows, dtype=np.int64), 0, n_rows - 1))


def test_pack_source_past_2_31_elements(hbmm):
    rows, K, beta = 33000, 65536, 128
    assert rows * K > TWO31
    gen = torch.Generator(device="cuda").manual_seed(7001)
    x = torch.empty((rows, K), dtype=torch.float32, device="cuda")
    for r0 in range(0, rows, 4096):   # filled in slabs: one randn call of 2^31 elements is not needed
        r1 = min(rows, r0 + 4096)
        x[r0:r1].normal_(generator=gen)
    bits, scales = hbmm.quantize_pack(x, beta)
    torch.cuda.synchronize()
    print("[large pack] gpu done", flush=True)

    pick = sample_rows(rows, K)
    host = x[torch.from_numpy(pick).cuda()].cpu().numpy()
    assert np.array_equal(words(bits[torch.from_numpy(pick).cuda()]), oracle.sign_pack(host))
    ref_s = oracle.block_scales(host, beta)
    got_s = scales[torch.from_numpy(pick).cuda()].cpu().numpy()
    assert np.all(np.abs(got_s - ref_s) <= 8 * 2.0 ** -24 * ref_s)

    # every row: number of set bits = number of non-negative elements; beta * sum of scales = sum |x|
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int32, device="cuda")
    for r0 in range(0, rows, 4096):
        r1 = min(rows, r0 + 4096)
        ones = lut[bits[r0:r1].view(torch.uint8).long()].sum(dim=1)
        assert torch.equal(ones, (x[r0:r1] >= 0).sum(dim=1).to(torch.int32)), f"rows {r0}..{r1}"
        l1 = x[r0:r1].abs().sum(dim=1, dtype=torch.float64)
        assert torch.allclose(scales[r0:r1].sum(dim=1, dtype=torch.float64) * beta, l1, rtol=1e-5, atol=0)


def test_gemm_output_past_2_31_elements(hbmm):
    M, N, K, beta = 46400, 46500, 256, 64
    assert M * N > TWO31
    A, B = synth.normal(7101, (M, K)), synth.normal(7102, (N, K))
    a_bits, a_s = hbmm.quantize_pack(dev(A), beta)
    b_bits, b_s = hbmm.quantize_pack(dev(B), beta)
    pick = sample_rows(M, N)
    sel = torch.from_numpy(pick).cuda()
    ra, rb = oracle.sign_pack(A[pick]), oracle.sign_pack(B)
    sa, sb = a_s[sel].cpu().numpy(), b_s.cpu().numpy()     # the GPU's own scales on both sides
    ref, T = oracle.popcount_gemm(ra, sa, beta, rb, sb, beta, K, want_T=True)

    got = hbmm.gemm(a_bits, a_s, beta, b_bits, b_s, beta, K)
    torch.cuda.synchronize()
    print("[large gemm] popcount kernel done", flush=True)
    assert_close_to_oracle(got[sel].cpu().numpy(), ref, T, "large gemm, sampled rows")

    # the fp4 matrix-core kernel tiles the output differently and must give the same bits everywhere
    other = hbmm.gemm(a_bits, a_s, beta, b_bits, b_s, beta, K, algo=hbmm.ALGO_MFMA_FP4)
    torch.cuda.synchronize()
    print("[large gemm] fp4 kernel done", flush=True)
    assert torch.equal(got, other)
    del other, got

    D = hbmm.gemm_int(a_bits, b_bits, K)
    torch.cuda.synchronize()
    print("[large gemm] integer kernel done", flush=True)
    assert np.array_equal(D[sel].cpu().numpy(), oracle.int_dot(ra, rb, K))
    # every output: same parity as K, and |D| <= K
    assert int(D.abs().max()) <= K
    assert not bool((D & 1).any())
