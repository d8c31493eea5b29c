"""Shared helpers of the GPU parity tests (host <-> device plumbing and tolerances only)."""
from __future__ import annotations

import numpy as np
import torch


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def words(t: torch.Tensor) -> np.ndarray:
    """Packed words come back as int32 tensors; view them as the uint32 they are."""
    return t.cpu().numpy().view(np.uint32)


# fp32 accumulation of nb scaled terms against the double-precision oracle: each term carries two
# fp32 roundings and each of the nb additions one more, so |err| <= (nb + 2) * 2^-24 * T with
# T = sum |terms| (nb <= 144 in every case used here, i.e. <= 8.7e-6 * T).  The bar is the stated
# 1e-5, taken relative to T because the outputs of symmetric random operands cancel towards 0.
REL_TOL = 1e-5


def assert_close_to_oracle(got: np.ndarray, ref: np.ndarray, T: np.ndarray, what: str = ""):
    err = np.abs(got.astype(np.float64) - ref)
    bound = REL_TOL * T + 1e-30
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, f"{what}: max err/(1e-5*T) = {worst:.3f}"
    # plain relative error where the reference is not cancelled away
    big = np.abs(ref) >= 1e-3 * np.abs(ref).max() if ref.size else np.zeros_like(ref, bool)
    if big.any():
        rel = float((err[big] / np.abs(ref[big])).max())
        assert rel <= 1e-3, f"{what}: max plain relative error {rel:.2e}"
    return worst
