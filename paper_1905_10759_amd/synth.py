"""Seeded synthetic inputs for the HBMM workloads.

This module holds no arithmetic of the method itself (no scales, signs, packing or
products): it only draws the full-precision operands.  Both the CPU oracle's tests and
the HIP path's tests/bench take their inputs from here, so the two sides always see
bit-identical fp32 arrays.

Generator: counter based.  Element ``i`` of stream ``seed`` is a pure function of
``(seed, i)`` (SplitMix64 finaliser over a Weyl sequence), so arrays can be produced in
any chunking/threading and are independent of the numpy/torch version.

Workloads (shapes follow ResNet-18 im2col GEMMs and square GEMMs; only layer *shapes*
are used, no dataset or trained weight):

====  ======================  =======  ======================================  ==========
name  M, K, N                 beta     A (M x K)                               B
====  ======================  =======  ======================================  ==========
tiny  64, 512, 64             32/32    N(0,1)                                  K x N, N(0,1)
c2x   3136, 576, 64           64/64    max(0, N(0,1))                          N x K, N(0, sqrt(2/K))
c5x   12544, 4608, 512        128/128  max(0, N(0,1))                          N x K, N(0, sqrt(2/K))
c5xw  12544, 4608, 512        1/128    max(0, N(0,1)) (kept fp32)              N x K, N(0, sqrt(2/K))
sq4k  4096, 4096, 4096        64/64    N(0,1)                                  N x K, N(0,1)
sq8k  8192, 8192, 8192        256/256  U[-1,1)                                 N x K, U[-1,1)
sq4k16  4096, 4096, 4096      16/16    N(0,1)  (the paper's benchmark setting)  N x K, N(0,1)
====  ======================  =======  ======================================  ==========
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int) -> np.uint64:
    with np.errstate(over="ignore"):
        return _mix64(np.array([seed], dtype=np.uint64) * _GOLDEN + _GOLDEN)[0]


def _bits(key: np.uint64, counters: np.ndarray) -> np.ndarray:
    """64 random bits per counter value."""
    with np.errstate(over="ignore"):
        return _mix64((counters + np.uint64(1)) * _GOLDEN + key)


def _unit(key: np.uint64, counters: np.ndarray) -> np.ndarray:
    """Uniform double in the open interval (0, 1): (top 53 bits + 0.5) / 2**53."""
    return ((_bits(key, counters) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _fill(kind: str, seed: int, lo: int, hi: int, out: np.ndarray) -> None:
    key = _key(seed)
    idx = np.arange(lo, hi, dtype=np.uint64)
    if kind == "uniform_pm1":
        out[lo:hi] = (2.0 * _unit(key, idx) - 1.0).astype(np.float32)
    elif kind == "normal":
        u1 = _unit(key, idx * np.uint64(2))
        u2 = _unit(key, idx * np.uint64(2) + np.uint64(1))
        out[lo:hi] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    else:
        raise ValueError(kind)


def _draw(kind: str, seed: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    spans = [(lo, min(lo + _CHUNK, n)) for lo in range(0, n, _CHUNK)]
    workers = max(1, min(16, os.cpu_count() or 1, len(spans)))
    if workers == 1:
        for lo, hi in spans:
            _fill(kind, seed, lo, hi, out)
    else:
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(lambda s: _fill(kind, seed, s[0], s[1], out), spans))
    return out


def normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    """i.i.d. N(0, std^2) as fp32 (Box-Muller in double, rounded once)."""
    n = int(np.prod(shape))
    x = _draw("normal", seed, n)
    if std != 1.0:
        x = (x.astype(np.float64) * std).astype(np.float32)
    return x.reshape(shape)


def uniform_pm1(seed: int, shape) -> np.ndarray:
    """i.i.d. uniform on [-1, 1) as fp32."""
    return _draw("uniform_pm1", seed, int(np.prod(shape))).reshape(shape)


def relu_normal(seed: int, shape) -> np.ndarray:
    """max(0, N(0,1)): about half the entries are exactly +0.0."""
    x = normal(seed, shape)
    return np.where(x > 0, x, np.float32(0.0)).astype(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    K: int
    N: int
    beta_a: int
    beta_w: int
    a_kind: str          # "normal" | "relu_normal" | "uniform_pm1"
    b_kind: str          # "normal" | "he_normal" | "uniform_pm1"
    b_layout: int        # 0: B stored N x K (K contiguous); 1: B stored K x N
    seed_a: int
    seed_b: int

    def make_a(self) -> np.ndarray:
        return _make(self.a_kind, self.seed_a, (self.M, self.K), self.K)

    def make_b(self) -> np.ndarray:
        shape = (self.N, self.K) if self.b_layout == 0 else (self.K, self.N)
        return _make(self.b_kind, self.seed_b, shape, self.K)


def _make(kind: str, seed: int, shape, K: int) -> np.ndarray:
    if kind == "normal":
        return normal(seed, shape)
    if kind == "relu_normal":
        return relu_normal(seed, shape)
    if kind == "he_normal":
        return normal(seed, shape, std=float(np.sqrt(2.0 / K)))
    if kind == "uniform_pm1":
        return uniform_pm1(seed, shape)
    raise ValueError(kind)


WORKLOADS = {
    w.name: w
    for w in (
        Workload("tiny", 64, 512, 64, 32, 32, "normal", "normal", 1, 1001, 1002),
        Workload("c2x", 3136, 576, 64, 64, 64, "relu_normal", "he_normal", 0, 2001, 2002),
        Workload("c5x", 12544, 4608, 512, 128, 128, "relu_normal", "he_normal", 0, 3001, 3002),
        Workload("c5xw", 12544, 4608, 512, 1, 128, "relu_normal", "he_normal", 0, 3001, 3002),
        # the paper's best binary-weight setting (Table 3: beta_w = 4, beta_a = 1) on the same layer shape
        Workload("c5xw4", 12544, 4608, 512, 1, 4, "relu_normal", "he_normal", 0, 3001, 3002),
        Workload("sq4k", 4096, 4096, 4096, 64, 64, "normal", "normal", 0, 4001, 4002),
        Workload("sq8k", 8192, 8192, 8192, 256, 256, "uniform_pm1", "uniform_pm1", 0, 5001, 5002),
        # the setting of the paper's own speed figure (square matrices, beta = 16)
        Workload("sq4k16", 4096, 4096, 4096, 16, 16, "normal", "normal", 0, 6001, 6002),
    )
}


@dataclass(frozen=True)
class ConvWorkload:
    """A convolution layer: activations batch x C x H x W (ReLU'd normal), filters N x C x KH x KW
    (He-normal), activation segments of beta_a along W, filter segments of beta_w over C*KH*KW."""
    name: str
    batch: int
    C: int
    H: int
    W: int
    N: int
    KH: int
    KW: int
    stride: int
    pad: int
    beta_a: int
    beta_w: int
    seed_a: int
    seed_w: int

    def make_a(self) -> np.ndarray:
        return relu_normal(self.seed_a, (self.batch, self.C, self.H, self.W))

    def make_w(self) -> np.ndarray:
        K = self.C * self.KH * self.KW
        return normal(self.seed_w, (self.N, self.C, self.KH, self.KW), std=float(np.sqrt(2.0 / K)))

    @property
    def macs(self) -> int:
        oh = (self.H + 2 * self.pad - self.KH) // self.stride + 1
        ow = (self.W + 2 * self.pad - self.KW) // self.stride + 1
        return self.batch * oh * ow * self.N * self.C * self.KH * self.KW


# ResNet-18 3x3 layers with the paper's convolution semantics.  beta_a divides the width except in conv5x (7 x 7
# maps, beta_a = 4: segments of 4 + 3 per row), which only the prepared-filter form of the layer takes.
CONV_WORKLOADS = {
    w.name: w
    for w in (
        ConvWorkload("conv2x_b1", 1, 64, 56, 56, 64, 3, 3, 1, 1, 8, 64, 7001, 7002),
        ConvWorkload("conv2x_b64", 64, 64, 56, 56, 64, 3, 3, 1, 1, 8, 64, 7001, 7002),
        ConvWorkload("conv3x_b64", 64, 128, 28, 28, 128, 3, 3, 1, 1, 4, 128, 7101, 7102),
        ConvWorkload("conv4x_b64", 64, 256, 14, 14, 256, 3, 3, 1, 1, 2, 128, 7201, 7202),
        ConvWorkload("conv3x_down_b64", 64, 64, 56, 56, 128, 3, 3, 2, 1, 8, 64, 7301, 7302),
        # the paper's own settings on conv3_x: HadaNet (beta_w, beta_a) = (4, 4) and the binary-weight (4, 1)
        ConvWorkload("conv3x_hadanet44_b64", 64, 128, 28, 28, 128, 3, 3, 1, 1, 4, 4, 7101, 7102),
        ConvWorkload("conv3x_hbwn41_b64", 64, 128, 28, 28, 128, 3, 3, 1, 1, 1, 4, 7101, 7102),
        ConvWorkload("conv5x_hadanet44_b64", 64, 512, 7, 7, 512, 3, 3, 1, 1, 4, 4, 7401, 7402),
    )
}
