"""ctypes front end of the C oracle (``hbmm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``; never by the product package.  It takes and returns
host numpy arrays and does no arithmetic of its own beyond calling the C functions in the
order the paper's definitions give (scale -> sign -> Hadamard product -> matrix product).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

__all__ = [
    "num_threads", "num_blocks", "ld_words", "block_scales", "sign_pack", "materialize",
    "dense_f64_gemm", "popcount_gemm", "int_dot", "binary_weight_gemm", "hbmm_dense",
    "hbmm_popcount", "as_rows_by_k", "binarize_backward", "conv_out_size", "materialize_activations",
    "materialize_filters", "conv2d_f64", "hbmm_conv2d",
]

_lib = None


def _load():
    global _lib
    if _lib is None:
        # HBMM_ORACLE_LIB: another build of the same source (the sanitizer test points it at an
        # instrumented one)
        path = os.environ.get("HBMM_ORACLE_LIB") or _build.build(force=False)
        lib = C.CDLL(str(path))
        i64, p = C.c_int64, C.c_void_p
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_block_scales.argtypes = [p, i64, i64, i64, i64, p, i64]
        lib.oracle_sign_pack.argtypes = [p, i64, i64, i64, p, i64]
        lib.oracle_materialize.argtypes = [p, i64, i64, i64, i64, p, i64, p]
        lib.oracle_dense_f64_gemm.argtypes = [p, p, i64, i64, i64, p]
        lib.oracle_popcount_gemm.argtypes = [p, i64, p, i64, i64, p, i64, p, i64, i64, i64, i64, i64, p, p]
        lib.oracle_int_dot.argtypes = [p, i64, p, i64, i64, i64, i64, p]
        lib.oracle_binary_weight_gemm.argtypes = [p, i64, p, i64, p, i64, i64, i64, i64, i64, p, p]
        lib.oracle_binarize_backward.argtypes = [p, p, i64, i64, i64, i64, i64, p, p]
        lib.oracle_conv2d_f64.argtypes = [p, p, i64, i64, i64, i64, i64, i64, i64, i64, i64, p, p]
        lib.oracle_binarize_backward.restype = None
        for name in ("oracle_block_scales", "oracle_sign_pack", "oracle_materialize", "oracle_dense_f64_gemm",
                     "oracle_popcount_gemm", "oracle_int_dot", "oracle_binary_weight_gemm"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32_rows(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 2:
        raise ValueError("expected a 2-D array")
    return x


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def num_blocks(K: int, beta: int) -> int:
    return (K + beta - 1) // beta


def ld_words(K: int) -> int:
    """32-bit words per packed row, rounded up to a multiple of 4 (16-byte rows)."""
    return ((K + 31) // 32 + 3) // 4 * 4


def as_rows_by_k(x: np.ndarray, layout: int) -> np.ndarray:
    """layout 0: x is rows x K already.  layout 1: x is K x rows (the usual K x N way of
    writing the right-hand operand); its transpose is the rows x K operand W^f."""
    x = np.asarray(x, dtype=np.float32)
    return np.ascontiguousarray(x if layout == 0 else x.T)


def block_scales(x, beta: int) -> np.ndarray:
    x = _f32_rows(x)
    rows, K = x.shape
    s = np.zeros((rows, num_blocks(K, beta)), dtype=np.float32)
    _load().oracle_block_scales(_ptr(x), rows, K, K, beta, _ptr(s), s.shape[1])
    return s


def sign_pack(x, ldw: int | None = None) -> np.ndarray:
    x = _f32_rows(x)
    rows, K = x.shape
    ldw = ld_words(K) if ldw is None else ldw
    bits = np.empty((rows, ldw), dtype=np.uint32)
    _load().oracle_sign_pack(_ptr(x), rows, K, K, _ptr(bits), ldw)
    return bits


def materialize(x, beta: int, scales: np.ndarray | None = None) -> np.ndarray:
    x = _f32_rows(x)
    rows, K = x.shape
    if scales is None:
        scales = block_scales(x, beta)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    out = np.empty((rows, K), dtype=np.float64)
    _load().oracle_materialize(_ptr(x), rows, K, K, beta, _ptr(scales), scales.shape[1], _ptr(out))
    return out


def dense_f64_gemm(At: np.ndarray, Bt: np.ndarray) -> np.ndarray:
    At = np.ascontiguousarray(At, dtype=np.float64)
    Bt = np.ascontiguousarray(Bt, dtype=np.float64)
    M, K = At.shape
    N, K2 = Bt.shape
    if K != K2:
        raise ValueError("K mismatch")
    out = np.empty((M, N), dtype=np.float64)
    _load().oracle_dense_f64_gemm(_ptr(At), _ptr(Bt), M, N, K, _ptr(out))
    return out


def popcount_gemm(a_bits, a_s, beta_a, b_bits, b_s, beta_w, K, want_T: bool = False):
    a_bits = np.ascontiguousarray(a_bits, dtype=np.uint32)
    b_bits = np.ascontiguousarray(b_bits, dtype=np.uint32)
    a_s = np.ascontiguousarray(a_s, dtype=np.float32)
    b_s = np.ascontiguousarray(b_s, dtype=np.float32)
    M, N = a_bits.shape[0], b_bits.shape[0]
    out = np.empty((M, N), dtype=np.float64)
    T = np.empty((M, N), dtype=np.float64) if want_T else None
    _load().oracle_popcount_gemm(_ptr(a_bits), a_bits.shape[1], _ptr(a_s), a_s.shape[1], beta_a,
                                 _ptr(b_bits), b_bits.shape[1], _ptr(b_s), b_s.shape[1], beta_w,
                                 M, N, K, _ptr(out), _ptr(T) if want_T else None)
    return (out, T) if want_T else out


def int_dot(a_bits, b_bits, K) -> np.ndarray:
    a_bits = np.ascontiguousarray(a_bits, dtype=np.uint32)
    b_bits = np.ascontiguousarray(b_bits, dtype=np.uint32)
    M, N = a_bits.shape[0], b_bits.shape[0]
    D = np.empty((M, N), dtype=np.int32)
    _load().oracle_int_dot(_ptr(a_bits), a_bits.shape[1], _ptr(b_bits), b_bits.shape[1], M, N, K, _ptr(D))
    return D


def binary_weight_gemm(A, b_bits, b_s, beta_w, want_T: bool = False):
    A = _f32_rows(A)
    b_bits = np.ascontiguousarray(b_bits, dtype=np.uint32)
    b_s = np.ascontiguousarray(b_s, dtype=np.float32)
    M, K = A.shape
    N = b_bits.shape[0]
    out = np.empty((M, N), dtype=np.float64)
    T = np.empty((M, N), dtype=np.float64) if want_T else None
    _load().oracle_binary_weight_gemm(_ptr(A), K, _ptr(b_bits), b_bits.shape[1], _ptr(b_s), b_s.shape[1],
                                      beta_w, M, N, K, _ptr(out), _ptr(T) if want_T else None)
    return (out, T) if want_T else out


def hbmm_dense(A, B, beta_a: int, beta_w: int) -> np.ndarray:
    """Dense path: materialise delta (.) Sign(.) for both rows x K operands, then the plain
    double-precision product (Eq. 2, Eq. 4 and the definition of a matrix product)."""
    return dense_f64_gemm(materialize(A, beta_a), materialize(B, beta_w))


def hbmm_popcount(A, B, beta_a: int, beta_w: int, want_T: bool = False):
    """Integer path: scales + packed signs + Eq. 7 (both operands rows x K, beta >= 2 each;
    for beta_a == 1 use :func:`binary_weight_gemm`)."""
    A, B = _f32_rows(A), _f32_rows(B)
    return popcount_gemm(sign_pack(A), block_scales(A, beta_a), beta_a,
                         sign_pack(B), block_scales(B, beta_w), beta_w, A.shape[1], want_T)


def binarize_backward(x, g, beta: int, want_T: bool = False):
    """Eq. 6 (with the straight-through estimator of Eq. 5): gradient w.r.t. x of delta (.) Sign(x)
    given the gradient g w.r.t. the binarised tensor; rows x K, segments along K."""
    x, g = _f32_rows(x), _f32_rows(g)
    if x.shape != g.shape:
        raise ValueError("x and g must have the same shape")
    rows, K = x.shape
    gx = np.empty((rows, K), dtype=np.float64)
    T = np.empty((rows, K), dtype=np.float64) if want_T else None
    _load().oracle_binarize_backward(_ptr(x), _ptr(g), rows, K, K, K, beta, _ptr(gx), _ptr(T) if want_T else None)
    return (gx, T) if want_T else gx


def conv_out_size(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def materialize_activations(A, beta_a: int) -> np.ndarray:
    """Eq. 3-4 for an activation tensor B x C x H x W (W, the width index y of Eq. 3, contiguous):
    delta over segments of beta_a along the width of every row of every channel, times Sign(A)."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B, C, H, W = A.shape
    # (the paper only asks beta_a <= w_in: when beta_a does not divide the width, the last segment of every
    # row is the shorter remainder and its delta the mean over its own length, as for any other operand)
    return materialize(A.reshape(B * C * H, W), beta_a).reshape(B, C, H, W)


def materialize_filters(Wf, beta_w: int) -> np.ndarray:
    """Eq. 1-2 for filters N x C x KH x KW: each filter flattened to C*KH*KW, segments of beta_w."""
    Wf = np.ascontiguousarray(Wf, dtype=np.float32)
    N = Wf.shape[0]
    return materialize(Wf.reshape(N, -1), beta_w).reshape(Wf.shape)


def conv2d_f64(At: np.ndarray, Wt: np.ndarray, stride: int, pad: int, want_T: bool = False):
    """Zero-padded convolution (cross-correlation) of materialised tensors, in double."""
    At = np.ascontiguousarray(At, dtype=np.float64)
    Wt = np.ascontiguousarray(Wt, dtype=np.float64)
    B, C, H, W = At.shape
    N, C2, KH, KW = Wt.shape
    if C != C2:
        raise ValueError("channel mismatch")
    OH, OW = conv_out_size(H, KH, stride, pad), conv_out_size(W, KW, stride, pad)
    out = np.empty((B, N, OH, OW), dtype=np.float64)
    T = np.empty_like(out) if want_T else None
    _load().oracle_conv2d_f64(_ptr(At), _ptr(Wt), B, C, H, W, N, KH, KW, stride, pad, _ptr(out),
                              _ptr(T) if want_T else None)
    return (out, T) if want_T else out


def hbmm_conv2d(A, Wf, beta_a: int, beta_w: int, stride: int = 1, pad: int = 0, want_T: bool = False):
    """A convolution layer of a HadaNet: activations binarised by Eq. 3-4, filters by Eq. 1-2, then
    the plain convolution of the two materialised tensors."""
    return conv2d_f64(materialize_activations(A, beta_a), materialize_filters(Wf, beta_w), stride, pad, want_T)
