"""Thin binding over ``libhbmm.so``: argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module allocates outputs with
torch (device memory and streams are the only things torch is used for), forwards raw device
pointers and the current HIP stream, and raises on a non-zero return code.  There is no CPU
fallback: if the library is missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libhbmm.so"

OK, EINVAL, EUNSUPPORTED, ELAUNCH = 0, -1, -2, -3
ALGO_POPCOUNT, ALGO_MFMA_I8, ALGO_MFMA_FP4, ALGO_MFMA_FP8, ALGO_FASTEST = 0, 1, 2, 3, -1

EXPORTS = (
    "hbmm_strerror", "hbmm_num_blocks", "hbmm_packed_ld_words", "hbmm_quantize_pack", "hbmm_gemm",
    "hbmm_gemm_int", "hbmm_dense_ref_gemm", "hbmm_binarize_backward", "hbmm_gemm_fused",
    "hbmm_quantize_pack_tensor", "hbmm_conv2d", "hbmm_binarize_backward_tensor",
    "hbmm_conv_filter_pieces_bytes", "hbmm_conv_prepare_filters", "hbmm_conv2d_prepared", "hbmm_probe_mfma_rate",
    "hbmm_quantize_pack_activations",
)


class HbmmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


def _load() -> C.CDLL:
    if not LIB_PATH.exists():
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1905_10759_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(str(LIB_PATH))
    i64, i32, p = C.c_int64, C.c_int32, C.c_void_p
    lib.hbmm_strerror.restype = C.c_char_p
    lib.hbmm_strerror.argtypes = [C.c_int]
    lib.hbmm_num_blocks.restype = i64
    lib.hbmm_num_blocks.argtypes = [i64, i32]
    lib.hbmm_packed_ld_words.restype = i64
    lib.hbmm_packed_ld_words.argtypes = [i64]
    lib.hbmm_quantize_pack.restype = C.c_int
    lib.hbmm_quantize_pack.argtypes = [p, i64, i64, i64, i32, i32, p, i64, p, i64, p]
    lib.hbmm_gemm.restype = C.c_int
    lib.hbmm_gemm.argtypes = [p, p, i64, i64, i32, p, p, i64, i64, i32, i64, i64, i64, p, i64, i32, p]
    lib.hbmm_gemm_int.restype = C.c_int
    lib.hbmm_gemm_int.argtypes = [p, i64, p, i64, i64, i64, i64, p, i64, p]
    lib.hbmm_gemm_fused.restype = C.c_int
    lib.hbmm_gemm_fused.argtypes = [p, i64, i32, p, p, i64, i64, i32, i64, i64, i64, p, i64, p]
    lib.hbmm_quantize_pack_tensor.restype = C.c_int
    lib.hbmm_quantize_pack_tensor.argtypes = [p, i64, i32, p, p, p]
    lib.hbmm_binarize_backward_tensor.restype = C.c_int
    lib.hbmm_binarize_backward_tensor.argtypes = [p, p, i64, i32, p, p]
    lib.hbmm_conv2d.restype = C.c_int
    lib.hbmm_conv2d.argtypes = [p, p, i32, p, p, i64, i64, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, i32, p]
    lib.hbmm_conv_filter_pieces_bytes.restype = i64
    lib.hbmm_conv_filter_pieces_bytes.argtypes = [i64, i64, i32, i32, i32]
    lib.hbmm_conv_prepare_filters.restype = C.c_int
    lib.hbmm_conv_prepare_filters.argtypes = [p, p, i64, i64, i32, i64, i64, i32, i32, i32, p, p]
    lib.hbmm_conv2d_prepared.restype = C.c_int
    lib.hbmm_conv2d_prepared.argtypes = [p, p, i32, p, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, p]
    lib.hbmm_quantize_pack_activations.restype = C.c_int
    lib.hbmm_quantize_pack_activations.argtypes = [p, i64, i64, i32, p, p, p]
    lib.hbmm_probe_mfma_rate.restype = C.c_int
    lib.hbmm_probe_mfma_rate.argtypes = [i32, i32, p, p]
    lib.hbmm_binarize_backward.restype = C.c_int
    lib.hbmm_binarize_backward.argtypes = [p, p, i64, i64, i64, i64, i32, p, i64, p]
    lib.hbmm_dense_ref_gemm.restype = C.c_int
    lib.hbmm_dense_ref_gemm.argtypes = [p, i64, p, i64, i32, i64, i64, i64, p, i64, p]
    return lib


lib = _load()


def strerror(code: int) -> str:
    return lib.hbmm_strerror(int(code)).decode()


def num_blocks(K: int, beta: int) -> int:
    return int(lib.hbmm_num_blocks(K, beta))


def packed_ld_words(K: int) -> int:
    return int(lib.hbmm_packed_ld_words(K))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise HbmmError(rc, where)


def _dev(t: torch.Tensor, dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype:
        raise TypeError(f"{name}: expected a {dtype} device tensor")


def _rows_view(t: torch.Tensor, name: str):
    """(rows, cols, leading dimension) of a 2-D tensor whose rows the library can walk: unit inner
    stride, rows that do not overlap.  The C ABI sees pointers and sizes only, so what it cannot check
    -- that the memory behind a pointer has the shape the sizes claim -- is checked here."""
    if t.dim() != 2:
        raise ValueError(f"{name}: expected a 2-D tensor, got {t.dim()}-D")
    rows, cols = t.shape
    if cols > 1 and t.stride(1) != 1:
        raise ValueError(f"{name}: the inner stride must be 1")
    ld = t.stride(0) if rows > 1 else max(cols, 1)
    if rows > 1 and ld < cols:
        raise ValueError(f"{name}: rows overlap (stride {ld} < {cols} columns)")
    return rows, cols, ld


def check_out(out: torch.Tensor, shape, name: str = "out") -> int:
    """A caller-supplied output matrix: exact shape, unit inner stride; returns its leading dimension."""
    rows, cols, ld = _rows_view(out, name)
    if (rows, cols) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(out.shape)} where {tuple(shape)} is written")
    return ld


def check_gemm_operand(bits, scales, beta: int, K: int, name: str):
    """One operand of hbmm_gemm as tensors: packed (bits rows x >= packed_ld_words(K) words, scales
    rows x >= K / beta) or, with beta == 1, unquantised (bits None, scales = the rows x K matrix).
    Returns (rows, ldw, lds)."""
    rows, cols, lds = _rows_view(scales, name + "_scales")
    if beta == 1:
        if bits is not None:
            raise ValueError(f"{name}: an unquantised operand (beta = 1) takes bits=None")
        if cols < K:
            raise ValueError(f"{name}: {cols} columns for K = {K}")
        return rows, 0, lds
    if bits is None:
        raise ValueError(f"{name}_bits missing (beta = {beta})")
    brows, bcols, ldw = _rows_view(bits, name + "_bits")
    if brows != rows:
        raise ValueError(f"{name}: {brows} rows of bits but {rows} rows of scales")
    if bcols < packed_ld_words(K):
        raise ValueError(f"{name}_bits: {bcols} words per row, K = {K} needs {packed_ld_words(K)}")
    if beta > 1 and cols < num_blocks(K, beta):
        raise ValueError(f"{name}_scales: {cols} scales per row, K = {K} with beta = {beta} needs {num_blocks(K, beta)}")
    return rows, ldw, lds


def quantize_pack(x: torch.Tensor, beta: int, layout: int = 0, bits: torch.Tensor | None = None,
                  scales: torch.Tensor | None = None):
    """hbmm_quantize_pack.  x: fp32 device matrix; layout 0 = rows x K, layout 1 = K x rows.
    Returns (bits int32[rows, ldw] holding the uint32 words, scales fp32[rows, nb])."""
    _dev(x, torch.float32, "x")
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D matrix with unit inner stride")
    rows, K = (x.shape[0], x.shape[1]) if layout == 0 else (x.shape[1], x.shape[0])
    ldx = x.stride(0) if x.shape[0] > 1 else x.shape[1]
    ldw, nb = packed_ld_words(K), num_blocks(K, beta)
    if bits is None:
        bits = torch.empty((rows, ldw), dtype=torch.int32, device=x.device)
    if scales is None:
        scales = torch.empty((rows, nb), dtype=torch.float32, device=x.device)
    _dev(bits, torch.int32, "bits")
    _dev(scales, torch.float32, "scales")
    brows, bcols, ldw_out = _rows_view(bits, "bits")
    srows, scols, lds_out = _rows_view(scales, "scales")
    if brows != rows or srows != rows or bcols < ldw or scols < nb:
        raise ValueError(f"bits / scales: need {rows} rows of >= {ldw} words and >= {nb} scales")
    rc = lib.hbmm_quantize_pack(x.data_ptr(), rows, K, ldx, layout, beta, bits.data_ptr(), ldw_out,
                                scales.data_ptr(), lds_out, _stream())
    _check(rc, "hbmm_quantize_pack")
    return bits, scales


def gemm(a_bits, a_scales, beta_a: int, b_bits, b_scales, beta_w: int, K: int, algo: int = ALGO_POPCOUNT,
         out: torch.Tensor | None = None) -> torch.Tensor:
    """hbmm_gemm.  An operand with beta == 1 is passed unquantised: bits=None and scales = the raw
    fp32 matrix (rows x K)."""
    _dev(b_scales, torch.float32, "b_scales")
    _dev(a_scales, torch.float32, "a_scales")
    for bits, name in ((a_bits, "a_bits"), (b_bits, "b_bits")):
        if bits is not None:
            _dev(bits, torch.int32, name)
    M, ldw_a, lds_a = check_gemm_operand(a_bits, a_scales, beta_a, K, "a")
    N, ldw_b, lds_b = check_gemm_operand(b_bits, b_scales, beta_w, K, "b")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scales.device)
    _dev(out, torch.float32, "out")
    ldc = check_out(out, (M, N))
    rc = lib.hbmm_gemm(a_bits.data_ptr() if a_bits is not None else 0, a_scales.data_ptr(), ldw_a, lds_a, beta_a,
                       b_bits.data_ptr() if b_bits is not None else 0, b_scales.data_ptr(), ldw_b, lds_b, beta_w,
                       M, N, K, out.data_ptr(), ldc, algo, _stream())
    _check(rc, "hbmm_gemm")
    return out


def gemm_int(a_bits, b_bits, K: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """hbmm_gemm_int: D[m, n] = K - 2 * hamming(a_row, b_row), int32."""
    _dev(a_bits, torch.int32, "a_bits")
    _dev(b_bits, torch.int32, "b_bits")
    (M, wa, ldw_a), (N, wb, ldw_b) = _rows_view(a_bits, "a_bits"), _rows_view(b_bits, "b_bits")
    if min(wa, wb) < packed_ld_words(K):
        raise ValueError(f"bits: {min(wa, wb)} words per row, K = {K} needs {packed_ld_words(K)}")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=a_bits.device)
    _dev(out, torch.int32, "out")
    ldd = check_out(out, (M, N))
    rc = lib.hbmm_gemm_int(a_bits.data_ptr(), ldw_a, b_bits.data_ptr(), ldw_b, M, N, K, out.data_ptr(), ldd, _stream())
    _check(rc, "hbmm_gemm_int")
    return out


def dense_ref_gemm(A: torch.Tensor, B: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """hbmm_dense_ref_gemm: C = A . B^T, A M x K, B N x K, fp32 or bf16 operands, fp32 result."""
    if A.dtype != B.dtype or A.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("A and B must both be fp32 or both bf16")
    _dev(A, A.dtype, "A")
    _dev(B, A.dtype, "B")
    (M, K, lda), (N, Kb, ldb) = _rows_view(A, "A"), _rows_view(B, "B")
    if Kb != K:
        raise ValueError(f"A has K = {K} columns, B has {Kb}")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _dev(out, torch.float32, "out")
    ldc = check_out(out, (M, N))
    rc = lib.hbmm_dense_ref_gemm(A.data_ptr(), lda, B.data_ptr(), ldb, 0 if A.dtype == torch.float32 else 1,
                                 M, N, K, out.data_ptr(), ldc, _stream())
    _check(rc, "hbmm_dense_ref_gemm")
    return out


def binarize_backward(x: torch.Tensor, grad_out: torch.Tensor, beta: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """hbmm_binarize_backward: gradient w.r.t. x of delta (.) Sign(x) (Eq. 6 with the STE of Eq. 5)."""
    _dev(x, torch.float32, "x")
    _dev(grad_out, torch.float32, "grad_out")
    if x.dim() != 2 or x.shape != grad_out.shape or x.stride(1) != 1 or grad_out.stride(1) != 1:
        raise ValueError("x and grad_out must be matching 2-D matrices with unit inner stride")
    rows, K = x.shape
    if out is None:
        out = torch.empty((rows, K), dtype=torch.float32, device=x.device)
    _dev(out, torch.float32, "out")
    check_out(out, (rows, K))
    ld = lambda t: t.stride(0) if rows > 1 else K
    rc = lib.hbmm_binarize_backward(x.data_ptr(), grad_out.data_ptr(), rows, K, ld(x), ld(grad_out), beta,
                                    out.data_ptr(), ld(out), _stream())
    _check(rc, "hbmm_binarize_backward")
    return out


def gemm_fused(A: torch.Tensor, beta_a: int, b_bits, b_scales, beta_w: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """hbmm_gemm_fused: quantize_pack(A) + gemm in one kernel (N <= 128), A given as raw fp32 M x K."""
    _dev(A, torch.float32, "A")
    _dev(b_bits, torch.int32, "b_bits")
    _dev(b_scales, torch.float32, "b_scales")
    M, K, lda = _rows_view(A, "A")
    N, ldw_b, lds_b = check_gemm_operand(b_bits, b_scales, beta_w, K, "b")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _dev(out, torch.float32, "out")
    ldc = check_out(out, (M, N))
    rc = lib.hbmm_gemm_fused(A.data_ptr(), lda, beta_a, b_bits.data_ptr(), b_scales.data_ptr(), ldw_b, lds_b, beta_w,
                             M, N, K, out.data_ptr(), ldc, _stream())
    _check(rc, "hbmm_gemm_fused")
    return out


def quantize_pack_tensor(x: torch.Tensor, beta: int, bits: torch.Tensor | None = None,
                         scales: torch.Tensor | None = None):
    """hbmm_quantize_pack_tensor: a contiguous fp32 tensor -> (bits int32[count / 32], scales fp32[count / beta]);
    existing output tensors of those sizes may be passed in."""
    _dev(x, torch.float32, "x")
    if not x.is_contiguous():
        raise ValueError("x must be contiguous")
    count = x.numel()
    if bits is None:
        bits = torch.empty((count // 32,), dtype=torch.int32, device=x.device)
    if scales is None:
        scales = torch.empty((count // max(beta, 1),), dtype=torch.float32, device=x.device)
    _dev(bits, torch.int32, "bits")
    _dev(scales, torch.float32, "scales")
    if bits.numel() < count // 32 or scales.numel() < count // max(beta, 1) or not bits.is_contiguous() or not scales.is_contiguous():
        raise ValueError("bits / scales too small or not contiguous")
    rc = lib.hbmm_quantize_pack_tensor(x.data_ptr(), count, beta, bits.data_ptr(), scales.data_ptr(), _stream())
    _check(rc, "hbmm_quantize_pack_tensor")
    return bits, scales


def conv2d(a_bits, a_scales, beta_a: int, shape, w_bits, w_scales, beta_w: int, kernel, stride: int = 1,
           pad: int = 0, out: torch.Tensor | None = None, algo: int = 0) -> torch.Tensor:
    """hbmm_conv2d: activations (B, C, H, W) = `shape` packed by quantize_pack_tensor (or, with
    beta_a = 1, a_bits=None and a_scales = the contiguous fp32 tensor), filters (N, C, KH, KW) packed
    by quantize_pack on the N x (C*KH*KW) matrix; `kernel` = (KH, KW)."""
    if a_bits is not None:
        _dev(a_bits, torch.int32, "a_bits")
    _dev(a_scales, torch.float32, "a_scales")
    _dev(w_bits, torch.int32, "w_bits")
    _dev(w_scales, torch.float32, "w_scales")
    B, Cc, H, W = (int(v) for v in shape)
    KH, KW = (int(v) for v in kernel)
    count = B * Cc * H * W
    N, ldw_w, lds_w = check_gemm_operand(w_bits, w_scales, beta_w, Cc * KH * KW, "w")
    if not a_scales.is_contiguous() or (a_bits is not None and not a_bits.is_contiguous()):
        raise ValueError("the packed activation tensor must be contiguous")
    if a_scales.numel() < count // max(beta_a, 1) or (a_bits is not None and a_bits.numel() < count // 32):
        raise ValueError(f"activations: too few words / scales for a tensor of {count} elements")
    OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    if out is None:
        out = torch.empty((B, N, OH, OW), dtype=torch.float32, device=a_scales.device)
    _dev(out, torch.float32, "out")
    if tuple(out.shape) != (B, N, OH, OW) or not out.is_contiguous():
        raise ValueError(f"out: a contiguous tensor of shape {(B, N, OH, OW)} is written")
    rc = lib.hbmm_conv2d(a_bits.data_ptr() if a_bits is not None else 0, a_scales.data_ptr(), beta_a, w_bits.data_ptr(),
                         w_scales.data_ptr(), ldw_w, lds_w, beta_w, B, Cc, H, W, N, KH, KW,
                         stride, pad, out.data_ptr(), algo, _stream())
    _check(rc, "hbmm_conv2d")
    return out


def quantize_pack_activations(x: torch.Tensor, beta: int, bits: torch.Tensor | None = None,
                              scales: torch.Tensor | None = None):
    """hbmm_quantize_pack_activations: a contiguous fp32 tensor whose last axis is the width W ->
    (bits int32[ceil(count / 32)], scales fp32[count / W * ceil(W / beta)]); segments of beta along the width, anew in
    every row, the last one of a row shorter when beta does not divide W."""
    _dev(x, torch.float32, "x")
    if not x.is_contiguous() or x.dim() < 1:
        raise ValueError("x must be a contiguous tensor")
    count, W = x.numel(), int(x.shape[-1])
    rows = count // max(W, 1)
    nseg = -(-W // max(beta, 1))
    if bits is None:
        bits = torch.empty(((count + 31) // 32,), dtype=torch.int32, device=x.device)
    if scales is None:
        scales = torch.empty((rows * nseg,), dtype=torch.float32, device=x.device)
    _dev(bits, torch.int32, "bits")
    _dev(scales, torch.float32, "scales")
    if bits.numel() < (count + 31) // 32 or scales.numel() < rows * nseg or not bits.is_contiguous() or not scales.is_contiguous():
        raise ValueError(f"bits / scales: need {(count + 31) // 32} words and {rows * nseg} scales, contiguous")
    rc = lib.hbmm_quantize_pack_activations(x.data_ptr(), rows, W, beta, bits.data_ptr(), scales.data_ptr(), _stream())
    _check(rc, "hbmm_quantize_pack_activations")
    return bits, scales


PIECES_BF16X3, PIECES_F16X2 = 0, 1   # `form` of the prepared convolution: exact three-piece split / two fp16 pieces


def conv_filter_pieces_bytes(N: int, C: int, KH: int, KW: int, form: int = PIECES_BF16X3) -> int:
    return int(lib.hbmm_conv_filter_pieces_bytes(N, C, KH, KW, form))


def conv_prepare_filters(w_bits, w_scales, beta_w: int, C: int, kernel, pieces: torch.Tensor | None = None,
                         form: int = PIECES_BF16X3) -> torch.Tensor:
    """hbmm_conv_prepare_filters: filters (N, C, KH, KW) packed by quantize_pack on the N x (C*KH*KW) matrix
    (or, with beta_w = 1, w_bits=None and w_scales = that fp32 matrix) -> the prepared form, a flat uint8
    device tensor of conv_filter_pieces_bytes(N, C, KH, KW, form) bytes."""
    if w_bits is not None:
        _dev(w_bits, torch.int32, "w_bits")
    _dev(w_scales, torch.float32, "w_scales")
    KH, KW = (int(v) for v in kernel)
    N, ldw_w, lds_w = check_gemm_operand(w_bits, w_scales, beta_w, C * KH * KW, "w")
    if form not in (PIECES_BF16X3, PIECES_F16X2):
        raise ValueError(f"form: {form} is neither PIECES_BF16X3 nor PIECES_F16X2")
    nbytes = conv_filter_pieces_bytes(N, C, KH, KW, form)
    if nbytes == 0 and N > 0 and C > 0:
        raise ValueError(f"filters: unsupported shape {(N, C, KH, KW)}")
    if pieces is None:
        pieces = torch.empty((nbytes,), dtype=torch.uint8, device=w_scales.device)
    _dev(pieces, torch.uint8, "pieces")
    if pieces.dim() != 1 or pieces.numel() < nbytes or not pieces.is_contiguous():
        raise ValueError(f"pieces: a flat contiguous tensor of at least {nbytes} bytes is written")
    rc = lib.hbmm_conv_prepare_filters(w_bits.data_ptr() if w_bits is not None else 0, w_scales.data_ptr(), ldw_w, lds_w,
                                       beta_w, N, C, KH, KW, form, pieces.data_ptr(), _stream())
    _check(rc, "hbmm_conv_prepare_filters")
    return pieces


def conv2d_prepared(a_bits, a_scales, beta_a: int, shape, pieces: torch.Tensor, N: int, kernel, stride: int = 1,
                    pad: int = 0, out: torch.Tensor | None = None, form: int = PIECES_BF16X3) -> torch.Tensor:
    """hbmm_conv2d_prepared: activations as for conv2d, filters as written by conv_prepare_filters for the
    same N, C = shape[1], kernel = (KH, KW) and form."""
    if a_bits is not None:
        _dev(a_bits, torch.int32, "a_bits")
    _dev(a_scales, torch.float32, "a_scales")
    _dev(pieces, torch.uint8, "pieces")
    B, Cc, H, W = (int(v) for v in shape)
    KH, KW = (int(v) for v in kernel)
    count = B * Cc * H * W
    if form not in (PIECES_BF16X3, PIECES_F16X2):
        raise ValueError(f"form: {form} is neither PIECES_BF16X3 nor PIECES_F16X2")
    if not pieces.is_contiguous() or pieces.numel() < conv_filter_pieces_bytes(N, Cc, KH, KW, form):
        raise ValueError(f"pieces: too few bytes for {N} filters of {(Cc, KH, KW)}")
    if not a_scales.is_contiguous() or (a_bits is not None and not a_bits.is_contiguous()):
        raise ValueError("the packed activation tensor must be contiguous")
    nscales = B * Cc * H * -(-W // max(beta_a, 1))
    if a_scales.numel() < nscales or (a_bits is not None and a_bits.numel() < (count + 31) // 32):
        raise ValueError(f"activations: too few words / scales for a tensor of {count} elements ({nscales} scales)")
    OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    if out is None:
        out = torch.empty((B, N, OH, OW), dtype=torch.float32, device=a_scales.device)
    _dev(out, torch.float32, "out")
    if tuple(out.shape) != (B, N, OH, OW) or not out.is_contiguous():
        raise ValueError(f"out: a contiguous tensor of shape {(B, N, OH, OW)} is written")
    rc = lib.hbmm_conv2d_prepared(a_bits.data_ptr() if a_bits is not None else 0, a_scales.data_ptr(), beta_a,
                                  pieces.data_ptr(), form, B, Cc, H, W, N, KH, KW, stride, pad, out.data_ptr(), _stream())
    _check(rc, "hbmm_conv2d_prepared")
    return out


def probe_mfma_rate(steps: int = 2000, blocks: int = 256) -> float:
    """hbmm_probe_mfma_rate, timed: the bf16 matrix-core rate (TFLOP/s) this device sustains on random register
    operands with `blocks` workgroups of eight waves (256 = one per compute unit).  A diagnostic."""
    sink = torch.empty((blocks * 512,), dtype=torch.float32, device="cuda")
    _check(lib.hbmm_probe_mfma_rate(steps, blocks, sink.data_ptr(), _stream()), "hbmm_probe_mfma_rate")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _check(lib.hbmm_probe_mfma_rate(steps, blocks, sink.data_ptr(), _stream()), "hbmm_probe_mfma_rate")
    e1.record()
    torch.cuda.synchronize()
    return steps * 24.0 * 8 * blocks * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12


def binarize_backward_tensor(x: torch.Tensor, grad_out: torch.Tensor, beta: int) -> torch.Tensor:
    """hbmm_binarize_backward_tensor: contiguous tensors of any shape, segments of beta consecutive elements."""
    _dev(x, torch.float32, "x")
    _dev(grad_out, torch.float32, "grad_out")
    if x.shape != grad_out.shape or not x.is_contiguous() or not grad_out.is_contiguous():
        raise ValueError("x and grad_out must be contiguous tensors of the same shape")
    out = torch.empty_like(x)
    rc = lib.hbmm_binarize_backward_tensor(x.data_ptr(), grad_out.data_ptr(), x.numel(), beta, out.data_ptr(), _stream())
    _check(rc, "hbmm_binarize_backward_tensor")
    return out
