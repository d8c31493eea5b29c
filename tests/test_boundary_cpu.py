"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
its size helpers agree with the layout contract, and argument validation rejects bad calls
before anything is launched (so these run without a GPU)."""
from __future__ import annotations

import ctypes as C
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
LIB = ROOT / "paper_1905_10759_amd" / "libhbmm.so"


@pytest.fixture(scope="module")
def lib():
    if not LIB.exists():
        from paper_1905_10759_amd import build
        build.build()
    return C.CDLL(str(LIB))


def declared_symbols():
    text = (ROOT / "include" / "hbmm.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hbmm_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"hbmm_quantize_pack", "hbmm_gemm", "hbmm_dense_ref_gemm", "hbmm_gemm_int"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_lists_same_symbols():
    src = (ROOT / "paper_1905_10759_amd" / "hbmm.py").read_text()
    for name in declared_symbols():
        assert f'"{name}"' in src, name


def test_size_helpers(lib):
    lib.hbmm_num_blocks.restype = C.c_int64
    lib.hbmm_num_blocks.argtypes = [C.c_int64, C.c_int32]
    lib.hbmm_packed_ld_words.restype = C.c_int64
    lib.hbmm_packed_ld_words.argtypes = [C.c_int64]
    assert lib.hbmm_num_blocks(512, 32) == 16
    assert lib.hbmm_num_blocks(513, 32) == 17
    assert lib.hbmm_num_blocks(10, 0) == 0
    assert [lib.hbmm_packed_ld_words(k) for k in (0, 1, 32, 33, 128, 129, 576, 8192)] == [0, 4, 4, 4, 4, 8, 20, 256]


def test_strerror(lib):
    lib.hbmm_strerror.restype = C.c_char_p
    assert lib.hbmm_strerror(0) == b"ok"
    for code in (-1, -2, -3, 7):
        assert len(lib.hbmm_strerror(code)) > 3


def test_validation_rejects_before_launch(lib):
    i64, i32, p = C.c_int64, C.c_int32, C.c_void_p
    qp = lib.hbmm_quantize_pack
    qp.argtypes = [p, i64, i64, i64, i32, i32, p, i64, p, i64, p]
    fake = 0x1000  # 16-byte aligned, never dereferenced: every call below fails validation first
    assert qp(None, 4, 64, 64, 0, 32, fake, 4, fake, 2, None) == -1          # null x
    assert qp(fake, 4, 64, 64, 0, 512, fake, 4, fake, 2, None) == -2         # beta above 256
    assert qp(fake, 4, 64, 64, 0, 1, fake, 4, fake, 64, None) == -2          # beta = 1: nothing to pack
    assert qp(fake, 4, 96, 96, 0, 64, fake, 4, fake, 1, None) == -1          # lds < ceil(K / beta) (last segment shorter)
    assert qp(fake, 4, 100, 100, 0, 7, fake, 4, fake, 14, None) == -1        # the same with a segment length of 7
    assert qp(fake, 4, 64, 32, 0, 32, fake, 4, fake, 2, None) == -1          # ldx < K
    assert qp(fake, 4, 64, 64, 0, 32, fake, 2, fake, 2, None) == -1          # ldw too small
    assert qp(fake, 4, 64, 64, 0, 32, fake, 6, fake, 2, None) == -1          # ldw not a multiple of 4
    assert qp(fake, 4, 64, 64, 0, 32, fake, 4, fake, 1, None) == -1          # lds too small
    assert qp(fake + 4, 4, 64, 64, 0, 32, fake, 4, fake, 2, None) == -1      # misaligned
    assert qp(fake, 4, 64, 64, 2, 32, fake, 4, fake, 2, None) == -1          # bad layout
    assert qp(fake, -1, 64, 64, 0, 32, fake, 4, fake, 2, None) == -1
    assert qp(None, 0, 64, 64, 0, 32, None, 4, None, 2, None) == 0           # empty is a no-op

    g = lib.hbmm_gemm
    g.argtypes = [p, p, i64, i64, i32, p, p, i64, i64, i32, i64, i64, i64, p, i64, i32, p]
    ok = dict(a=fake, sa=fake, ldwa=4, ldsa=2, ba=32, b=fake, sb=fake, ldwb=4, ldsb=2, bw=32, M=8, N=8, K=64,
              C=fake, ldc=8, algo=0)

    def call(**kw):
        a = {**ok, **kw}
        return g(a["a"], a["sa"], a["ldwa"], a["ldsa"], a["ba"], a["b"], a["sb"], a["ldwb"], a["ldsb"], a["bw"],
                 a["M"], a["N"], a["K"], a["C"], a["ldc"], a["algo"], None)

    assert call(C=None) == -1
    assert call(ldc=4) == -1
    assert call(ba=48, algo=1) == -2              # not a power of two: the general kernel only (algo 0 or -1)
    assert call(ba=300) == -2
    assert call(ba=48, K=1 << 24, ldsa=1 << 20, ldsb=1 << 20, ldwa=1 << 20, ldwb=1 << 20) == -2   # general kernel: K < 2^24
    assert call(ba=48, ldsa=1) == -1              # lds_a < ceil(K / beta_a)
    assert call(bw=512) == -2
    assert call(ba=1, a=None, bw=1, b=None, ldsa=64, ldsb=64) == -2   # two unquantised operands: a plain dense product
    assert call(ba=16, ldsa=4, algo=1) == -2      # the int8 comparison variant needs word-sized segments
    assert call(K=48, ba=16, bw=16, ldsa=3, ldsb=3, algo=3) == -2   # K not a multiple of 32: general kernel only
    assert call(ba=16, ldsa=3) == -1              # lds_a < K / beta_a
    assert call(algo=5) == -2
    assert call(K=96, ba=64, bw=32) == -1         # lds_b < ceil(K / beta_w)
    assert call(K=96, ba=64, bw=32, ldsb=3, algo=2) == -2   # a shorter last segment: general kernel only
    assert call(a=None) == -1
    assert call(ba=1, a=fake, ldsa=64) == -1      # beta_a = 1 takes raw A through a_scales, a_bits must be NULL
    assert call(ba=1, a=None, ldsa=8) == -1       # lds_a is then the leading dimension of A (>= K)
    assert call(ldwa=2) == -1
    assert call(M=0) == 0 and call(N=0) == 0

    gi = lib.hbmm_gemm_int
    gi.argtypes = [p, i64, p, i64, i64, i64, i64, p, i64, p]
    assert gi(None, 4, fake, 4, 8, 8, 64, fake, 8, None) == -1
    assert gi(fake, 4, fake, 4, 8, 8, 64, fake, 4, None) == -1
    assert gi(fake, 4, fake, 4, 0, 8, 64, fake, 8, None) == 0

    bw = lib.hbmm_binarize_backward
    bw.argtypes = [p, p, i64, i64, i64, i64, i32, p, i64, p]
    assert bw(fake, fake, 4, 64, 64, 64, 300, fake, 64, None) == -2    # beta above 256
    assert bw(fake, fake, 4, 64, 64, 64, 0, fake, 64, None) == -1
    assert bw(fake, None, 4, 64, 64, 64, 8, fake, 64, None) == -1
    assert bw(fake, fake, 4, 64, 32, 64, 8, fake, 64, None) == -1      # ldx < K
    assert bw(fake, fake, 0, 64, 64, 64, 8, fake, 64, None) == 0

    d = lib.hbmm_dense_ref_gemm
    d.argtypes = [p, i64, p, i64, i32, i64, i64, i64, p, i64, p]
    assert d(fake, 64, fake, 64, 3, 8, 8, 64, fake, 8, None) == -2
    assert d(None, 64, fake, 64, 0, 8, 8, 64, fake, 8, None) == -1
    assert d(fake, 32, fake, 64, 0, 8, 8, 64, fake, 8, None) == -1


def test_validation_of_the_fused_tensor_and_convolution_entry_points(lib):
    """Only calls that must fail (or are empty) before anything is launched: the pointers are fake."""
    i64, i32, p = C.c_int64, C.c_int32, C.c_void_p
    fake = 0x1000
    gf = lib.hbmm_gemm_fused
    gf.argtypes = [p, i64, i32, p, p, i64, i64, i32, i64, i64, i64, p, i64, p]
    assert gf(fake, 64, 32, fake, fake, 4, 2, 32, 8, 200, 64, fake, 200, None) == -2     # N > 128
    assert gf(fake, 64, 16, fake, fake, 4, 2, 32, 8, 8, 64, fake, 8, None) == -2         # beta_a < 32
    assert gf(fake, 62, 32, fake, fake, 4, 2, 32, 8, 8, 64, fake, 8, None) == -1         # lda < K
    assert gf(None, 64, 32, fake, fake, 4, 2, 32, 8, 8, 64, fake, 8, None) == -1
    assert gf(fake, 64, 32, fake, fake, 4, 2, 32, 0, 8, 64, fake, 8, None) == 0

    qt = lib.hbmm_quantize_pack_tensor
    qt.argtypes = [p, i64, i32, p, p, p]
    assert qt(fake, 120, 4, fake, fake, None) == -2          # not a multiple of 128
    assert qt(fake, 256, 3, fake, fake, None) == -2          # beta not a power of two
    assert qt(fake, 128, 256, fake, fake, None) == -2        # beta does not divide the 128-element view
    assert qt(None, 1024, 4, fake, fake, None) == -1
    assert qt(fake, -1, 4, fake, fake, None) == -1
    assert qt(None, 0, 4, None, None, None) == 0

    bt = lib.hbmm_binarize_backward_tensor
    bt.argtypes = [p, p, i64, i32, p, p]
    assert bt(fake, fake, 120, 4, fake, None) == -2
    assert bt(fake, fake, 1024, 3, fake, None) == -2
    assert bt(fake, None, 1024, 4, fake, None) == -1
    assert bt(None, None, 0, 4, None, None) == 0

    cv = lib.hbmm_conv2d
    cv.argtypes = [p, p, i32, p, p, i64, i64, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, i32, p]
    ok = dict(ab=fake, asc=fake, ba=4, wb=fake, ws=fake, ldw=12, lds=9, bw=32, B=1, C=32, H=8, W=8, N=8, KH=3, KW=3,
              stride=1, pad=1, out=fake, algo=0)

    def conv(**kw):
        a = {**ok, **kw}
        return cv(a["ab"], a["asc"], a["ba"], a["wb"], a["ws"], a["ldw"], a["lds"], a["bw"], a["B"], a["C"], a["H"],
                  a["W"], a["N"], a["KH"], a["KW"], a["stride"], a["pad"], a["out"], a["algo"], None)

    assert conv(ba=16) == -2                 # beta_a does not divide the width
    assert conv(bw=48) == -2                 # beta_w not a power of two
    assert conv(C=20) == -2                  # C*KH*KW not a multiple of 32
    assert conv(bw=64) == -2                 # 288 is not a multiple of 64
    assert conv(KH=7, KW=7, pad=3) == -2     # more than 32 taps
    assert conv(stride=0) == -1
    assert conv(algo=2) == -1
    assert conv(out=None) == -1
    assert conv(ab=None) == -1
    assert conv(lds=8) == -1                 # lds_w < K / beta_w
    assert conv(ldw=8) == -1                 # ldw_w < K / 32 rounded up to a multiple of 4
    assert conv(H=1, pad=0) == -1            # window larger than the padded input
    assert conv(B=0) == 0 and conv(N=0) == 0

    # the prepared-filter form
    nb = lib.hbmm_conv_filter_pieces_bytes
    nb.restype, nb.argtypes = i64, [i64, i64, i32, i32, i32]
    assert nb(128, 128, 3, 3, 0) == 128 * 128 * 9 * 6
    assert nb(40, 20, 3, 3, 0) == 64 * 32 * 9 * 6          # filters rounded up to 32, channels to 32
    assert nb(40, 20, 3, 3, 1) == 64 * 32 * 9 * 4 + 64 * 4   # two fp16 pieces and one exponent per filter
    assert nb(8, 8, 0, 3, 0) == 0 and nb(-1, 8, 3, 3, 0) == 0 and nb(8, 8, 40, 3, 0) == 0
    assert nb(8, 8, 3, 3, 2) == 0 and nb(8, 8, 3, 3, -1) == 0     # no such form
    pf_raw = lib.hbmm_conv_prepare_filters
    pf_raw.argtypes = [p, p, i64, i64, i32, i64, i64, i32, i32, i32, p, p]
    assert pf_raw(fake, fake, 12, 9, 32, 8, 32, 3, 3, 2, fake, None) == -2      # no such form
    assert pf_raw(fake, fake, 12, 9, 32, 8, 32, 3, 3, 1, None, None) == -1

    def pf(*a):
        return pf_raw(*a[:9], 0, *a[9:])
    assert pf(fake, fake, 12, 9, 32, 8, 32, 3, 3, None, None) == -1        # no output buffer
    assert pf(fake, fake, 12, 8, 32, 8, 32, 3, 3, fake, None) == -1        # lds_w < ceil(K / beta_w)
    assert pf(fake, fake, 12, 57, 5, 8, 32, 3, 3, fake, None) == -1        # beta_w = 5: 58 scales per filter
    assert pf(fake, fake, 8, 9, 32, 8, 32, 3, 3, fake, None) == -1         # ldw_w too small
    assert pf(fake, fake, 12, 288, 1, 8, 32, 3, 3, fake, None) == -1       # beta_w = 1 takes the filters through w_scales
    assert pf(None, fake, 12, 100, 1, 8, 32, 3, 3, fake, None) == -1       # ... with a leading dimension >= K
    assert pf(fake, fake, 12, 9, 300, 8, 32, 3, 3, fake, None) == -2       # beta_w above 256
    assert pf(fake, fake, 12, 9, 32, 8, 1 << 22, 3, 3, fake, None) == -2   # C*KH*KW beyond 2^24
    assert pf(None, None, 12, 9, 32, 0, 32, 3, 3, None, None) == 0
    qa = lib.hbmm_quantize_pack_activations
    qa.argtypes = [p, i64, i64, i32, p, p, p]
    assert qa(fake, 64, 7, 1, fake, fake, None) == -2          # beta = 1: nothing to pack
    assert qa(fake, 64, 7, 300, fake, fake, None) == -2
    assert qa(fake, 64, 7, 4, None, fake, None) == -1
    assert qa(fake + 4, 64, 7, 4, fake, fake, None) == -1      # misaligned
    assert qa(fake, 1 << 20, 1 << 20, 4, fake, fake, None) == -1   # more than 2^31 elements
    assert qa(None, 0, 7, 4, None, None, None) == 0
    cp = lib.hbmm_conv2d_prepared
    cp.argtypes = [p, p, i32, p, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, p]
    okp = dict(ab=fake, asc=fake, ba=4, pieces=fake, form=0, B=1, C=32, H=8, W=8, N=8, KH=3, KW=3, stride=1, pad=1, out=fake)

    def convp(**kw):
        a = {**okp, **kw}
        return cp(a["ab"], a["asc"], a["ba"], a["pieces"], a["form"], a["B"], a["C"], a["H"], a["W"], a["N"], a["KH"], a["KW"],
                  a["stride"], a["pad"], a["out"], None)

    assert convp(form=2) == -2 and convp(form=-1) == -2
    assert convp(form=1, pieces=None) == -1
    assert convp(ba=300) == -2               # beta_a above 256 (any other beta_a goes, also one that does not divide the width)
    assert convp(W=200, pad=1) == -2         # an output row of 200 positions does not fit a tile
    assert convp(W=128, KH=5, KW=5, pad=2) == -2   # the patch of one output row: 132 x 5 pixels
    assert convp(pieces=None) == -1
    assert convp(out=None) == -1
    assert convp(ab=None) == -1
    assert convp(ba=1) == -1                 # unquantised activations travel through a_scales, a_bits must be NULL
    assert convp(stride=0) == -1
    assert convp(H=1, pad=0) == -1
    assert convp(B=0) == 0 and convp(N=0) == 0


def test_compiled_gemm_keeps_inflight_scalar_registers_untouched():
    """The popcount GEMM waits for its asm-issued scalar loads by hand; the compiled ISA must not touch
    their destination registers before that wait (checked on freshly compiled gfx950 assembly)."""
    from paper_1905_10759_amd import check_isa
    assert check_isa.compile_and_check(verbose=False) == 0


def test_isa_checker_detects_a_planted_early_use(tmp_path):
    """The checker itself: a use of an in-flight register before the wait must be reported."""
    from paper_1905_10759_amd import check_isa
    good = """
\t;;#ASMSTART
\ts_load_dwordx2 s[4:5], s[0:1], s2
\t;;#ASMEND
\tv_xor_b32_e32 v1, s8, v2
\ts_waitcnt lgkmcnt(0)
\tv_xor_b32_e32 v1, s4, v2
"""
    bad = good.replace("v_xor_b32_e32 v1, s8, v2", "v_xor_b32_e32 v1, s5, v2")
    (tmp_path / "good.s").write_text(good)
    (tmp_path / "bad.s").write_text(bad)
    assert check_isa.check(str(tmp_path / "good.s"), verbose=False) == 0
    assert check_isa.check(str(tmp_path / "bad.s"), verbose=False) == 1


def test_binding_checks_what_the_c_abi_cannot_see():
    """The C ABI gets pointers and sizes; whether the memory behind a pointer has that shape only the
    binding can tell.  A mismatch must raise before any call is made (on the device it would be an
    out-of-bounds access, not an error code).  The checkers work on shapes and strides only, so CPU
    tensors serve."""
    import torch

    from paper_1905_10759_amd import hbmm

    K, beta = 128, 32
    bits = torch.zeros((6, 4), dtype=torch.int32)
    scales = torch.zeros((6, 4), dtype=torch.float32)
    assert hbmm.check_gemm_operand(bits, scales, beta, K, "a") == (6, 4, 4)
    wide = torch.zeros((6, 12), dtype=torch.float32)
    assert hbmm.check_gemm_operand(bits, wide[:, :4], beta, K, "a") == (6, 4, 12)          # a padded leading dimension is fine
    assert hbmm.check_gemm_operand(None, torch.zeros((6, K)), 1, K, "a") == (6, 0, K)       # unquantised operand
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits[:5], scales, beta, K, "a")                             # rows of bits != rows of scales
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits, scales, beta, 256, "a")                               # K needs 8 words and 8 scales per row
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits, scales[:, :3], beta, K, "a")                          # too few scales
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits, wide[:, ::3], beta, K, "a")                           # inner stride 3
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits, torch.zeros((6, K)), 1, K, "a")                       # beta = 1 takes no bits
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(None, torch.zeros((6, K - 1)), 1, K, "a")                   # unquantised operand narrower than K
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(None, scales, beta, K, "a")                                 # packed operand without bits
    with pytest.raises(ValueError):
        hbmm.check_gemm_operand(bits, torch.zeros((6, 4, 1)), beta, K, "a")                 # not a matrix

    out = torch.zeros((6, 9), dtype=torch.float32)
    assert hbmm.check_out(out, (6, 9)) == 9
    assert hbmm.check_out(torch.zeros((6, 20))[:, :9], (6, 9)) == 20
    with pytest.raises(ValueError):
        hbmm.check_out(out, (6, 10))                                                        # wrong shape
    with pytest.raises(ValueError):
        hbmm.check_out(out.t(), (9, 6))                                                     # transposed view: inner stride 6
    with pytest.raises(ValueError):
        hbmm.check_out(torch.zeros(9).expand(6, 9), (6, 9))                                 # rows overlap


def test_binding_entry_points_validate_before_the_call(monkeypatch):
    """gemm / gemm_fused / dense_ref_gemm / conv2d run the checks above on their arguments: with the
    device-tensor test switched off, mismatched CPU tensors must raise ValueError and never reach
    the library."""
    import torch

    from paper_1905_10759_amd import hbmm

    monkeypatch.setattr(hbmm, "_dev", lambda t, dtype, name: None)
    monkeypatch.setattr(hbmm, "_stream", lambda: 0)

    class Untouchable:
        def __getattr__(self, name):
            raise AssertionError(f"library call {name} reached with mismatched arguments")

    monkeypatch.setattr(hbmm, "lib", Untouchable())
    monkeypatch.setattr(hbmm, "packed_ld_words", lambda K: ((K + 31) // 32 + 3) // 4 * 4)
    monkeypatch.setattr(hbmm, "num_blocks", lambda K, beta: (K + beta - 1) // beta)
    bits = torch.zeros((6, 4), dtype=torch.int32)
    scales = torch.zeros((6, 4), dtype=torch.float32)
    with pytest.raises(ValueError):
        hbmm.gemm(bits, scales, 32, bits[:5], scales, 32, 128)
    with pytest.raises(ValueError):
        hbmm.gemm(bits, scales, 32, bits, scales, 32, 128, out=torch.zeros((6, 7)))
    with pytest.raises(ValueError):
        hbmm.gemm(bits, scales, 32, bits, scales, 32, 512)                                  # K larger than the rows hold
    with pytest.raises(ValueError):
        hbmm.gemm_int(bits, bits, 512)
    with pytest.raises(ValueError):
        hbmm.dense_ref_gemm(torch.zeros((4, 64)), torch.zeros((5, 32)))                     # K mismatch
    with pytest.raises(ValueError):
        hbmm.dense_ref_gemm(torch.zeros((64, 4)).t(), torch.zeros((5, 64)))                 # strided A
    with pytest.raises(ValueError):
        hbmm.gemm_fused(torch.zeros((64, 4)).t(), 32, bits, scales, 32)                     # strided A
    with pytest.raises(ValueError):
        hbmm.gemm_fused(torch.zeros((9, 128)), 32, bits, scales, 32, out=torch.zeros((9, 5)))
    act_bits, act_scales = torch.zeros(8, dtype=torch.int32), torch.zeros(64)              # a 1 x 4 x 8 x 8 tensor, beta_a = 4
    with pytest.raises(ValueError):
        hbmm.conv2d(act_bits[:7], act_scales, 4, (1, 4, 8, 8), bits, scales, 32, (4, 8), 1, 0)           # too few activation words
    with pytest.raises(ValueError):
        hbmm.conv2d(act_bits, act_scales, 4, (1, 4, 8, 8), bits, scales, 32, (4, 8), 1, 0, out=torch.zeros((1, 6, 5, 2)))   # out is 1 x 6 x 5 x 1
    # the prepared-filter layer and the activation packing for widths that beta does not divide
    monkeypatch.setattr(hbmm, "conv_filter_pieces_bytes", lambda N, C, KH, KW, form=0: (N + 31) // 32 * ((C + 31) // 32) * KH * KW * 6144)
    pieces = torch.zeros(6144 * 2 * 9, dtype=torch.uint8)          # 40 filters of 20 x 3 x 3: two blocks of 32, one channel group
    x7 = torch.zeros((2, 20, 7, 7))
    a7_bits, a7_scales = torch.zeros((2 * 20 * 49 + 31) // 32, dtype=torch.int32), torch.zeros(2 * 20 * 7 * 2)
    with pytest.raises(ValueError):
        hbmm.conv2d_prepared(a7_bits, a7_scales, 4, x7.shape, pieces[:-1], 40, (3, 3), 1, 1)              # prepared filters too short
    with pytest.raises(ValueError):
        hbmm.conv2d_prepared(a7_bits, a7_scales[:-1], 4, x7.shape, pieces, 40, (3, 3), 1, 1)              # 2 scales per row of 7: one missing
    with pytest.raises(ValueError):
        hbmm.conv2d_prepared(a7_bits[:-1], a7_scales, 4, x7.shape, pieces, 40, (3, 3), 1, 1)              # too few words
    with pytest.raises(ValueError):
        hbmm.conv2d_prepared(a7_bits, a7_scales, 4, x7.shape, pieces, 40, (3, 3), 1, 1, out=torch.zeros((2, 40, 7, 6)))
    with pytest.raises(ValueError):
        hbmm.conv_prepare_filters(bits, scales, 32, 20, (3, 3))                                          # 180 elements per filter need 8 words, 6 scales
    with pytest.raises(ValueError):
        hbmm.conv_prepare_filters(torch.zeros((40, 8), dtype=torch.int32), torch.zeros((40, 6)), 32, 20, (3, 3), pieces[:100])
    with pytest.raises(ValueError):
        hbmm.quantize_pack_activations(x7.permute(0, 1, 3, 2), 4)                                         # not contiguous
    with pytest.raises(ValueError):
        hbmm.quantize_pack_activations(x7, 4, a7_bits[:-1], a7_scales)
    with pytest.raises(ValueError):
        hbmm.quantize_pack_activations(x7, 4, a7_bits, a7_scales[:-1])
