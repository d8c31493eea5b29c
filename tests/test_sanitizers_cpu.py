"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; no sanitizer ever runs on
the GPU).  Two builds, each exercised in a child process that has the sanitizer runtime loaded first:

* the C oracle (gcc -fsanitize=address,undefined): the oracle pins run against it, ragged shapes and
  brute-force cases included, so an out-of-bounds index or a signed overflow in the checker itself
  would abort the child;
* the C-ABI layer of the library (csrc/api.hip with its host side instrumented, kernel launchers
  replaced by counting stubs): the validation tests of tests/test_boundary_cpu.py run against it, plus calls
  that pass validation and reach the (stubbed) launchers through the dispatch code."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _child_env(runtime: str, **extra) -> dict:
    env = dict(os.environ)
    # the sanitizer runtime has to come first in the child's preload list; whatever is there stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra)
    return env


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not available")
    runtime = subprocess.run([gcc, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not runtime or not Path(runtime).exists():
        pytest.skip("gcc's AddressSanitizer runtime not available")
    lib = tmp_path / "liboracle_hbmm_san.so"
    subprocess.run([gcc, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-mpopcnt", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    str(ROOT / "oracle" / "hbmm_oracle.c"), "-o", str(lib), "-lm"], check=True)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        str(ROOT / "tests" / "test_oracle_pins.py")],
                       env=_child_env(os.path.realpath(runtime), HBMM_ORACLE_LIB=str(lib)),
                       capture_output=True, text=True, cwd=str(ROOT), timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


_API_CHILD = r"""
import ctypes, sys
sys.path.insert(0, {tests!r})
lib = ctypes.CDLL({lib!r})
import test_boundary_cpu as t
t.test_validation_rejects_before_launch(lib)
t.test_validation_of_the_fused_tensor_and_convolution_entry_points(lib)
# calls that pass validation: the dispatch code runs up to the (stubbed) launchers
i64, i32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
fake = 0x1000
lib.hbmm_stub_launches.restype = ctypes.c_int
g = lib.hbmm_gemm
g.argtypes = [p, p, i64, i64, i32, p, p, i64, i64, i32, i64, i64, i64, p, i64, i32, p]
n0 = lib.hbmm_stub_launches()
for (ba, bw, algo) in [(32, 32, 0), (64, 256, 0), (64, 64, 1), (64, 64, 2), (16, 16, 3), (32, 32, -1), (256, 256, -1),
                       (1, 128, 0), (1, 4, 0), (4, 1, 0), (4, 4, 0), (2, 16, 0), (16, 2, 0), (8, 64, 0)]:
    a_bits = None if ba == 1 else fake
    b_bits = None if bw == 1 else fake
    rc = g(a_bits, fake, 8, 256, ba, b_bits, fake, 8, 256, bw, 300, 200, 256, fake, 200, algo, None)
    assert rc == 0, (ba, bw, algo, rc)
qp = lib.hbmm_quantize_pack
qp.argtypes = [p, i64, i64, i64, i32, i32, p, i64, p, i64, p]
for beta in (2, 4, 8, 16, 32, 64, 128, 256):
    assert qp(fake, 7, 256, 256, 0, beta, fake, 8, fake, 128, None) == 0
    assert qp(fake, 7, 256, 8, 1, beta, fake, 8, fake, 128, None) == 0
cv = lib.hbmm_conv2d
cv.argtypes = [p, p, i32, p, p, i64, i64, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, i32, p]
for (ba, bw) in [(4, 32), (1, 4), (4, 4), (2, 8), (8, 16)]:
    assert cv(None if ba == 1 else fake, fake, ba, fake, fake, 12, 144, bw, 2, 32, 8, 8, 40, 3, 3, 1, 1, fake, 0, None) == 0
# the general kernels: other segment lengths, a shorter last segment, K that does not fill a word
for (ba, bw, K) in [(3, 5, 19), (7, 1, 100), (1, 6, 96), (48, 64, 200), (32, 32, 40)]:
    rc = g(None if ba == 1 else fake, fake, 8, 256, ba, None if bw == 1 else fake, fake, 8, 256, bw, 30, 20, K, fake, 20, -1, None)
    assert rc == 0, (ba, bw, K, rc)
assert qp(fake, 7, 100, 100, 0, 7, fake, 4, fake, 15, None) == 0
assert qp(fake, 7, 19, 8, 1, 5, fake, 4, fake, 4, None) == 0
pf = lib.hbmm_conv_prepare_filters
pf.argtypes = [p, p, i64, i64, i32, i64, i64, i32, i32, i32, p, p]
cp = lib.hbmm_conv2d_prepared
cp.argtypes = [p, p, i32, p, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, p, p]
for (ba, bw) in [(4, 32), (1, 4), (4, 5), (2, 1)]:
    K = 20 * 9
    for form in (0, 1):
        assert pf(None if bw == 1 else fake, fake, 8, K, bw, 40, 20, 3, 3, form, fake, None) == 0
        assert cp(None if ba == 1 else fake, fake, ba, fake, form, 2, 20, 8, 8, 40, 3, 3, 1, 1, fake, None) == 0
qa = lib.hbmm_quantize_pack_activations
qa.argtypes = [p, i64, i64, i32, p, p, p]
assert qa(fake, 64 * 7, 7, 4, fake, fake, None) == 0       # ragged width: the general kernel
assert qa(fake, 64 * 8, 8, 3, fake, fake, None) == 0
assert qa(fake, 64 * 8, 8, 4, fake, fake, None) == 0       # the tuned kernel through the flat view
assert cp(fake, fake, 3, fake, 0, 2, 20, 7, 7, 40, 3, 3, 1, 1, fake, None) == 0
assert lib.hbmm_stub_launches() - n0 == 14 + 16 + 5 + 5 + 2 + 16 + 4
print("api under sanitizers: ok")
"""


def test_c_abi_layer_under_asan_and_ubsan(tmp_path):
    if not Path(HIPCC).exists():
        pytest.skip("hipcc not available")
    found = sorted(Path("/opt/rocm/lib/llvm/lib/clang").glob("*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not found:
        pytest.skip("clang's AddressSanitizer runtime not available")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    objs = []
    for src in (ROOT / "paper_1905_10759_amd" / "csrc" / "api.hip", ROOT / "tests" / "sanitize" / "launch_stubs.cpp"):
        obj = tmp_path / (src.stem + ".o")
        # (device code is compiled as usual -- api.hip holds one small fill kernel -- and only the host
        # side is instrumented)
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-x", "hip", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer",
                        *san, "-c", str(src), "-o", str(obj)], check=True, stderr=subprocess.DEVNULL)
        objs.append(str(obj))
    lib = tmp_path / "libhbmm_host_san.so"
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                    "-fsanitize=undefined", "-shared-libsan", *objs, "-o", str(lib)], check=True, stderr=subprocess.DEVNULL)
    code = _API_CHILD.format(tests=str(ROOT / "tests"), lib=str(lib))
    r = subprocess.run([sys.executable, "-c", code], env=_child_env(str(found[-1])), capture_output=True, text=True,
                       cwd=str(ROOT), timeout=600)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "api under sanitizers: ok" in r.stdout and "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
