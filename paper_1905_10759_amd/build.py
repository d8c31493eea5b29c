"""Build ``libhbmm.so`` (the C-ABI library) from ``csrc/*.hip`` with hipcc for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libhbmm.so"
OBJ = HERE / "_build"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # packed fp32 VALU forms are kept out of generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources() -> list[Path]:
    return sorted(CSRC.glob("*.hip"))


def _compile(src: Path) -> Path:
    obj = OBJ / (src.stem + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", str(src), "-o", str(obj)], check=True)
    return obj


def build(force: bool = True) -> Path:
    srcs = sources()
    deps = srcs + list(CSRC.glob("*.h")) + [HERE.parent / "include" / "hbmm.h"]
    if LIB.exists() and not force and all(LIB.stat().st_mtime >= d.stat().st_mtime for d in deps):
        return LIB
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        objs = list(pool.map(_compile, srcs))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(LIB)], check=True)
    from . import check_isa
    if check_isa.compile_and_check(verbose=False):
        LIB.unlink()
        raise RuntimeError("check_isa: an in-flight scalar-load register is touched before its wait; library removed")
    return LIB


if __name__ == "__main__":
    print(build())
