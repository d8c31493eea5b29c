"""Compile the C oracle into ``oracle/liboracle_hbmm.so`` with gcc (host only, no GPU code)."""
from __future__ import annotations

import subprocess
from pathlib import Path

HERE = Path(__file__).resolve().parent
SRC = HERE / "hbmm_oracle.c"
LIB = HERE / "liboracle_hbmm.so"


def build(force: bool = True) -> Path:
    if LIB.exists() and not force and LIB.stat().st_mtime >= SRC.stat().st_mtime:
        return LIB
    # -mpopcnt only: the library is built on one machine and run on another, so no -march=native.
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-mpopcnt", "-Wall", "-Wextra",
           str(SRC), "-o", str(LIB), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
