"""Static check of the compiled popcount GEMM.

The kernel issues its scalar loads of Q words through inline asm, which the compiler's
wait-count insertion does not track; the kernel waits for them itself (``s_waitcnt lgkmcnt(0)``)
before the first use.  This script compiles ``csrc/gemm_popcount.hip`` to gfx950 assembly and
verifies, for every such load, that no instruction between the load and the next
``s_waitcnt lgkmcnt(0)`` reads or writes the load's destination SGPRs (a register copy, spill or
re-use placed there by the register allocator would read data that has not arrived yet).

Run as ``python -m paper_1905_10759_amd.check_isa``; ``build.build()`` runs it after compiling.
"""
from __future__ import annotations

import re
import subprocess
import sys
import tempfile
from pathlib import Path
def regs(tok):
    out=set()
    for m in re.finditer(r"s\[(\d+):(\d+)\]", tok):
        out.update(range(int(m.group(1)), int(m.group(2))+1))
    for m in re.finditer(r"\bs(\d+)\b", tok):
        out.add(int(m.group(1)))
    return out
def check(path, verbose=True):
    inflight={}; bad=0; n=0; inasm=False
    for ln,line in enumerate(open(path),1):
        t=line.strip()
        if t.startswith(";;#ASMSTART"): inasm=True; continue
        if t.startswith(";;#ASMEND"): inasm=False; continue
        if not t or t.startswith((";",".")) or t.endswith(":"): continue
        t=t.split(";")[0].strip()
        if t.startswith("s_waitcnt") and "lgkmcnt(0)" in t:
            inflight.clear(); continue
        parts=t.split(None,1)
        ops=parts[1] if len(parts)>1 else ""
        used=regs(ops)
        if parts[0].startswith("s_load") and inasm:
            dst=regs(ops.split(",")[0]); src=regs(",".join(ops.split(",")[1:]))
            hit=src & set(inflight)
            if hit: print(f"{path}:{ln}: load reads in-flight {sorted(hit)}: {t}"); bad+=1
            for r in dst: inflight[r]=ln
            n+=1; continue
        hit=used & set(inflight)
        if hit:
            print(f"{path}:{ln}: touches in-flight s{sorted(hit)} (loaded at line {[inflight[r] for r in sorted(hit)]}): {t}"); bad+=1
    if verbose:
        print(f"check_isa: {n} asm scalar loads checked, {bad} violations")
    if n == 0:
        raise RuntimeError("check_isa: found no asm scalar loads; the check is not looking at the right code")
    return bad


def compile_and_check(verbose: bool = True) -> int:
    from . import build as _build

    src = _build.CSRC / "gemm_popcount.hip"
    with tempfile.TemporaryDirectory() as tmp:
        out = Path(tmp) / "gemm_popcount.s"
        subprocess.run([_build.HIPCC, *_build.FLAGS, "-S", "--cuda-device-only", str(src), "-o", str(out)],
                       check=True, stderr=subprocess.DEVNULL)
        return check(str(out), verbose)


if __name__ == "__main__":
    sys.exit(1 if compile_and_check() else 0)
