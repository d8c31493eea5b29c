#!/usr/bin/env python3
"""Benchmark of the HBMM hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already
resident in HBM:  quantize_pack(A)  ->  quantize_pack(B)  ->  hbmm_gemm  (XNOR + popcount with the
fused block-scale epilogue).  The headline workload is the 8192^3 square HBMM with
beta_a = beta_w = 256, the configuration the popcount-roofline target is stated on.

Prints ONE JSON line.  `value` is effective GOPS of the step (2*M*N*K / step time).  `roofline`
describes the dominant kernel (the popcount GEMM) against the integer-VALU popcount peak;
`cpu_baseline` is the CPU oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

# Peak used for the GEMM: 256 CUs x 64 VALU lanes x 2.4 GHz lane-ops/s; one v_xor_b32 plus one
# accumulating v_bcnt_u32_b32 retire 32 binary multiply-adds = 64 binary ops per lane per 2 issues.
VALU_LANE_OPS = 256 * 64 * 2.4e9
POPCOUNT_PEAK_TOPS = VALU_LANE_OPS * 32 / 1e12      # 1258.3
HBM_PEAK_GBS = 8000.0
BF16_PEAK_TFLOPS = 2500.0
FP4_PEAK_TFLOPS = 10100.0                           # dense fp4 MFMA


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="sq8k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip comparison kernels and the other configs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy per step (known-size reference for HBM counters)")
    return ap.parse_args()


def kernel_source_digest(*files: str) -> str:
    """sha256 over the kernel sources a profile summary belongs to (csrc/ file names)."""
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update((ROOT / "paper_1905_10759_amd" / "csrc" / f).read_bytes())
    return h.hexdigest()[:16]


def profiled_traffic(kernel_file: str, *sources: str) -> dict:
    """HBM bytes per launch measured with rocprofv3 counters for the headline workload.  bench.py cannot
    collect counters itself: the figure comes from the committed summary under profiles/ (two --pmc runs
    of this bench, FETCH_SIZE and WRITE_SIZE, scaled by what a plain copy of known size reads).  The
    summary records a digest of the kernel sources it was taken from; if they have changed since, the
    figure is stale and reported as null."""
    info = {"traffic": None, "traffic_source": f"profiles/{kernel_file} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                               "bench, calibrated with a 256 MiB device copy; not measured in this run)"}
    try:
        text = (ROOT / "profiles" / kernel_file).read_text()
    except OSError:
        info["traffic_source"] += "; summary missing"
        return info
    recorded = value = None
    for line in text.splitlines():
        if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
            value = float(line.split("=", 1)[1])
        if line.startswith("KERNEL_SOURCES_SHA256="):
            recorded = line.split("=", 1)[1].strip()
    if recorded is not None and sources and recorded != kernel_source_digest(*sources):
        info["traffic_source"] += "; kernel sources changed since the summary was taken: figure withheld"
        return info
    info["traffic"] = value
    return info


def pack_bytes(rows: int, K: int, beta: int) -> float:
    return rows * K * (4.0 + 1.0 / 8.0 + 4.0 / beta)


def time_loop(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]


def back_to_back_ms(calls, reps, torch, warm=3):
    """Average time of one call when `calls` (a list of closures, walked round robin) are queued back to
    back between ONE pair of events: kernel time, not launch or event latency."""
    for i in range(warm * len(calls)):
        calls[i % len(calls)]()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        calls[i % len(calls)]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


VALU_EPILOGUE_LANE_OPS = VALU_LANE_OPS      # lane-ops / s of plain vector instructions (one per lane per cycle)


def split_kernel_roofline(M, N, K, beta_a, beta_w, ms):
    """Roofline of the matrix-core path (an unquantised operand or a segment shorter than a word): bf16 MFMA
    flops actually issued -- 3 piece products per element pair, 6 when both operands are rebuilt -- against
    the dense bf16 peak; for beta = 16 also the vector-ALU bound of its epilogue (one FMA and one clear per
    output per 16-element segment)."""
    pieces = 6 if max(beta_a, beta_w) < 16 or (min(beta_a, beta_w) == 1 and max(beta_a, beta_w) < 16) else 3
    flops = pieces * 2.0 * M * N * K
    r = {"bound": "mfma", "kernel": "mfma_split_gemm_kernel", "piece_products": pieces,
         "achieved": flops / (ms * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
         "frac": flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS}
    g = max(beta_a, beta_w) if min(beta_a, beta_w) < 16 else min(beta_a, beta_w)   # the sign side's segment
    if pieces == 3 and g == 16:
        lane_ops = 2.0 * M * N * (K / 16)
        r["epilogue_alu_bound_ms"] = lane_ops / VALU_EPILOGUE_LANE_OPS * 1e3
        r["frac_of_epilogue_alu_bound"] = r["epilogue_alu_bound_ms"] / ms
    return r


def cpu_baseline(w, A, B):
    """The oracle's own integer path (scales + sign-pack + Eq. 7) on a row sample of A against all
    of B, and its dense double-precision path on a smaller sample; both as they stand."""
    import oracle

    threads = oracle.num_threads()
    rows_i = w.M
    t0 = time.perf_counter()
    a_bits, a_s = oracle.sign_pack(A[:rows_i]), oracle.block_scales(A[:rows_i], w.beta_a)
    b_bits, b_s = oracle.sign_pack(B), oracle.block_scales(B, w.beta_w)
    oracle.popcount_gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K)
    t_int = time.perf_counter() - t0
    rows_d = min(w.M, 3072)
    t0 = time.perf_counter()
    oracle.dense_f64_gemm(oracle.materialize(A[:rows_d], w.beta_a), oracle.materialize(B, w.beta_w))
    t_dense = time.perf_counter() - t0
    return {
        "value": 2.0 * rows_i * w.N * w.K / t_int / 1e9,
        "unit": "GOPS",
        "cores": threads,
        "nproc": os.cpu_count(),
        "physical_cores": _physical_cores(),
        "omp_num_threads_env": os.environ.get("OMP_NUM_THREADS"),
        "kind": "oracle",
        "sample": f"integer path (scales + sign-pack of both operands + Eq.7 popcount product), all {rows_i} rows of A "
                  f"x all {w.N} rows of B: {t_int:.2f} s; dense f64 path (materialise + naive product) on the first "
                  f"{rows_d} rows of A x all of B: {2.0 * rows_d * w.N * w.K / t_dense / 1e9:.2f} GOPS in {t_dense:.2f} s",
        "dense_f64_gops": 2.0 * rows_d * w.N * w.K / t_dense / 1e9,
        "cpu_model": _cpu_model(),
    }


def _physical_cores():
    """Distinct (physical id, core id) pairs of /proc/cpuinfo; None if the file does not say."""
    try:
        cores, phys = set(), None
        for line in open("/proc/cpuinfo"):
            if line.startswith("physical id"):
                phys = line.split(":", 1)[1].strip()
            elif line.startswith("core id"):
                cores.add((phys, line.split(":", 1)[1].strip()))
        return len(cores) or None
    except OSError:
        return None


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the HBMM path shards over rows of A without any "
              "collective; multi-GPU is a design note, not code). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1905_10759_amd import hbmm, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    w = synth.WORKLOADS[args.workload]
    A_h, B_h = w.make_a(), w.make_b()
    A, B = torch.from_numpy(A_h).cuda(), torch.from_numpy(B_h).cuda()
    rows_b = w.N
    ldw, nba, nbw = hbmm.packed_ld_words(w.K), hbmm.num_blocks(w.K, max(w.beta_a, 1)), hbmm.num_blocks(w.K, w.beta_w)
    a_bits = torch.empty((w.M, ldw), dtype=torch.int32, device="cuda")
    b_bits = torch.empty((rows_b, ldw), dtype=torch.int32, device="cuda")
    a_s = torch.empty((w.M, nba), dtype=torch.float32, device="cuda")
    b_s = torch.empty((rows_b, nbw), dtype=torch.float32, device="cuda")
    C = torch.empty((w.M, w.N), dtype=torch.float32, device="cuda")
    binary_act = w.beta_a != 1

    cal_src = cal_dst = None
    if args.copy_calibration:
        cal_src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB
        cal_dst = torch.empty_like(cal_src)

    marks = []   # (pack_a0, pack_a1/pack_b0, pack_b1/gemm0, gemm1) per timed step

    def step(record=False):
        if record:
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            e[0].record()
        if binary_act:
            hbmm.quantize_pack(A, w.beta_a, 0, a_bits, a_s)
        if record:
            e[1].record()
        hbmm.quantize_pack(B, w.beta_w, w.b_layout, b_bits, b_s)
        if record:
            e[2].record()
        if binary_act:
            hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_POPCOUNT, C)
        else:
            hbmm.gemm(None, A, 1, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_POPCOUNT, C)
        if record:
            e[3].record()
            marks.append(e)
        if cal_src is not None:
            cal_dst.copy_(cal_src)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(args.steps):
        step(record=True)
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    total_ms = start.elapsed_time(stop)
    ms_per_step = total_ms / args.steps
    ops = 2.0 * w.M * w.N * w.K

    t_pack_a = float(np.mean([e[0].elapsed_time(e[1]) for e in marks]))
    t_pack_b = float(np.mean([e[1].elapsed_time(e[2]) for e in marks]))
    t_gemm = float(np.mean([e[2].elapsed_time(e[3]) for e in marks]))

    out = {
        "metric": "hbmm_effective_gops",
        "value": ops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 xor/popcount -> i32, f32 block-scale accumulate",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: HBMM M={w.M} K={w.K} N={w.N}, beta_a={w.beta_a} beta_w={w.beta_w}, "
                        f"A {w.a_kind}, B {w.b_kind}; step = pack(A) + pack(B) + hbmm_gemm(algo 0)",
            "M": w.M, "K": w.K, "N": w.N, "beta_a": w.beta_a, "beta_w": w.beta_w,
        },
        "wall_ms_per_step": wall_ms / args.steps,
        "kernel_ms": {"pack_a": t_pack_a, "pack_b": t_pack_b, "gemm": t_gemm,
                      "gemm_median": float(np.median([e[2].elapsed_time(e[3]) for e in marks])),
                      "gemm_min": float(np.min([e[2].elapsed_time(e[3]) for e in marks]))},
    }
    word_sized = w.beta_a >= 32 and w.beta_w >= 32
    if word_sized:
        out["roofline"] = {
            "kernel": "popcount_gemm_kernel (hbmm_gemm algo 0)",
            "bound": "alu",
            "achieved": ops / (t_gemm * 1e-3) / 1e12,
            "peak": POPCOUNT_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": ops / (t_gemm * 1e-3) / 1e12 / POPCOUNT_PEAK_TOPS,
            "traffic": None,
            "traffic_unit": "HBM bytes per launch (FETCH_SIZE + WRITE_SIZE counters, calibrated)",
            # packed bits and scales of both operands in, fp32 C out
            "algorithmic_bytes": (w.M + w.N) * (w.K / 8.0) + 4.0 * (w.M * (w.K // w.beta_a) + w.N * (w.K // w.beta_w)) + 4.0 * w.M * w.N,
        }
        if w.name == "sq8k":
            out["roofline"].update(profiled_traffic("popcount_gemm_kernel_sq8k.txt", "gemm_popcount.hip", "tile_map.h"))
    else:
        # beta = 1 or a segment shorter than 32 runs on the matrix cores: the dense side is split into
        # three bf16 pieces, so the kernel issues 3 x 2MNK bf16 flops per launch (6 when both sides are rebuilt).
        out["roofline"] = split_kernel_roofline(w.M, w.N, w.K, w.beta_a, w.beta_w, t_gemm)
        out["roofline"]["traffic"] = None
    if binary_act and w.b_layout == 0:
        # Pack timed on its own: launches queued back to back (A, B, A, B, ...: 2 x 268 MB of source at
        # the headline size, more than the 256 MB last-level cache) between one pair of events, so the
        # figure is kernel time and not launch latency.
        n_pack = 2 * max(10, args.steps)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n_pack // 2):
            hbmm.quantize_pack(A, w.beta_a, 0, a_bits, a_s)
            hbmm.quantize_pack(B, w.beta_w, 0, b_bits, b_s)
        e1.record()
        torch.cuda.synchronize()
        t_pack = e0.elapsed_time(e1) / n_pack
        gbs = 0.5 * (pack_bytes(w.M, w.K, w.beta_a) + pack_bytes(w.N, w.K, w.beta_w)) / (t_pack * 1e-3) / 1e9
        out["roofline_pack"] = {
            "kernel": "pack_rows_kernel (hbmm_quantize_pack)", "bound": "hbm", "achieved": gbs,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
            "traffic": None, "algorithmic_bytes": 0.5 * (pack_bytes(w.M, w.K, w.beta_a) + pack_bytes(w.N, w.K, w.beta_w)),
            "ms_per_launch": t_pack, "launches": n_pack,
        }
        if w.name == "sq8k":
            out["roofline_pack"].update(profiled_traffic("pack_rows_kernel_sq8k.txt", "pack.hip", "wave_ops.h"))
        # context for that fraction: what a plain device-to-device copy of the same sources reaches on this
        # device (library copy kernel; bytes read + bytes written per second)
        dst = torch.empty_like(A)
        dst.copy_(A)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n_pack // 2):
            dst.copy_(A)
            dst.copy_(B)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 2.0 * A.numel() * 4 / (e0.elapsed_time(e1) / n_pack * 1e-3) / 1e9
        out["roofline_pack"]["device_copy_GBs"] = copy_gbs
        out["roofline_pack"]["achieved_vs_device_copy"] = gbs / copy_gbs
        del dst

    if binary_act and w.b_layout == 0 and min(w.beta_a, w.beta_w) >= 64:
        try:
            # The same step with the product on the matrix cores in 4-bit floats (hbmm_gemm algo 2: same
            # result bit for bit).  Reported next to the headline, which stays on the XNOR + popcount kernel.
            def step4():
                hbmm.quantize_pack(A, w.beta_a, 0, a_bits, a_s)
                hbmm.quantize_pack(B, w.beta_w, 0, b_bits, b_s)
                hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_MFMA_FP4, C)

            for _ in range(args.warmup):
                step4()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                step4()
            e1.record()
            torch.cuda.synchronize()
            ms4 = e0.elapsed_time(e1) / args.steps
            tg = time_loop(lambda: hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_MFMA_FP4, C),
                           args.steps, 2, torch)
            g4 = float(np.mean(tg))
            out["step_with_fp4_mfma_variant"] = {
                "ms_per_step": ms4, "value": ops / (ms4 * 1e-3) / 1e9, "unit": "GOPS", "gemm_ms": g4,
                "speedup_vs_headline_step": ms_per_step / ms4,
                "roofline": {"kernel": "mfma_fp4_gemm_kernel (hbmm_gemm algo 2)", "bound": "mfma",
                             "achieved": ops / (g4 * 1e-3) / 1e12, "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": ops / (g4 * 1e-3) / 1e12 / FP4_PEAK_TFLOPS, "traffic": None},
            }
            if w.name == "sq8k":
                out["step_with_fp4_mfma_variant"]["roofline"].update(profiled_traffic("mfma_fp4_gemm_kernel_sq8k.txt", "gemm_mfma_fp4.hip"))
        except Exception as e:   # a comparison figure must never take the headline line down
            out["step_with_fp4_mfma_variant"] = {"error": f"{type(e).__name__}: {e}"}

    if not args.no_extras:
        try:
            out["comparisons"] = extras(w, A, B, a_bits, a_s, b_bits, b_s, C, torch, hbmm, synth, args)
        except Exception as e:   # comparison figures must never take the headline line down
            out["comparisons"] = {"error": f"{type(e).__name__}: {e}"}
    if not args.no_cpu_baseline:
        import oracle
        out["cpu_baseline"] = cpu_baseline(w, A_h, oracle.as_rows_by_k(B_h, w.b_layout))
    print(json.dumps(out))


def extras(w, A, B, a_bits, a_s, b_bits, b_s, C, torch, hbmm, synth, args):
    """Comparison points next to the headline: dense GEMMs on the same shape and the int8 matrix-core
    variant; then the other workloads (kernel times only)."""
    res = {}
    ops = 2.0 * w.M * w.N * w.K
    steps, warm = max(5, args.steps // 3), 2

    def gops(ms):
        return ops / (ms * 1e-3) / 1e9

    if w.beta_a != 1 and w.b_layout == 0:
        try:
            ts = time_loop(lambda: hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_MFMA_I8, C),
                           steps, warm, torch)
            res["hbmm_gemm_int8_mfma"] = {"ms": float(sum(ts) / len(ts)), "gops": gops(sum(ts) / len(ts))}
        except hbmm.HbmmError as e:
            res["hbmm_gemm_int8_mfma"] = {"error": str(e)}
        try:
            ts = time_loop(lambda: hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_MFMA_FP4, C),
                           steps, warm, torch)
            ms4 = float(sum(ts) / len(ts))
            # dense fp4 MFMA peak 10.1 PFLOP/s; 2MNK flops per launch
            res["hbmm_gemm_fp4_mfma"] = {"ms": ms4, "gops": gops(ms4), "frac_of_fp4_mfma_peak": gops(ms4) / 10.1e6}
        except hbmm.HbmmError as e:
            res["hbmm_gemm_fp4_mfma"] = {"error": str(e)}
        Ab, Bb = A.to(torch.bfloat16), B.to(torch.bfloat16)
        try:
            ts = time_loop(lambda: hbmm.dense_ref_gemm(Ab, Bb, C), steps, warm, torch)
            res["dense_ref_bf16"] = {"ms": float(sum(ts) / len(ts)), "gflops": gops(sum(ts) / len(ts))}
        except hbmm.HbmmError as e:
            res["dense_ref_bf16"] = {"error": str(e)}
        ts = time_loop(lambda: torch.matmul(Ab, Bb.t()), steps, warm, torch)
        res["torch_matmul_bf16"] = {"ms": float(sum(ts) / len(ts)), "gflops": gops(sum(ts) / len(ts))}
        # "speedup vs bf16 GEMM": the library GEMM on the same shape against each HBMM product kernel
        t_lib = res["torch_matmul_bf16"]["ms"]
        tg0 = time_loop(lambda: hbmm.gemm(a_bits, a_s, w.beta_a, b_bits, b_s, w.beta_w, w.K, hbmm.ALGO_POPCOUNT, C), steps, warm, torch)
        res["speedup_vs_torch_matmul_bf16"] = {"popcount": t_lib / float(sum(tg0) / len(tg0))}
        if "ms" in res.get("hbmm_gemm_fp4_mfma", {}):
            res["speedup_vs_torch_matmul_bf16"]["fp4_mfma"] = t_lib / res["hbmm_gemm_fp4_mfma"]["ms"]
        del Ab, Bb
    # gradient through the binarisation (Eq. 5-6): 8 bytes read + 4 written per element
    try:
        gsrc, gout = torch.randn_like(A), torch.empty_like(A)
        beta_b = max(w.beta_a, 2)
        ts = time_loop(lambda: hbmm.binarize_backward(A, gsrc, beta_b, gout), steps, warm, torch)
        ms = float(sorted(ts)[len(ts) // 2])
        res["binarize_backward"] = {"ms": ms, "GBs": 12.0 * w.M * w.K / (ms * 1e-3) / 1e9, "beta": beta_b,
                                    "frac_of_hbm_peak": 12.0 * w.M * w.K / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del gsrc, gout
    except hbmm.HbmmError as e:
        res["binarize_backward"] = {"error": str(e)}
    res["paper_context"] = "paper reports ~10x for its CPU HBMM kernel over a classical fp32 matmul on a Xeon Gold 6128 (beta=16)"

    # (20 warm-up launches each: these kernels are short, and the inputs are generated on the host in
    # between, so the device has clocked down every time a new workload starts)
    others = {}
    for name, ww in synth.WORKLOADS.items():
        if name == w.name:
            continue
        Ah, Bh = ww.make_a(), ww.make_b()
        dA, dB = torch.from_numpy(Ah).cuda(), torch.from_numpy(Bh).cuda()
        bb, bs = hbmm.quantize_pack(dB, ww.beta_w, ww.b_layout)
        entry = {}
        if ww.beta_a != 1:
            ab, as_ = hbmm.quantize_pack(dA, ww.beta_a)
            # pack(A) on its own: launches queued back to back over enough copies of the source (at least
            # 512 MB together, at most 16) that it cannot stay in the 256 MB last-level cache
            ncopy = max(1, min(16, -(-512 * 2**20 // (dA.numel() * 4))))
            srcs = [dA] + [dA.clone() for _ in range(ncopy - 1)]
            t_pack_a = back_to_back_ms([(lambda x=x: hbmm.quantize_pack(x, ww.beta_a, 0, ab, as_)) for x in srcs], 60, torch)
            from_hbm = ncopy * dA.numel() * 4 >= 512 * 2**20
            entry["pack_a_ms"] = t_pack_a
            gbs_a = pack_bytes(ww.M, ww.K, ww.beta_a) / (t_pack_a * 1e-3) / 1e9
            if from_hbm:
                entry["pack_a_GBs"] = gbs_a
                entry["pack_a_frac_of_hbm_peak"] = gbs_a / HBM_PEAK_GBS
            else:   # too small to be pushed out of the cache with 16 copies: not an HBM figure
                entry["pack_a_GBs_cache_resident"] = gbs_a
            entry["pack_a_sources_rotated"] = ncopy
            del srcs
            tg = time_loop(lambda: hbmm.gemm(ab, as_, ww.beta_a, bb, bs, ww.beta_w, ww.K), 30, 20, torch)
            # the fastest kernel for these segment lengths (hbmm_gemm algo -1: fp4 / fp8 matrix-core variants)
            tf = time_loop(lambda: hbmm.gemm(ab, as_, ww.beta_a, bb, bs, ww.beta_w, ww.K, hbmm.ALGO_FASTEST), 30, 20, torch)
            entry["gemm_fastest_algo_ms"] = min(tf)
            entry["gemm_fastest_algo_gops"] = 2.0 * ww.M * ww.N * ww.K / (min(tf) * 1e-3) / 1e9
        else:
            tg = time_loop(lambda: hbmm.gemm(None, dA, 1, bb, bs, ww.beta_w, ww.K), 30, 20, torch)
        entry["gemm_ms"] = min(tg)
        entry["gemm_gops"] = 2.0 * ww.M * ww.N * ww.K / (min(tg) * 1e-3) / 1e9
        if min(ww.beta_a, ww.beta_w) >= 32:   # the XNOR + popcount kernel
            entry["gemm_frac_of_popcount_peak"] = entry["gemm_gops"] / (POPCOUNT_PEAK_TOPS * 1e3)
            entry["roofline"] = {"bound": "alu", "kernel": "popcount_gemm_kernel", "achieved": entry["gemm_gops"] / 1e3,
                                 "peak": POPCOUNT_PEAK_TOPS, "unit": "TOP/s", "frac": entry["gemm_frac_of_popcount_peak"]}
        else:
            entry["roofline"] = split_kernel_roofline(ww.M, ww.N, ww.K, ww.beta_a, ww.beta_w, entry["gemm_ms"])
        # the full-precision comparison on the same shape: the library's bf16 GEMM and this
        # repository's own dense kernel (operands in the same rows x K form)
        try:
            dBr = dB.t().contiguous() if ww.b_layout == 1 else dB
            Ab16, Bb16 = dA.to(torch.bfloat16), dBr.to(torch.bfloat16)
            tl = time_loop(lambda: torch.matmul(Ab16, Bb16.t()), 30, 20, torch)
            entry["torch_matmul_bf16_ms"] = min(tl)
            entry["speedup_vs_torch_matmul_bf16"] = {"gemm": min(tl) / entry["gemm_ms"]}
            if "gemm_fastest_algo_ms" in entry:
                entry["speedup_vs_torch_matmul_bf16"]["gemm_fastest_algo"] = min(tl) / entry["gemm_fastest_algo_ms"]
            if ww.K % 64 == 0:
                Cd = torch.empty((ww.M, ww.N), dtype=torch.float32, device="cuda")
                td = time_loop(lambda: hbmm.dense_ref_gemm(Ab16, Bb16, Cd), 20, 10, torch)
                entry["dense_ref_bf16_ms"] = min(td)
                del Cd
            del Ab16, Bb16, dBr
        except (hbmm.HbmmError, RuntimeError) as e:
            entry["torch_matmul_bf16_ms"] = f"unavailable: {type(e).__name__}"
        if ww.M * ww.N * ww.K < 1e9 and ww.beta_a != 1:
            # launch-bound shapes: the whole step (pack A, pack B, gemm) queued back to back, and the same
            # three launches captured once into a HIP graph and replayed (the library allocates nothing
            # and never synchronises, so it can be captured as is)
            Cw = torch.empty((ww.M, ww.N), dtype=torch.float32, device="cuda")

            def whole_step():
                hbmm.quantize_pack(dA, ww.beta_a, 0, ab, as_)
                hbmm.quantize_pack(dB, ww.beta_w, ww.b_layout, bb, bs)
                hbmm.gemm(ab, as_, ww.beta_a, bb, bs, ww.beta_w, ww.K, hbmm.ALGO_POPCOUNT, Cw)

            reps = 200
            whole_step()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                whole_step()
            e1.record()
            torch.cuda.synchronize()
            entry["step_ms_back_to_back"] = e0.elapsed_time(e1) / reps
            if ww.N <= 128 and min(ww.beta_a, ww.beta_w) >= 32:
                # weights packed once, activations quantised, packed and multiplied by one launch
                try:
                    Cf = torch.empty_like(Cw)
                    hbmm.gemm_fused(dA, ww.beta_a, bb, bs, ww.beta_w, Cf)
                    torch.cuda.synchronize()
                    e0.record()
                    for _ in range(reps):
                        hbmm.gemm_fused(dA, ww.beta_a, bb, bs, ww.beta_w, Cf)
                    e1.record()
                    torch.cuda.synchronize()
                    entry["step_ms_fused_single_launch"] = e0.elapsed_time(e1) / reps
                    entry["fused_matches_three_launches"] = bool(torch.equal(Cf, Cw))
                    del Cf
                except hbmm.HbmmError as e:
                    entry["step_ms_fused_single_launch"] = f"unavailable: {e}"
            try:
                side = torch.cuda.Stream()
                with torch.cuda.stream(side):
                    whole_step()
                    side.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=side):
                        whole_step()
                    graph.replay()
                    side.synchronize()
                    ref = Cw.clone()
                    e0.record(side)
                    for _ in range(reps):
                        graph.replay()
                    e1.record(side)
                    side.synchronize()
                entry["step_ms_hip_graph"] = e0.elapsed_time(e1) / reps
                entry["hip_graph_matches_eager"] = bool(torch.equal(ref, Cw))
            except Exception as e:   # graph capture is a convenience figure, never a failure of the bench
                entry["step_ms_hip_graph"] = f"unavailable: {type(e).__name__}"
        others[name] = entry
        del dA, dB
    res["other_workloads"] = others

    # convolution layers computed directly from the packed tensors (no im2col matrix), and the fused
    # quantise+pack+product on the im2col shape of the first of them
    convs = {}
    for name, cw in synth.CONV_WORKLOADS.items():
        try:
            dA = torch.from_numpy(cw.make_a()).cuda()
            dW = torch.from_numpy(cw.make_w().reshape(cw.N, -1)).cuda()
            wb, ws = hbmm.quantize_pack(dW, cw.beta_w)
            entry = {"beta_a": cw.beta_a, "beta_w": cw.beta_w}
            ragged = cw.W % cw.beta_a != 0    # only the prepared-filter form takes a width that beta_a does not divide
            if cw.beta_a == 1:      # binary-weight layer: the activations go in as they are
                ab, asc = None, dA
            elif ragged:
                ab, asc = hbmm.quantize_pack_activations(dA, cw.beta_a)
                entry["quantize_ms"] = back_to_back_ms([lambda: hbmm.quantize_pack_activations(dA, cw.beta_a, ab, asc)], 40, torch)
                entry["quantize_kernel"] = "pack_activations_any_kernel (untuned)"
            else:
                ab, asc = hbmm.quantize_pack_tensor(dA, cw.beta_a)
                # queued back to back between one pair of events (a single launch of the small layers is
                # shorter than the events' own resolution)
                tq = back_to_back_ms([lambda: hbmm.quantize_pack_tensor(dA, cw.beta_a, ab, asc)], 40, torch)
                qbytes = dA.numel() * (4.0 + 1.0 / 8.0 + 4.0 / cw.beta_a)
                entry["quantize_ms"] = tq
                entry["quantize_GBs_cache_resident" if dA.numel() * 4 < 512 * 2**20 else "quantize_GBs"] = qbytes / (tq * 1e-3) / 1e9
            oh, ow = (cw.H + 2 * cw.pad - cw.KH) // cw.stride + 1, (cw.W + 2 * cw.pad - cw.KW) // cw.stride + 1
            out = torch.empty((cw.batch, cw.N, oh, ow), dtype=torch.float32, device="cuda")
            if not ragged:
                hbmm.conv2d(ab, asc, cw.beta_a, dA.shape, wb, ws, cw.beta_w, (cw.KH, cw.KW), cw.stride, cw.pad, out)
                tc = back_to_back_ms([lambda: hbmm.conv2d(ab, asc, cw.beta_a, dA.shape, wb, ws, cw.beta_w, (cw.KH, cw.KW),
                                                          cw.stride, cw.pad, out)], 20, torch)
                pieces = 6 if cw.beta_w < 16 else 3
                entry.update({"conv_ms": tc, "conv_effective_gflops": 2.0 * cw.macs / (tc * 1e-3) / 1e9,
                              "roofline": {"bound": "mfma", "kernel": "conv_patch_kernel / mfma_split_gemm_kernel (conv mode)",
                                           "piece_products": pieces,
                                           "achieved": pieces * 2.0 * cw.macs / (tc * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS,
                                           "unit": "TFLOP/s", "frac": pieces * 2.0 * cw.macs / (tc * 1e-3) / 1e12 / BF16_PEAK_TFLOPS}})
            # the same layer with the filters prepared ahead of time (once per set of weights, outside the timed
            # region like the packing of the filters itself); six piece products per element pair
            try:
                prepared = hbmm.conv_prepare_filters(wb, ws, cw.beta_w, cw.C, (cw.KH, cw.KW))
                tprep = back_to_back_ms([lambda: hbmm.conv_prepare_filters(wb, ws, cw.beta_w, cw.C, (cw.KH, cw.KW), prepared)], 20, torch)
                hbmm.conv2d_prepared(ab, asc, cw.beta_a, dA.shape, prepared, cw.N, (cw.KH, cw.KW), cw.stride, cw.pad, out)
                tp = back_to_back_ms([lambda: hbmm.conv2d_prepared(ab, asc, cw.beta_a, dA.shape, prepared, cw.N, (cw.KH, cw.KW),
                                                                   cw.stride, cw.pad, out)], 20, torch)
                entry.update({"conv_prepared_ms": tp, "prepare_filters_ms": tprep,
                              "roofline_prepared": {"bound": "mfma", "kernel": "conv_direct_kernel", "piece_products": 6,
                                                    "achieved": 6 * 2.0 * cw.macs / (tp * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS,
                                                    "unit": "TFLOP/s", "frac": 6 * 2.0 * cw.macs / (tp * 1e-3) / 1e12 / BF16_PEAK_TFLOPS}})
                del prepared
                # the two-piece form of the same layer: operands scaled into fp16's range and written as two fp16
                # pieces (22 significant bits), three piece products per element pair
                f16x2 = hbmm.PIECES_F16X2
                prepared = hbmm.conv_prepare_filters(wb, ws, cw.beta_w, cw.C, (cw.KH, cw.KW), form=f16x2)
                hbmm.conv2d_prepared(ab, asc, cw.beta_a, dA.shape, prepared, cw.N, (cw.KH, cw.KW), cw.stride, cw.pad, out, form=f16x2)
                t2 = back_to_back_ms([lambda: hbmm.conv2d_prepared(ab, asc, cw.beta_a, dA.shape, prepared, cw.N, (cw.KH, cw.KW),
                                                                   cw.stride, cw.pad, out, form=f16x2)], 20, torch)
                entry.update({"conv_prepared_f16x2_ms": t2,
                              "roofline_prepared_f16x2": {"bound": "mfma", "kernel": "conv_direct_kernel (two fp16 pieces)",
                                                          "piece_products": 3,
                                                          "achieved": 3 * 2.0 * cw.macs / (t2 * 1e-3) / 1e12, "peak": BF16_PEAK_TFLOPS,
                                                          "unit": "TFLOP/s", "frac": 3 * 2.0 * cw.macs / (t2 * 1e-3) / 1e12 / BF16_PEAK_TFLOPS}})
                del prepared
            except Exception as e:
                entry["conv_prepared_error"] = str(e)
            convs[name] = entry
            del dA, dW, out
        except Exception as e:
            convs[name] = {"error": str(e)}
    res["conv2d"] = convs
    # what the matrix cores sustain on this device with nothing else in the loop (pseudo-random register operands,
    # one workgroup of eight waves per compute unit): the ceiling that the fractions of the bf16 peak above can reach
    try:
        hbmm.probe_mfma_rate(500, 256)
        res["mfma_bf16_sustained_TFLOPs"] = min(hbmm.probe_mfma_rate(4000, 256) for _ in range(3))
    except Exception as e:
        res["mfma_bf16_sustained_TFLOPs"] = {"error": str(e)}
    try:
        M, K, N, beta = 3136 * 64, 576, 64, 64
        dA = torch.from_numpy(synth.relu_normal(8001, (M, K))).cuda()
        dB = torch.from_numpy(synth.normal(8002, (N, K))).cuda()
        bb, bs = hbmm.quantize_pack(dB, beta)
        ab, as_ = hbmm.quantize_pack(dA, beta)
        Cw = torch.empty((M, N), dtype=torch.float32, device="cuda")

        def two_step():
            hbmm.quantize_pack(dA, beta, 0, ab, as_)
            hbmm.gemm(ab, as_, beta, bb, bs, beta, K, hbmm.ALGO_POPCOUNT, Cw)

        t2 = time_loop(two_step, 10, 2, torch)
        tf = time_loop(lambda: hbmm.gemm_fused(dA, beta, bb, bs, beta, Cw), 10, 2, torch)
        res["fused_im2col_conv2x_b64"] = {"M": M, "K": K, "N": N, "beta": beta, "pack_then_gemm_ms": min(t2),
                                          "fused_ms": min(tf), "fused_GBs_of_A": 4.0 * M * K / (min(tf) * 1e-3) / 1e9}
        del dA, dB, Cw
    except Exception as e:
        res["fused_im2col_conv2x_b64"] = {"error": str(e)}
    return res


if __name__ == "__main__":
    main()
