"""bench.py's output contract, checked on the device with a short run: one JSON line with the metric,
the roofline of the dominant kernel and the CPU baseline, internally consistent."""
from __future__ import annotations

import json
import subprocess
import sys
from pathlib import Path

import pytest

pytestmark = pytest.mark.gpu
ROOT = Path(__file__).resolve().parent.parent


def test_bench_prints_one_consistent_json_line():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--steps", "3", "--warmup", "1", "--no-extras"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"]
    M, N, K = d["config"]["M"], d["config"]["N"], d["config"]["K"]
    assert d["value"] == pytest.approx(2.0 * M * N * K / (d["ms_per_step"] * 1e-3) / 1e9, rel=1e-9)
    rf = d["roofline"]
    assert rf["bound"] == "alu" and rf["unit"] == "TOP/s" and rf["peak"] == pytest.approx(1258.2912)
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], rel=1e-9)
    assert rf["achieved"] == pytest.approx(2.0 * M * N * K / (d["kernel_ms"]["gemm"] * 1e-3) / 1e12, rel=1e-6)
    assert 0.3 < rf["frac"] < 1.2                      # a healthy device lands near 0.85
    assert rf["traffic"] is None or rf["traffic"] > 0
    assert "profiles/" in rf["traffic_source"] and rf["algorithmic_bytes"] > 0     # where the counter figure comes from
    assert rf["traffic"] is None or rf["traffic"] >= 0.9 * rf["algorithmic_bytes"]
    rp = d["roofline_pack"]
    assert rp["bound"] == "hbm" and rp["peak"] == 8000.0 and rp["frac"] == pytest.approx(rp["achieved"] / 8000.0, rel=1e-9)
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["unit"] == d["unit"] and cb["sample"]
    assert cb["nproc"] >= 1 and "physical_cores" in cb and "cpu_model" in cb


def test_bench_comparison_rows_carry_a_bound_and_a_fraction():
    """Every row next to the headline -- the other workloads, the convolution layers, the backward --
    states which roofline bounds it and the fraction it reaches; pack figures say whether they are HBM
    figures or cache-resident ones."""
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--steps", "3", "--warmup", "1", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([ln for ln in r.stdout.splitlines() if ln.strip()][-1])
    cmp_ = d["comparisons"]
    assert "error" not in cmp_, cmp_
    for name, e in cmp_["other_workloads"].items():
        rf = e["roofline"]
        assert rf["bound"] in ("alu", "mfma") and 0 < rf["frac"] < 1.5, name
        assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"], rel=1e-9), name
        if "pack_a_ms" in e:
            assert ("pack_a_GBs" in e) != ("pack_a_GBs_cache_resident" in e), name
    assert cmp_["other_workloads"]["c5xw4"]["roofline"]["piece_products"] == 6
    assert "frac_of_epilogue_alu_bound" in cmp_["other_workloads"]["sq4k16"]["roofline"]
    for name, e in cmp_["conv2d"].items():
        assert "error" not in e, (name, e)
        if "conv_ms" in e:      # (a width that beta_a does not divide runs in the prepared-filter form only)
            assert e["roofline"]["bound"] == "mfma" and 0 < e["roofline"]["frac"] < 1.0, name
        assert "conv_prepared_error" not in e, (name, e)
        assert e["roofline_prepared"]["piece_products"] == 6 and 0 < e["roofline_prepared"]["frac"] < 1.0, name
        assert e["roofline_prepared_f16x2"]["piece_products"] == 3 and 0 < e["roofline_prepared_f16x2"]["frac"] < 1.0, name
        assert 0 < e["conv_prepared_f16x2_ms"] < e["conv_prepared_ms"], name
    # the sustained matrix-core rate lies below the published peak and above half of it
    assert 0.4 * 2500 < cmp_["mfma_bf16_sustained_TFLOPs"] < 2500
    assert 0 < cmp_["binarize_backward"]["frac_of_hbm_peak"] < 1.2
