"""Host-side logic that needs no GPU: the input generators, the benchmark's refusal of more than one
GPU, and the layout helpers the binding and the oracle must agree on."""
from __future__ import annotations

import subprocess
import sys
from pathlib import Path

import numpy as np

import oracle
from paper_1905_10759_amd import synth

ROOT = Path(__file__).resolve().parent.parent


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr + r.stdout


def test_generators_are_seeded_and_independent_of_chunking():
    a = synth.normal(42, (3, 1000))
    b = synth.normal(42, (3000,))
    assert np.array_equal(a.reshape(-1), b)                       # value i depends on (seed, i) only
    assert not np.array_equal(a, synth.normal(43, (3, 1000)))
    u = synth.uniform_pm1(7, (100000,))
    assert u.min() >= -1.0 and u.max() < 1.0 and abs(float(u.mean())) < 0.02
    n = synth.normal(8, (200000,))
    assert abs(float(n.mean())) < 0.01 and abs(float(n.std()) - 1.0) < 0.01
    r = synth.relu_normal(9, (100000,))
    assert r.min() == 0.0 and 0.45 < float((r == 0).mean()) < 0.55
    assert not np.signbit(r[r == 0]).any()                        # +0.0, so that Sign(0) = +1 is what gets exercised


def test_workload_tables_satisfy_the_library_constraints():
    for w in synth.WORKLOADS.values():
        assert w.K % 32 == 0 and w.K % max(w.beta_a, 1) == 0 and w.K % w.beta_w == 0
        assert oracle.ld_words(w.K) % 4 == 0 and oracle.ld_words(w.K) * 32 >= w.K
    for c in synth.CONV_WORKLOADS.values():
        assert c.W % c.beta_a == 0 and (c.C * c.KH * c.KW) % c.beta_w == 0 and (c.C * c.KH * c.KW) % 32 == 0
        assert (c.batch * c.C * c.H * c.W) % 128 == 0 and c.KH * c.KW <= 32
