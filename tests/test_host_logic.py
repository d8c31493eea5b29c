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
        assert (c.C * c.KH * c.KW) % c.beta_w == 0 and (c.C * c.KH * c.KW) % 32 == 0
        # a width that beta_a does not divide is the one layer kept for the prepared-filter form (7 x 7 maps)
        assert c.W % c.beta_a == 0 or c.name.startswith("conv5x")
        assert (c.batch * c.C * c.H * c.W) % 128 == 0 and c.KH * c.KW <= 32


def test_workgroup_to_tile_map_covers_every_tile_once(tmp_path):
    """The XCD-balanced workgroup -> tile map of the tiled products (csrc/tile_map.h), built for the
    host: over ragged grids every tile is produced exactly once, every XCD gets the same share (+-1),
    and consecutive workgroups of one XCD stay inside few super-tiles."""
    src = tmp_path / "map_check.cpp"
    src.write_text(r'''
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "tile_map.h"
int main(int argc, char **argv) {
    const int tp = atoi(argv[1]), tq = atoi(argv[2]), sup_p = atoi(argv[3]), sup_q = atoi(argv[4]);
    // sup_q == 0: the popcount product's map (128-tile super-tiles, plain for sup_p == 0); else the general one
    auto map = [&](int b, int &p, int &q) {
        return sup_q == 0 ? hbmm::popcount_map_tile(b, tp, tq, sup_p, p, q) : hbmm::xcd_map_tile(b, tp, tq, sup_p, sup_q, p, q);
    };
    const long long blocks = sup_q == 0 ? hbmm::popcount_map_blocks(tp, tq, sup_p) : hbmm::xcd_map_blocks((long long)tp * tq);
    const int window = sup_q == 0 ? 128 : sup_p * sup_q;
    std::vector<int> seen((size_t)tp * tq, 0);
    long long per_xcd[8] = {0};
    long long none = 0, windows_bad = 0;
    for (long long b = 0; b < blocks; ++b) {
        int p = -1, q = -1;
        if (!map((int)b, p, q)) { ++none; continue; }
        if (p < 0 || p >= tp || q < 0 || q >= tq) { printf("out of range at %lld\n", b); return 1; }
        ++seen[(size_t)q * tp + p];
        ++per_xcd[b % 8];
    }
    for (int v : seen) if (v != 1) { printf("tile seen %d times\n", v); return 1; }
    long long lo = per_xcd[0], hi = per_xcd[0];
    for (long long v : per_xcd) { lo = v < lo ? v : lo; hi = v > hi ? v : hi; }
    if (sup_p != 0) {
        // one super-tile's worth of consecutive workgroups of one XCD: distinct P tiles + distinct Q tiles they touch
        for (int x = 0; x < 8; ++x)
            for (long long s = 0; (s + window) * 8 <= blocks; s += window) {
                std::vector<char> ps(tp, 0), qs(tq, 0);
                int np = 0, nq = 0, p, q;
                for (long long j = s; j < s + window; ++j)
                    if (map((int)(j * 8 + x), p, q)) {
                        if (!ps[p]) { ps[p] = 1; ++np; }
                        if (!qs[q]) { qs[q] = 1; ++nq; }
                    }
                if (np + nq > 3 * (sup_p + window / sup_p)) ++windows_bad;
            }
    }
    printf("%lld %lld %lld %lld %lld\n", blocks, none, lo, hi, windows_bad);
    return 0;
}
''')
    exe = tmp_path / "map_check"
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", str(ROOT / "paper_1905_10759_amd" / "csrc"), str(src), "-o", str(exe)],
                   check=True, timeout=120)
    for tp, tq, sup_p, sup_q in [(64, 128, 16, 0), (48, 96, 16, 0), (33, 67, 16, 0), (17, 1000, 16, 0), (5, 700, 4, 0),
                                 (3, 999, 2, 0), (1, 4099, 1, 0), (363, 727, 16, 0), (32, 64, 0, 0), (7, 11, 0, 0),
                                 (16, 129, 16, 0), (100, 3, 16, 0),
                                 # the matrix-core kernels' 8 x 4 super-tiles
                                 (32, 32, 8, 4), (48, 9, 8, 4), (5, 32, 8, 4), (1, 1, 8, 4), (3, 2, 8, 4), (182, 182, 8, 4)]:
        r = subprocess.run([str(exe), str(tp), str(tq), str(sup_p), str(sup_q)], capture_output=True, text=True, timeout=120)
        assert r.returncode == 0, (tp, tq, sup_p, r.stdout)
        blocks, none, lo, hi, bad = map(int, r.stdout.split())
        assert blocks - none == tp * tq and none < 8, (tp, tq, sup_p)
        assert hi - lo <= 1 or sup_p == 0, (tp, tq, sup_p, lo, hi)
        assert bad == 0, (tp, tq, sup_p, bad)
