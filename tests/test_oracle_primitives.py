"""Pins of the oracle's primitives: Philox, sampler tables, histogram bins (CPU only)."""
import os
import subprocess
import sys

import numpy as np
import pytest
from scipy import stats

PHILOX_HELPER = r"""
// Independent Philox4x32-10: PyTorch's CPU engine (counter = offset lo/hi, subsequence lo/hi; key = seed).
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  for (int i = 1; i + 2 < argc; i += 3) {
    unsigned long long seed = strtoull(argv[i], 0, 10), subseq = strtoull(argv[i + 1], 0, 10), off = strtoull(argv[i + 2], 0, 10);
    at::Philox4_32 e(seed, subseq, off);
    unsigned a = e(), b = e(), c = e(), d = e();
    printf("%u %u %u %u\n", a, b, c, d);
  }
  return 0;
}
"""


def test_philox_matches_independent_implementation(oracle_mod, tmp_path):
    """Counter (c0,c1,c2,c3) and key (seed lo, seed hi) against PyTorch's header-only engine,
    whose counter is (offset lo, offset hi, subsequence lo, subsequence hi)."""
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    src = tmp_path / "philox_ref.cpp"
    exe = tmp_path / "philox_ref"
    src.write_text(PHILOX_HELPER)
    subprocess.check_call(["g++", "-O1", "-std=c++17", f"-I{inc}", str(src), "-o", str(exe)])
    rng = np.random.default_rng(7)
    cases = [(0, 0, 0, 0, 0), (1, 0, 0, 0, 0), (1, 5, 1, 7, 3), (2**64 - 1, 2**32 - 1, 2**32 - 1, 2**32 - 1, 2**32 - 1)]
    for _ in range(60):
        cases.append((int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2)),) + tuple(int(v) for v in rng.integers(0, 2**32, 4)))
    args = []
    for seed, c0, c1, c2, c3 in cases:
        args += [str(seed), str(c2 | (c3 << 32)), str(c0 | (c1 << 32))]
    out = subprocess.check_output([str(exe)] + args, text=True).split("\n")
    for (seed, c0, c1, c2, c3), line in zip(cases, out):
        want = np.array([int(v) for v in line.split()], dtype=np.uint32)
        got = oracle_mod.philox(seed, c0, c1, c2, c3)
        assert np.array_equal(got, want), (seed, c0, c1, c2, c3)


def test_philox_words_are_uniform(oracle_mod):
    w = np.array([oracle_mod.philox(1, s, 0, g, 0) for s in range(64) for g in range(64)], dtype=np.uint64)
    for j in range(4):
        u = w[:, j] / 2.0**32
        assert stats.kstest(u, "uniform").pvalue > 1e-4
    bits = ((w[:, 0][:, None] >> np.arange(32, dtype=np.uint64)) & np.uint64(1)).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.05)


@pytest.mark.parametrize("mean", [1.0, 2.5, 64.0, 128.0, 512.0, 2000.0])
def test_geometric_table_is_the_quantile_function(oracle_mod, mean):
    """Pr(X >= k) = (1-p)^(k-1) (EC, log-survival check): the table holds the 2^16 mid-point quantiles."""
    t = oracle_mod.length_table(0, mean).astype(np.int64)
    assert t.min() >= 1 and np.all(np.diff(t) >= 0)
    ks = np.unique(np.concatenate([np.arange(1, 50), np.linspace(1, t.max(), 200).astype(int)]))
    emp = np.searchsorted(t, ks, side="right") / 65536.0
    cdf = stats.geom.cdf(ks, 1.0 / mean)
    assert np.max(np.abs(emp - cdf)) <= 1.0 / 65536 + 1e-12
    assert abs(t.mean() - mean) <= 3e-4 * mean + 1e-9


@pytest.mark.parametrize("median,sigma", [(256.0, 0.8), (4096.0, 0.8), (128.0, 1.0), (4096.0, 1.0), (16.0, 1.0)])
def test_lognormal_table_is_the_rounded_clamped_quantile_function(oracle_mod, median, sigma):
    t = oracle_mod.length_table(1, median, sigma).astype(np.int64)
    assert t.min() >= 1 and t.max() <= 32768 and np.all(np.diff(t) >= 0)
    ks = np.unique(np.geomspace(1, 32767, 300).astype(int))
    emp = np.searchsorted(t, ks, side="right") / 65536.0
    cdf = stats.lognorm.cdf(ks + 0.5, s=sigma, scale=median)   # round-to-nearest: X_int <= k  <=>  X < k + 0.5
    assert np.max(np.abs(emp - cdf)) <= 1.0 / 65536 + 1e-12
    assert np.sum(t == 32768) / 65536.0 == pytest.approx(stats.lognorm.sf(32767.5, s=sigma, scale=median), abs=1.0 / 65536)


def test_const_table(oracle_mod):
    assert np.all(oracle_mod.length_table(2, 600.0) == 600)
    assert np.all(oracle_mod.length_table(2, 0.2) == 1)
    assert np.all(oracle_mod.length_table(2, 1e9) == 32768)


def test_arrival_and_class_thresholds(oracle_mod):
    from paper_2602_02987_amd import workloads as W
    cfg = W.config(5, N=64, replications=1)
    o = oracle_mod.Oracle(cfg)
    rows = cfg.mod_period
    _, _, cthr, athr = o.tables(0, rows=rows)
    lam = sum(c.lam for c in cfg.classes)
    for row in (0, rows // 4, rows // 2, 3 * rows // 4, 12345):
        m = lam * cfg.c0 * (1.0 + cfg.mod_amp * np.sin(2 * np.pi * row / rows))
        want = stats.poisson.cdf([0, 1, 2], m) * 2.0**32
        assert np.all(np.abs(athr[row].astype(np.float64) - want) <= 2.0), row
    cum = np.cumsum([c.lam for c in cfg.classes])[:-1] / lam
    assert np.all(np.abs(cthr[:cfg.K - 1].astype(np.float64) - cum * 2.0**32) <= 2.0)


def test_histogram_bins(oracle_mod):
    edges = [oracle_mod.hedge(b) for b in range(720)]
    assert edges[:17] == list(range(17))
    assert all(b > a for a, b in zip(edges, edges[1:]))
    rng = np.random.default_rng(3)
    for v in [0, 1, 15, 16, 17, 31, 32, 10_000_000, 48_400_000, 2**40 + 12345] + [int(x) for x in rng.integers(0, 2**47, 200)]:
        b = oracle_mod.hbin(v)
        assert edges[b] <= v and (b == 719 or v < edges[b + 1])
    for b in range(16, 719):
        assert edges[b + 1] / edges[b] <= 1.0 + 1.0 / 16 + 1e-12   # 16 bins per octave
    assert oracle_mod.hbin(2**60) == 719
