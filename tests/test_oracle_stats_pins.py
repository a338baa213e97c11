"""Pins of the figures oracle_stats derives from the tallies (CPU only): revenue under the per-class choice of
bundled or separate charging (paper Sec. 2.3), the fairness indicators of Sec. 5.2, utilisation, waits, occupancy
means and latency percentiles. Two sources outside the oracle: a hand-computed two-request instance
(tests/golden/two_class_stats.txt) and, on a long overloaded run, a restatement in numpy from the raw tallies and
histograms with the paper's definitions written out (max over pairs, sorted samples)."""
import os

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import GI, GOLDEN, TI, _heavy, one_class


def _two_class_cfg():
    cls = [one_class(2.0, 600, 3, price_in=1.0, price_out=1.0, bundled=1),
           one_class(2.0, 100, 2, price_in=0.5, price_out=2.0, bundled=0)]
    return W.SimConfig(name="two-class", K=2, N=2, B=2, C=256, c0=0.010, c_pre=0.00005, c_dec=0.0002, classes=cls, M=1,
                       x_star=[0.1, 0.1], qp_star=[0.0, 0.0], queue_cap=16, dbuf_cap=16)


def _seed_with_the_two_arrivals(oracle_mod, cfg):
    """A seed whose arrivals in steps 0..10 are exactly: one of class 0 in step 0, one of class 1 in step 2."""
    want = {0: (1, 0), 2: (0, 1)}
    for cand in range(1, 200000):
        o = oracle_mod.Oracle(cfg, max_reps=1)
        prev = np.zeros(2, dtype=np.int64)
        ok = True
        for s in range(11):
            o.run(1, 1, cand)
            a = o.tallies(0)[0][:, TI["A"]].astype(np.int64)
            if tuple(a - prev) != want.get(s, (0, 0)):
                ok = False
                break
            prev = a
        del o
        if ok:
            return cand
    raise AssertionError("no seed with the wanted arrival pattern")


def test_two_class_example_by_hand(oracle_mod):
    cfg = _two_class_cfg()
    seed = _seed_with_the_two_arrivals(oracle_mod, cfg)
    expect = {}
    for line in open(os.path.join(GOLDEN, "two_class_stats.txt")):
        if line.startswith("#") or not line.strip():
            continue
        steps, field, k, num, _slash, den = line.split()
        expect.setdefault(int(steps), []).append((field, None if k == "-" else int(k), float(num) / float(den)))
    assert sorted(expect) == [10, 11] and sum(len(v) for v in expect.values()) == 77
    o = oracle_mod.Oracle(cfg, max_reps=1)
    o.set_check(1)
    done = 0
    for steps in sorted(expect):
        o.run(steps - done, 1, seed)
        done = steps
        st = o.stats()
        for field, k, value in expect[steps]:
            got = st[field] if k is None else st[field][k]
            assert got == pytest.approx(value, rel=1e-12, abs=1e-300), (steps, field, k, got, value)
    assert o.violations() == (0, 0)
    t, g = o.tallies(0)
    assert [int(v) for v in t[:, TI["WAIT_STEPS"]]] == [0, 4]
    assert int(g[GI["ITERS_MIX"]]) == 4 and int(g[GI["ITERS_SOLO"]]) == 3


def _percentile_from_hist(hist, q, hedge):
    """Lower edge of the bin that holds the sample of rank ceil(q n / 100), by expanding the histogram."""
    bins = np.repeat(np.arange(hist.size), hist.astype(np.int64))
    if bins.size == 0:
        return 0.0
    rank = -(-q * bins.size // 100)
    return hedge(int(bins[rank - 1])) * 1e-9


@pytest.mark.parametrize("over", [dict(), dict(M=12), dict(M=2, B=3)])
def test_derived_figures_restated_from_raw_tallies(oracle_mod, over):
    """Every derived field of oracle_stats on a long overloaded run of three classes with different prices and
    charging rules, recomputed here from the per-replication tallies and histograms."""
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, **over)
    o = oracle_mod.Oracle(cfg)
    o.run(4000)
    st = o.stats()
    K, R = cfg.K, cfg.replications
    t = sum(o.tallies(r)[0].astype(np.float64) for r in range(R))
    g = sum(o.tallies(r)[1].astype(np.float64) for r in range(R))
    hists = [sum(o.hist(r, w).astype(np.int64) for r in range(R)) for w in range(3)]
    dt = cfg.c0
    server_time = cfg.N * 4000 * dt * R
    server_steps = cfg.N * 4000 * R
    col = lambda name: t[:, TI[name]]
    done = col("S_DM") + col("S_DS")
    approx = lambda v: pytest.approx(v, rel=1e-12, abs=1e-300)
    bundled = np.array([c.price_in * col("TOKP_DEC")[k] + c.price_out * col("TOKD_DEC")[k] for k, c in enumerate(cfg.classes)])
    separate = np.array([c.price_in * col("TOKP_PRE")[k] + c.price_out * col("TOKD_DEC")[k] for k, c in enumerate(cfg.classes)])
    flags = [c.bundled for c in cfg.classes]
    assert flags == [1, 0, 1]                                       # both charging rules occur
    mixed = np.where(np.array(flags) == 1, bundled, separate)
    assert np.all(bundled != separate)                               # requests are in flight: the two rules differ
    for k in range(K):
        assert st["rev_mixed"][k] == approx(mixed[k] / server_time)
        assert st["arrival_rate"][k] == approx(col("A")[k] / server_time)
        assert st["completion_rate"][k] == approx(done[k] / server_time)
        assert st["served_fraction"][k] == approx(done[k] / col("A")[k])
        assert st["tok_rate_prefill"][k] == approx(col("TOK_PREF")[k] / server_time)
        assert st["tok_rate_decode"][k] == approx(col("TOK_EMIT")[k] / server_time)
        assert st["mean_wait"][k] == approx(col("WAIT_STEPS")[k] * dt / col("U_P")[k])
        assert st["e2e_mean"][k] == approx(col("E2E_SUM")[k] * 1e-9 / done[k])
        assert st["tbt_mean"][k] == approx(col("TBT_SUM")[k] * 1e-9 / col("TOK_EMIT")[k])
        for name, tally in (("mean_qp", "SUM_QP"), ("mean_qd", "SUM_QD"), ("mean_x", "SUM_X"), ("mean_ym", "SUM_YM"),
                            ("mean_ys", "SUM_YS")):
            assert st[name][k] == approx(col(tally)[k] / server_steps)
        for w, pre in enumerate(("ttft", "e2e", "tbt")):
            for q in (50, 95, 99):
                assert st[f"{pre}_p{q}"][k] == approx(_percentile_from_hist(hists[w][k], q, oracle_mod.hedge))
    assert st["rev_mixed_total"] == approx(mixed.sum() / server_time)
    assert st["rev_bundled_total"] == approx(bundled.sum() / server_time)
    assert st["rev_separate_total"] == approx(separate.sum() / server_time)
    x = col("SUM_X") / server_steps
    ys = col("SUM_YS") / server_steps
    assert st["fair_gap_x"] == approx(max(x[i] - x[j] for i in range(K) for j in range(K)))       # Sec. 5.2
    assert st["fair_gap_ys"] == approx(max(ys[i] - ys[j] for i in range(K) for j in range(K)))
    assert st["fair_gap_x"] > 0 and (st["fair_gap_ys"] > 0 or cfg.M == cfg.N)
    assert st["fair_min_served"] == approx(min(done[k] / col("A")[k] for k in range(K)))
    assert st["util_mix"] == approx(g[GI["BUSY_MIX"]] * 1e-9 / server_time)
    assert st["util_solo"] == approx(g[GI["BUSY_SOLO"]] * 1e-9 / server_time)
    assert st["iter_rate"] == approx((g[GI["ITERS_MIX"]] + g[GI["ITERS_SOLO"]]) / server_time)
    assert 0 < st["util_mix"] + st["util_solo"] <= 1.0 + 1e-9
