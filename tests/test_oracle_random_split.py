"""Pins of the oracle's SLI-aware randomized decode router (paper Sec. 5.2: a class-i decode goes to the solo group
with probability p_s,i, else to the mixed group; each group has its own buffer). CPU only."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import plan as P
from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import GI, TI, _heavy, _lp_instance, one_class


def _thr32(p):
    return min(int(np.floor(p * 4294967296.0)), 4294967295)


def test_the_split_follows_word_1_of_the_completion_block(oracle_mod):
    """One mixed server with B = 1 (no decode slot of its own) and one solo server: every prefill completes on
    server 0, the jobs sent to the mixed group wait for ever, so the mixed buffer lists exactly the completions
    whose word 1 of block (step, stream 10, server 0, replication) is not below floor(p_s * 2^32)."""
    p_s = 0.37
    cfg = W.SimConfig(name="split", K=1, N=2, B=1, C=64, c0=0.010, c_pre=0.0, c_dec=0.0,
                      classes=[one_class(1.0, 60, 3)], M=1, x_star=[0.5], qp_star=[0.0], queue_cap=4096, dbuf_cap=4096,
                      replications=3, steps=5000, seed=8, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[p_s])
    o = oracle_mod.Oracle(cfg)
    o.set_check(1)
    sp = np.zeros((cfg.replications, cfg.steps), dtype=np.int64)
    for s in range(cfg.steps):
        o.run(1)
        for r in range(cfg.replications):
            sp[r, s] = o.tallies(r)[0][0, TI["S_P"]]
    assert o.violations() == (0, 0)
    n_solo = n_all = 0
    for r in range(cfg.replications):
        done = np.nonzero(np.diff(sp[r], prepend=0))[0]
        to_mixed = [s for s in done if int(oracle_mod.philox(cfg.seed, int(s), 10, 0, r)[1]) >= _thr32(p_s)]
        waiting = o.queue(r, -2)
        assert len(waiting) == len(to_mixed) > 20
        t, _ = o.tallies(r)
        assert t[0, TI["U_DM"]] == 0                       # nothing is ever placed on the mixed server
        assert t[0, TI["U_DS"]] + len(o.queue(r, -1)) == len(done) - len(to_mixed)
        sv = o.slots(r)
        assert sv["n_dec"][0] == 0
        n_solo += len(done) - len(to_mixed); n_all += len(done)
    assert abs(n_solo / n_all - p_s) < 4.0 * np.sqrt(p_s * (1 - p_s) / n_all)


def test_groups_do_not_share_their_buffers(oracle_mod):
    """p_s = 1: the mixed group never holds a decode even while the solo group is full and its buffer long;
    p_s = 0: the solo group stays empty."""
    base = _heavy(queue_cap=4096, dbuf_cap=4096)
    for p_s in (1.0, 0.0):
        cfg = replace(base, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[p_s] * base.K)
        o = oracle_mod.Oracle(cfg)
        o.set_check(1)
        o.run(3000)
        assert o.violations() == (0, 0)
        for r in range(cfg.replications):
            nd = o.slots(r)["n_dec"]
            t, _ = o.tallies(r)
            # one job in 2^32 still takes the other side at p_s = 1 (the threshold is a 32-bit integer): none here
            if p_s == 1.0:
                assert nd[:cfg.M].sum() == 0 and t[:, TI["U_DM"]].sum() == 0 and len(o.queue(r, -2)) == 0
                assert nd[cfg.M:].min() == cfg.B and len(o.queue(r, -1)) > 50      # saturated, jobs wait
            else:
                assert nd[cfg.M:].sum() == 0 and len(o.queue(r, -1)) == 0
                assert t[:, TI["U_DM"]].sum() + t[:, TI["U_DS"]].sum() > 0


def test_solo_only_split_equals_solo_first_routing_while_the_solo_group_has_room(oracle_mod):
    """With p_s = 1 and a solo group that never fills, the randomized router and the solo-first router make the
    same placements: identical state digests and tallies."""
    cfg = W.config(2, N=64, replications=2, steps=4000)
    a = oracle_mod.Oracle(cfg); a.run(4000)
    b = oracle_mod.Oracle(replace(cfg, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[1.0, 1.0])); b.run(4000)
    for r in range(cfg.replications):
        assert a.tallies(r)[0][:, TI["U_DM"]].sum() == 0       # the solo-first router never needed the mixed group
        assert a.digest(r) == b.digest(r)
        assert np.array_equal(a.tallies(r)[0], b.tallies(r)[0])


def test_decode_occupancies_track_the_planned_split(oracle_mod):
    """Occupancy convergence under the randomized router (Sec. 5.2): on the binding-capacity instance the
    time-averaged mixed and solo decode occupancies of every class approach y_m*, y_s* of the plan, and the
    decode buffers stay short; the solo-first router, by contrast, fills the solo pool without regard to class."""
    cfg = _lp_instance(256, 1, 60000, (1024, 3072), (400, 160))
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    ps = P.solo_probabilities(pl)
    assert np.any((ps > 0.1) & (ps < 0.9)) and pl.ym.sum() > 1.0 and pl.ys.sum() > 1.0   # a genuine split
    cfg = replace(cfg, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[float(v) for v in ps])
    o = oracle_mod.Oracle(cfg)
    o.run(20000); s0 = o.stats()
    o.run(40000); s1 = o.stats()
    t = s1["tally"].astype(np.float64) - s0["tally"].astype(np.float64)
    ns = cfg.N * cfg.replications * 40000
    ym = t[:cfg.K, TI["SUM_YM"]] / ns; ys = t[:cfg.K, TI["SUM_YS"]] / ns
    # split of each class's decode tokens between the pools = split of mu*y in the plan
    share = ys * pl.mu_s / (ys * pl.mu_s + ym * pl.mu_m)
    assert np.allclose(share, ps, atol=0.03)
    assert np.allclose(ym + ys, pl.ym + pl.ys, rtol=0.08)


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_FCFS])
def test_invariants_hold_every_step_under_the_randomized_router(oracle_mod, gate):
    for over in (dict(), dict(M=1), dict(B=1, M=6), dict(M=11)):
        cfg = replace(_heavy(gate, **over), route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.8, 0.3, 0.55])
        o = oracle_mod.Oracle(cfg)
        o.set_check(1)
        o.run(cfg.steps)
        assert o.violations() == (0, 0), over
        t, g = o.tallies(0)
        if not over:
            assert g[GI["OVERFLOW"]] == 1 and t[:, TI["DROP_D"]].sum() > 0 and t[:, TI["U_DM"]].sum() > 0


def test_bad_split_probabilities_are_rejected(oracle_mod):
    cfg = replace(_heavy(), route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.5, 1.5, 0.2])
    with pytest.raises(ValueError):
        oracle_mod.Oracle(cfg)
    with pytest.raises(ValueError):
        oracle_mod.Oracle(replace(_heavy(), route_mode=4))
