"""Pins of the oracle's general SLI-aware router (paper EC, "General SLI-aware Extension": solo probabilities
p_s,i, one buffer per pool, and within a pool a class drawn with the weights varpi restricted to the classes that
wait, its head-of-line job taken). CPU only."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import plan as P
from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import GI, TI, _heavy, _lp_instance, one_class


def _thr32(p):
    return min(max(int(np.floor(p * 4294967296.0)), 0), 4294967295)


def _units(w):
    return min(max(int(np.floor(w * 1048576.0 + 0.5)), 1), 1048576)


def _cls(jw):
    return (int(jw) >> 29) & 7


def _weighted(cfg, **kw):
    return replace(cfg, route_mode=W.ROUTE_WEIGHTED_SPLIT, **kw)


def test_one_class_is_the_randomized_router(oracle_mod):
    """With a single class there is nothing to select: state and tallies equal those of the randomized router."""
    cls = [one_class(2.5, 300, 200)]
    base = W.SimConfig(name="ws-one", K=1, N=12, B=3, C=256, c0=0.010, c_pre=0.00005, c_dec=0.0002, classes=cls, M=4,
                       x_star=[0.3], qp_star=[0.0], queue_cap=64, dbuf_cap=16, replications=2, steps=3000, seed=9)
    a = oracle_mod.Oracle(replace(base, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.6])); a.run(3000)
    b = oracle_mod.Oracle(_weighted(base, p_solo=[0.6], w_solo=[1.0], w_mixed=[1.0])); b.run(3000)
    for r in range(2):
        assert a.digest(r) == b.digest(r)
        assert np.array_equal(a.tallies(r)[0], b.tallies(r)[0])
    assert a.tallies(0)[0][0, TI["U_DM"]] > 5 and a.tallies(0)[0][0, TI["SUM_QD"]] > 1000     # both pools, buffers in use


@pytest.mark.parametrize("over", [dict(), dict(M=1), dict(M=11), dict(B=2, M=6)])
def test_selections_replayed_step_by_step(oracle_mod, over):
    """The whole router re-stated in Python and replayed on every step's inputs (as for the base router): the
    completions of the step split by their group word, each pool's buffer, the weighted class draws from the
    pinned Philox, least-loaded placement. Placements per server and both buffers must match the oracle's."""
    p_solo, ws, wm = [0.8, 0.3, 0.55], [0.5, 0.0, 0.2], [0.1, 0.6, 0.3]      # (a zero weight: served only when alone)
    cfg = _weighted(_heavy(queue_cap=100000, dbuf_cap=100000, replications=1, **over), p_solo=p_solo, w_solo=ws, w_mixed=wm)
    units = [[_units(v) for v in ws], [_units(v) for v in wm]]
    o = oracle_mod.Oracle(cfg)
    prev_sl = {g: [] for g in range(cfg.N)}
    prev_sv = dict(rem=np.zeros(cfg.N, np.int32), pfjob=np.zeros(cfg.N, np.uint64))
    buf = [[], []]
    multi = picked_late = 0
    for s in range(1500):
        o.run(1)
        sl, sv = o.slots(0), o.servers(0)
        now = {g: sorted(int(v) for v in sl["job"][g, :sl["n_dec"][g]]) for g in range(cfg.N)}
        for g in range(cfg.N):
            if prev_sv["rem"][g] > 0 and (sv["rem"][g] == 0 or sv["pfjob"][g] != prev_sv["pfjob"][g]):
                jw = int(prev_sv["pfjob"][g])
                solo = int(oracle_mod.philox(cfg.seed, s, 10, g, 0)[1]) < _thr32(p_solo[_cls(jw)])
                buf[0 if solo else 1].append(jw)
        stayed = {}
        for g in range(cfg.N):
            a, b = list(prev_sl[g]), list(now[g])
            keep = []
            for jw in a:
                if jw in b:
                    b.remove(jw); keep.append(jw)
            stayed[g] = keep
        loads = np.array([len(stayed[g]) for g in range(cfg.N)])
        placed = {}
        for pool, (lo, hi, cap) in enumerate(((cfg.M, cfg.N, cfg.B), (0, cfg.M, cfg.B - 1))):
            j = 0
            while buf[pool]:
                cand = [g for g in range(lo, hi) if loads[g] < cap]
                if not cand:
                    break
                dst = min(cand, key=lambda g: (loads[g], g))
                waiting = sorted({_cls(jw) for jw in buf[pool]})
                total = sum(units[pool][c] for c in waiting)
                x = (int(oracle_mod.philox(cfg.seed, s, 11 + pool, j, 0)[0]) * total) >> 32
                cum = 0
                for c in waiting:
                    cum += units[pool][c]
                    if x < cum:
                        break
                i = next(i for i, jw in enumerate(buf[pool]) if _cls(jw) == c)
                multi += len(waiting) > 1
                picked_late += i > 0
                placed.setdefault(dst, []).append(buf[pool].pop(i))
                loads[dst] += 1
                j += 1
        for g in range(cfg.N):
            assert sorted(stayed[g] + placed.get(g, [])) == now[g], (over, s, g)
        assert [int(v) for v in o.queue(0, -1)] == buf[0], (over, s)
        assert [int(v) for v in o.queue(0, -2)] == buf[1], (over, s)
        prev_sl = now
        prev_sv = dict(rem=sv["rem"].copy(), pfjob=sv["pfjob"].copy())
    assert multi > 40 and picked_late > 20, (over, multi, picked_late)   # the class draw mattered


def test_class_shares_of_a_saturated_pool_follow_the_weights(oracle_mod):
    """While every class waits in the solo pool's buffer, each freed solo slot goes to class i with probability
    varpi_s,i: over many placements the class shares of the placements approach the weights (binomial error)."""
    cls = [one_class(1.2, 40, 30), one_class(1.2, 40, 30), one_class(1.2, 40, 30)]
    cfg = W.SimConfig(name="ws-shares", K=3, N=40, B=4, C=256, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=36,
                      x_star=[0.25, 0.25, 0.25], qp_star=[0.0] * 3, queue_cap=4096, dbuf_cap=200000, replications=4,
                      steps=40000, seed=3)
    w = [0.6, 0.3, 0.1]
    o = oracle_mod.Oracle(_weighted(cfg, p_solo=[1.0, 1.0, 1.0], w_solo=w, w_mixed=[1 / 3] * 3))
    o.run(5000)
    t0 = o.stats()["tally"].astype(np.float64)
    o.run(35000)
    t = o.stats()["tally"].astype(np.float64) - t0
    assert min(len([1 for jw in o.queue(r, -1) if _cls(jw) == c]) for r in range(4) for c in range(3)) > 50   # all wait
    n = t[:3, TI["U_DS"]]
    share = n / n.sum()
    sigma = np.sqrt(np.array(w) * (1 - np.array(w)) / n.sum())
    assert n.sum() > 20000 and np.all(np.abs(share - w) < 5 * sigma), (share, sigma)


def test_invariants_and_bad_weights(oracle_mod):
    for over in (dict(), dict(M=1), dict(B=1, M=6)):
        cfg = _weighted(_heavy(**over), p_solo=[0.8, 0.3, 0.55], w_solo=[0.5, 0.3, 0.2], w_mixed=[0.1, 0.6, 0.3])
        cfg = replace(cfg, classes=[replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))])
        o = oracle_mod.Oracle(cfg)
        o.set_check(1)
        o.run(cfg.steps)
        assert o.violations() == (0, 0), over
    t, g = o.tallies(0)
    assert t[:, TI["AB_D"]].sum() > 0
    with pytest.raises(ValueError):
        oracle_mod.Oracle(_weighted(_heavy(), p_solo=[0.5, 0.5, 0.5], w_solo=[0.5, 1.5, 0.2], w_mixed=[0.3, 0.3, 0.4]))
    with pytest.raises(ValueError):
        oracle_mod.Oracle(replace(_heavy(), route_mode=4))


def test_plan_weights_are_the_pools_class_shares():
    cfg = _lp_instance(256, 1, 1000, (1024, 3072), (400, 160))
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    ws, wm = P.selection_weights(pl)
    assert ws.sum() == pytest.approx(1.0) and wm.sum() == pytest.approx(1.0)
    assert np.allclose(ws, pl.mu_s * pl.ys / (pl.mu_s * pl.ys).sum()) and np.allclose(wm, pl.mu_m * pl.ym / (pl.mu_m * pl.ym).sum())
    c2 = W.with_weighted_split(cfg)
    assert c2.route_mode == W.ROUTE_WEIGHTED_SPLIT and c2.w_solo == [float(v) for v in ws] and c2.p_solo == [float(v) for v in P.solo_probabilities(pl)]
