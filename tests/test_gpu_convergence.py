"""The paper's convergence experiment (EC "Convergence Analysis"; Theorems 2 and 4) on the HIP library, at
scales the CPU oracle is too slow for: the two-class synthetic instance at n = 5 ... 8000 servers, five seeds
each. Checks what the fluid limit fixes at any size, not the paper's figures (they are plots): per-server revenue
approaches the LP optimum R* and the spread over seeds narrows, the prefill occupancies and backlogs move towards
x*, q_p*, the decode buffer empties, and under the randomized router the class-wise decode occupancies approach
y_m*, y_s*. One small scale is also compared with the oracle bit by bit."""
import numpy as np
import pytest

from paper_2602_02987_amd import plan as P
from paper_2602_02987_amd import workloads as W
from test_gpu_parity import B, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI

pytestmark = pytest.mark.gpu

WARM, MEAS = 20_000, 40_000      # 178 s and 356 s of simulated time; a decode lasts about 10 to 30 s, patience 10 s


def _measure(Bm, n, **kw):
    cfg = W.convergence_instance(n, **kw)
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes], objective="bundled" if kw.get("bundled") else "separate")
    sim = Bm.Sim(cfg)
    sim.run(WARM)
    t0 = np.stack([sim.tallies(r)[0][:cfg.K].astype(np.float64) for r in range(cfg.replications)])
    sim.run(MEAS)
    t1 = np.stack([sim.tallies(r)[0][:cfg.K].astype(np.float64) for r in range(cfg.replications)])
    assert not sim.stats()["overflow"], n
    t = t1 - t0                                             # [seed][class][tally]
    pre = "TOKP_DEC" if kw.get("bundled") else "TOKP_PRE"
    price_in = np.array([c.price_in for c in cfg.classes]); price_out = np.array([c.price_out for c in cfg.classes])
    rev = (t[:, :, TI[pre]] * price_in + t[:, :, TI["TOKD_DEC"]] * price_out).sum(axis=1) / (n * MEAS * cfg.c0)
    occ = {k: t[:, :, TI["SUM_" + k]].mean(axis=0) / (n * MEAS) for k in ("X", "QP", "QD", "YM", "YS")}
    return cfg, pl, rev, occ


def test_revenue_queues_and_occupancies_approach_the_plan(B):
    scales = (5, 50, 500, 8000)
    res = {n: _measure(B, n) for n in scales}
    pl = res[5][1]
    qp_star = np.array(res[5][0].qp_star)
    assert qp_star[0] > 1.0 and abs(qp_star[1]) < 1e-9 and pl.ys.sum() > 4.0    # class 0 is held back, decode binds
    gap = {n: abs(res[n][2].mean() / pl.value - 1.0) for n in scales}
    spread = {n: res[n][2].std() / pl.value for n in scales}
    assert gap[8000] < 0.004 and gap[500] < 0.006 and gap[5] > 0.01, gap
    assert spread[8000] < spread[500] < spread[50] < spread[5], spread
    for a, b in zip(scales, scales[1:]):                     # every figure moves towards its fluid value
        assert abs(res[b][3]["X"][0] - pl.x[0]) < abs(res[a][3]["X"][0] - pl.x[0]), (a, b)
        assert res[b][3]["QP"][0] > res[a][3]["QP"][0], (a, b)
        assert res[b][3]["QD"].sum() < res[a][3]["QD"].sum(), (a, b)
    big = res[8000][3]
    assert np.allclose(big["X"], pl.x, rtol=0.08), (big["X"], pl.x)
    assert abs(big["QP"][0] - qp_star[0]) < 0.25 * qp_star[0] and big["QP"][1] < 0.03
    assert big["QD"].sum() < 0.35
    assert (big["YM"] + big["YS"]).sum() == pytest.approx((pl.ym + pl.ys).sum(), rel=0.01)   # every decode slot in use


def test_completion_revenue_approaches_the_plan_from_below(B):
    """Bundled charging (Theorem 2): requests that give up in the decode buffer earn nothing, so the finite system
    stays below R* and closes the gap as it grows."""
    scales = (5, 50, 500, 8000)
    gap = []
    for n in scales:
        cfg, pl, rev, occ = _measure(B, n, bundled=True)
        gap.append(rev.mean() / pl.value - 1.0)
    assert all(g < 0.0 for g in gap) and gap[0] < gap[1] < gap[2] < gap[3], gap
    assert gap[0] < -0.10 and gap[3] > -0.035, gap


def test_randomized_router_brings_class_occupancies_to_the_plan(B):
    """Theorem 4: with the plan's solo probabilities the class-wise mixed and solo decode occupancies approach
    y_m*, y_s*; the solo-first router reaches the same totals with another class mix."""
    cfg, pl, rev, occ = _measure(B, 8000, random_split=True)
    assert 0.5 < cfg.p_solo[0] < 0.99 and cfg.p_solo[1] == 1.0
    assert np.allclose(occ["YM"], pl.ym, rtol=0.03, atol=0.005), (occ["YM"], pl.ym)
    assert np.allclose(occ["YS"], pl.ys, rtol=0.06), (occ["YS"], pl.ys)
    _, _, _, plain = _measure(B, 8000)
    assert abs(plain["YM"][1] - pl.ym[1]) > 0.2               # class 1 decodes on mixed servers without the split
    err_split = np.abs(occ["YS"] - pl.ys).sum() + np.abs(occ["YM"] - pl.ym).sum()
    err_plain = np.abs(plain["YS"] - pl.ys).sum() + np.abs(plain["YM"] - pl.ym).sum()
    assert err_split < 0.5 * err_plain, (err_split, err_plain)


def test_weighted_router_brings_class_occupancies_to_the_plan(B):
    """The general form of the router (weights = the plan's class shares of each pool's decode completions) reaches
    the same class-wise occupancies."""
    cfg, pl, rev, occ = _measure(B, 8000, weighted_split=True)
    assert cfg.route_mode == W.ROUTE_WEIGHTED_SPLIT and abs(sum(cfg.w_solo) - 1.0) < 1e-9
    assert np.allclose(occ["YM"], pl.ym, rtol=0.03, atol=0.005), (occ["YM"], pl.ym)
    assert np.allclose(occ["YS"], pl.ys, rtol=0.06), (occ["YS"], pl.ys)
    assert abs(rev.mean() / pl.value - 1.0) < 0.004


def test_one_scale_bit_by_bit(B, oracle_mod):
    for kw in (dict(), dict(random_split=True), dict(bundled=True), dict(weighted_split=True)):
        cfg = W.convergence_instance(50, seeds=3, **kw)
        run_both(B, oracle_mod, cfg, 12_000, checkpoints=2)
