"""GPU parity under the general SLI-aware router (paper EC, "General SLI-aware Extension": solo probabilities,
one buffer per pool, weighted class selection among the classes that wait, FCFS within a class): the HIP library
against the CPU oracle through the C ABI, bit-exact, both pool buffers included."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy, _lp_instance

pytestmark = pytest.mark.gpu


def _weighted(cfg, p_solo, w_solo, w_mixed, thetas=None):
    cfg = replace(cfg, route_mode=W.ROUTE_WEIGHTED_SPLIT, p_solo=[float(v) for v in p_solo],
                  w_solo=[float(v) for v in w_solo], w_mixed=[float(v) for v in w_mixed])
    if thetas is not None:
        cfg = replace(cfg, classes=[replace(c, theta=float(t)) for c, t in zip(cfg.classes, thetas)])
    return cfg


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_FCFS])
@pytest.mark.parametrize("thetas", [None, (4.0, 0.0, 25.0)])
def test_heavy_small_instances_with_the_weighted_router(B, oracle_mod, gate, thetas):
    """Both buffers in use and overflowing, with and without abandonment, empty groups, B = 1, a zero weight,
    one-sided solo probabilities."""
    for over, ps, ws, wm in ((dict(), (0.8, 0.3, 0.55), (0.5, 0.3, 0.2), (0.1, 0.6, 0.3)),
                             (dict(M=0), (0.8, 0.3, 0.55), (0.5, 0.3, 0.2), (0.1, 0.6, 0.3)),
                             (dict(M=12), (0.8, 0.3, 0.55), (0.5, 0.3, 0.2), (0.1, 0.6, 0.3)),
                             (dict(B=1, M=6), (0.5, 0.5, 0.5), (1.0, 0.0, 0.0), (0.0, 0.0, 1.0)),
                             (dict(M=1), (1.0, 0.0, 0.5), (0.2, 0.2, 0.6), (0.6, 0.2, 0.2)),
                             (dict(N=1, M=1, B=3), (0.4, 0.4, 0.4), (0.3, 0.3, 0.4), (0.3, 0.3, 0.4)),
                             (dict(dbuf_cap=4096), (0.2, 0.9, 0.6), (0.05, 0.9, 0.05), (0.4, 0.2, 0.4)),
                             (dict(dbuf_cap=3, queue_cap=5), (0.6, 0.5, 0.4), (0.5, 0.3, 0.2), (0.1, 0.6, 0.3))):
        cfg = _weighted(_heavy(gate, **over), ps, ws, wm, thetas)
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])
        if not over:
            assert os_["tally"][:, TI["SUM_QD"]].sum() > 1000 and os_["tally"][:, TI["DROP_D"]].sum() > 0


def test_weights_from_the_plan_on_the_binding_capacity_instance(B, oracle_mod):
    cfg = W.with_weighted_split(_lp_instance(256, 2, 8000, (1024, 3072), (400, 160)))
    assert cfg.route_mode == W.ROUTE_WEIGHTED_SPLIT
    sim, orc = run_both(B, oracle_mod, cfg, 8000, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())
    for c in cfg.classes:
        c.theta = 0.5
    sim, orc = run_both(B, oracle_mod, cfg, 8000, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())


def test_every_workgroup_shape_with_the_weighted_router(B, oracle_mod):
    """One, two, eight and sixteen waves; passes that take requests from both buffers, more requests than a pass
    stages, long buffers in which the chosen class sits far behind the head."""
    for N, M, Bcap, steps, lam, ps, th in ((60, 20, 8, 1500, (2.2, 1.8), (0.6, 0.4), 0.0),
                                           (700, 200, 8, 600, (2.2, 1.8), (0.6, 0.4), 3.0),
                                           (4000, 1500, 8, 200, (2.4, 2.0), (0.7, 0.2), 0.0),
                                           (8192, 5000, 8, 60, (2.5, 2.0), (0.5, 0.5), 3.0),
                                           (8192, 300, 2, 300, (2.5, 2.0), (0.9, 0.8), 0.0),
                                           (8192, 300, 2, 300, (2.5, 2.0), (0.9, 0.8), 9.0)):
        cls = [_limits_class(lam=lam[0], out_p0=300.0, theta=th), _limits_class(lam=lam[1], in_p0=40.0, out_p0=500.0, theta=th)]
        cfg = _weighted(_limits_cfg(f"ws-shapes-{N}-{M}-{Bcap}", cls, N=N, M=M, B=Bcap, steps=steps, replications=1,
                                    dbuf_cap=2048, queue_cap=8192), ps, (0.85, 0.15), (0.3, 0.7))
        sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=2)
        assert sim.stats()["overflow"] == bool(orc.tallies(0)[1][5])


def test_bad_weights_are_rejected(B):
    good = _weighted(_heavy(), (0.5, 0.5, 0.5), (0.3, 0.3, 0.4), (0.3, 0.3, 0.4))
    B.Sim(good)
    for bad in (replace(good, w_solo=[0.3, 1.3, 0.4]), replace(good, w_mixed=[-0.1, 0.5, 0.6]), replace(good, p_solo=[0.5, 2.0, 0.5]),
                replace(good, route_mode=4)):
        with pytest.raises(B.SimError):
            B.Sim(bad)


def test_config5_width_with_the_weighted_router_on_a_sampled_replication(B, oracle_mod):
    """Config 5 at its full width, the plan's solo probabilities and weights, impatient classes, eight decode
    slots per server (so that both buffers fill within the run) and a moving split."""
    cfg = W.with_weighted_split(W.config(5, replications=2, mod_period=20000), lam_plan=None)
    cfg = replace(cfg, B=8)
    for c in cfg.classes:
        c.theta = 0.5
    reps = cfg.replications
    sim = B.Sim(cfg, max_replications=reps); orc = oracle_mod.Oracle(cfg, max_reps=reps); orc.select([1])
    from parity import assert_replication_equal
    for n, m in ((700, None), (700, cfg.M * 2), (600, cfg.M // 2)):
        if m is not None:
            sim.set_split(m); orc.set_split(m)
        sim.run(n, reps); orc.run(n, reps)
        assert_replication_equal(sim, orc, 1, what="cfg5 width, weighted router")
    t, _ = orc.tallies(1)
    assert t[:, TI["AB_D"]].sum() > 100 and t[:, TI["U_DM"]].sum() > 1000 and t[:, TI["SUM_QD"]].sum() > 100000
