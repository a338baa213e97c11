"""GPU parity under the SLI-aware randomized decode router (paper Sec. 5.2): the HIP library against the CPU
oracle through the C ABI, bit-exact, both group buffers included."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import plan as P
from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy, _lp_instance, one_class

pytestmark = pytest.mark.gpu


def _split(cfg, p_solo):
    return replace(cfg, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[float(v) for v in p_solo])


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_heavy_small_instances_with_the_randomized_router(B, oracle_mod, gate):
    """Both buffers in use, both overflowing (capacity 12 each), empty groups, B = 1, certain and impossible sides."""
    for over, ps in ((dict(), (0.8, 0.3, 0.55)), (dict(M=0), (0.8, 0.3, 0.55)), (dict(M=12), (0.8, 0.3, 0.55)),
                     (dict(B=1, M=6), (0.5, 0.5, 0.5)), (dict(M=1), (1.0, 0.0, 0.5)), (dict(N=1, M=1, B=3), (0.4, 0.4, 0.4)),
                     (dict(dbuf_cap=4096), (0.2, 0.9, 0.6))):
        cfg = _split(_heavy(gate, **over), ps)
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])
        if not over:
            assert len(orc.queue(0, -1)) + len(orc.queue(0, -2)) > 0 and os_["tally"][:, TI["DROP_D"]].sum() > 0


def test_the_split_is_the_oracle_s(B, oracle_mod):
    cfg = W.SimConfig(name="split", K=1, N=2, B=1, C=64, c0=0.010, c_pre=0.0, c_dec=0.0,
                      classes=[one_class(1.0, 60, 3)], M=1, x_star=[0.5], qp_star=[0.0], queue_cap=4096, dbuf_cap=4096,
                      replications=3, steps=5000, seed=8, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.37])
    sim, orc = run_both(B, oracle_mod, cfg, 5000, checkpoints=2)
    assert len(orc.queue(0, -2)) > 20


def test_planned_split_on_the_binding_capacity_instance(B, oracle_mod):
    cfg = _lp_instance(256, 2, 8000, (1024, 3072), (400, 160))
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    cfg = _split(cfg, P.solo_probabilities(pl))
    sim, orc = run_both(B, oracle_mod, cfg, 8000, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())


def test_every_workgroup_shape_with_the_randomized_router(B, oracle_mod):
    """One, two, four, eight and sixteen waves; routing passes that take jobs from both rings, more jobs than a pass
    stages, several gate passes per step beside routing to the mixed group, full groups and long buffers."""
    for N, M, Bcap, steps, lam, ps in ((60, 20, 8, 1500, (2.2, 1.8), (0.6, 0.4)), (100, 30, 8, 1200, (2.2, 1.8), (0.6, 0.4)),
                                       (200, 60, 8, 1000, (2.2, 1.8), (0.6, 0.4)), (700, 200, 8, 600, (2.2, 1.8), (0.6, 0.4)),
                                       (4000, 1500, 8, 200, (2.4, 2.0), (0.7, 0.2)),
                                       (8192, 5000, 8, 60, (2.5, 2.0), (0.5, 0.5)),
                                       (8192, 300, 2, 300, (2.5, 2.0), (0.9, 0.8))):
        cls = [_limits_class(lam=lam[0], out_p0=300.0), _limits_class(lam=lam[1], in_p0=40.0, out_p0=500.0)]
        cfg = _split(_limits_cfg(f"rr-shapes-{N}-{M}-{Bcap}", cls, N=N, M=M, B=Bcap, steps=steps, replications=1,
                                 dbuf_cap=2048, queue_cap=8192), ps)
        sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=2)
        t, g = orc.tallies(0)
        assert t[:, TI["U_DM"]].sum() > 0 and t[:, TI["U_DS"]].sum() > 0, N
        assert sim.stats()["overflow"] == bool(g[5])


def test_config5_width_with_the_randomized_router_on_a_sampled_replication(B, oracle_mod):
    cfg = W.config(5, replications=2, mod_period=20000)
    cfg = W.with_random_split(cfg, lam_plan=[c.lam / 0.95 for c in cfg.classes])
    assert cfg.route_mode == W.ROUTE_RANDOM_SPLIT and 0.0 <= min(cfg.p_solo) < max(cfg.p_solo) <= 1.0
    run_both(B, oracle_mod, cfg, 2500, oracle_reps=[1], checkpoints=2)


def test_bad_split_probabilities_are_rejected(B):
    with pytest.raises(B.SimError):
        B.Sim(_split(_heavy(), (0.5, 1.5, 0.5)))


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_FCFS])
def test_randomized_router_with_abandonment(B, oracle_mod, gate):
    """Both group buffers hold dead entries, are compacted and overflow; requests leave from either."""
    for over, ps in ((dict(), (0.8, 0.3, 0.55)), (dict(M=1), (1.0, 0.0, 0.5)), (dict(B=1, M=6), (0.5, 0.5, 0.5)),
                     (dict(dbuf_cap=4096, queue_cap=4096), (0.2, 0.9, 0.6)), (dict(N=1, M=1, B=1), (0.4, 0.4, 0.4))):
        cfg = _split(_heavy(gate, **over), ps)
        cfg.classes = [replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))]
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])
        if not over:
            assert os_["tally"][:, TI["AB_D"]].sum() > 0 and os_["tally"][:, TI["AB_P"]].sum() > 0


def test_randomized_router_with_abandonment_on_wide_workgroups(B, oracle_mod):
    for N, M, Bcap, steps, ps in ((700, 30, 8, 900, (0.6, 0.4)), (8192, 300, 2, 300, (0.9, 0.8)), (8192, 5000, 8, 60, (0.5, 0.5))):
        cls = [_limits_class(lam=2.4, theta=3.0, out_p0=300.0), _limits_class(lam=2.0, in_p0=40.0, out_p0=500.0, theta=9.0)]
        cfg = _split(_limits_cfg(f"ab-rr-{N}-{M}-{Bcap}", cls, N=N, M=M, B=Bcap, steps=steps, replications=1,
                                 dbuf_cap=2048, queue_cap=8192), ps)
        sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=2)
        t, g = orc.tallies(0)
        assert sim.stats()["overflow"] == bool(g[5])
        if M < 1000:
            assert t[:, TI["AB_P"]].sum() > 500
        if Bcap == 2:
            assert t[:, TI["AB_D"]].sum() > 1000
