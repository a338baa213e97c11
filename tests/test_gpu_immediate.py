"""GPU parity under immediate same-slot decode (route_mode IMMEDIATE: the "I" decode rule of the paper's ablation
study, with every server in the mixed group for the "WSP" policies)."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_heavy_small_instances_with_immediate_decode(B, oracle_mod, gate):
    for over in (dict(M=12), dict(M=12, B=1), dict(M=12, B=2), dict(M=5), dict(M=12, queue_cap=4096), dict(N=1, M=1, B=3)):
        cfg = replace(_heavy(gate, **over), route_mode=W.ROUTE_IMMEDIATE)
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])
        assert os_["tally"][:, TI["SUM_QD"]].sum() == 0 and os_["tally"][:, TI["U_DS"]].sum() > 0


def test_immediate_decode_with_abandonment_and_a_moving_split(B, oracle_mod):
    cfg = replace(_heavy(M=12), route_mode=W.ROUTE_IMMEDIATE)
    cfg.classes = [replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))]
    sim = B.Sim(cfg); orc = oracle_mod.Oracle(cfg)
    from parity import assert_replication_equal
    for m, steps in ((None, 500), (4, 500), (12, 500), (8, 400)):
        if m is not None:
            sim.set_split(m); orc.set_split(m)
        sim.run(steps); orc.run(steps)
        for r in range(cfg.replications):
            assert_replication_equal(sim, orc, r, what=f"immediate, M={m}")
    assert orc.stats()["tally"][:, TI["AB_P"]].sum() > 0


def test_every_workgroup_shape_with_immediate_decode(B, oracle_mod):
    """Every server mixed (the policies without static planning): one, two, eight and sixteen waves, rows that
    fill to B, several gate passes per step."""
    for N, Bcap, steps, lam in ((60, 8, 1500, (2.2, 1.8)), (700, 8, 600, (2.2, 1.8)), (4000, 8, 200, (2.4, 2.0)),
                                (8192, 4, 120, (2.5, 2.0)), (3000, 128, 400, (2.4, 2.0))):
        cls = [_limits_class(lam=lam[0], out_p0=300.0), _limits_class(lam=lam[1], in_p0=40.0, out_p0=500.0)]
        cfg = replace(_limits_cfg(f"im-shapes-{N}-{Bcap}", cls, N=N, M=N, B=Bcap, steps=steps, replications=1,
                                  queue_cap=16384), route_mode=W.ROUTE_IMMEDIATE)
        sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=2)
        t, _ = orc.tallies(0)
        assert t[:, TI["U_DS"]].sum() > 100
        if Bcap <= 8:
            assert orc.slots(0)["n_dec"].max() == Bcap


def test_config5_width_with_immediate_decode(B, oracle_mod):
    cfg = W.config(5, replications=2, mod_period=20000)
    cfg = replace(cfg, M=3000, route_mode=W.ROUTE_IMMEDIATE)
    run_both(B, oracle_mod, cfg, 2000, oracle_reps=[1], checkpoints=2)
