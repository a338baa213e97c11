"""GPU parity with abandonment (paper Sec. 2.3: exponential patience in the prefill queues and in the decode
buffer): the HIP library against the CPU oracle through the C ABI, bit-exact, deadlines of the waiting requests
included."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy, one_class

pytestmark = pytest.mark.gpu


def _impatient(cfg, thetas):
    cfg.classes = [replace(c, theta=float(th)) for c, th in zip(cfg.classes, thetas)]
    return cfg


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_heavy_small_instances_with_abandonment(B, oracle_mod, gate):
    """Overloaded small instances, one patient class among two impatient ones: rings of 8 to 40 entries fill with
    dead entries and are compacted, the gate and the router skip dead entries, drops still follow the live counts."""
    for over in (dict(), dict(M=0), dict(M=12), dict(B=1, M=6), dict(name="heavy-prefill", M=1, queue_cap=8),
                 dict(N=1, M=1, B=3), dict(N=1, M=1, B=1)):
        cfg = _impatient(_heavy(gate, **over), (4.0, 0.0, 25.0))
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])
        if not over or "queue_cap" in over:
            assert os_["tally"][:, TI["AB_P"]].sum() > 0
    t = orc.stats()["tally"]
    assert t[:, TI["AB_D"]].sum() > 0   # the last instance has no decode slot at all


def test_queues_nobody_leaves_by_service(B, oracle_mod):
    cls = [replace(one_class(1.1, 100, 10), theta=5.0), replace(one_class(0.7, 100, 10), theta=12.0)]
    cfg = W.SimConfig(name="ab-nogate", K=2, N=24, B=4, C=64, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=0,
                      x_star=[0.1, 0.1], qp_star=[0.0, 0.0], queue_cap=4096, dbuf_cap=16, replications=2, steps=1500,
                      seed=21)
    run_both(B, oracle_mod, cfg, 1500, checkpoints=3)
    cls = [replace(one_class(2.0, 60, 5), theta=8.0)]
    cfg = W.SimConfig(name="ab-noroute", K=1, N=1, B=1, C=64, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=1,
                      x_star=[0.5], qp_star=[0.0], queue_cap=4096, dbuf_cap=4096, replications=3, steps=6000, seed=4)
    run_both(B, oracle_mod, cfg, 6000, checkpoints=2)


def test_paper_patience_rate_on_an_overloaded_network(B, oracle_mod):
    """theta = 0.1 (the rate of the paper's own convergence instance) on the two-class network at 1.4 times its
    arrival rates: queues of hundreds of requests, patience of up to 11783 steps, launches of 2048 steps."""
    cfg = W.config(2, N=256, replications=3)
    for c in cfg.classes:
        c.lam *= 1.4
        c.theta = 0.1
    sim, orc = run_both(B, oracle_mod, cfg, 9000, checkpoints=3)
    assert_stats_equal(sim.stats(), orc.stats())
    t = orc.stats()["tally"]
    assert t[:, TI["AB_P"]].sum() > 200


def test_every_workgroup_shape_with_abandonment(B, oracle_mod):
    """One wave (N = 60), two, eight and sixteen waves. Prefill-bound instances whose queues hold thousands of
    requests, a third or more of which abandon; decode-bound ones whose buffer fills, overflows and is
    compacted; and one with several gate passes per step (more than 256 admissions)."""
    for N, M, Bcap, steps, lam in ((60, 3, 8, 2500, (2.2, 1.8)), (700, 30, 8, 900, (2.2, 1.8)),
                                   (4000, 160, 8, 300, (2.4, 2.0)), (8192, 5000, 8, 60, (2.5, 2.0)),
                                   (8192, 300, 8, 200, (2.5, 2.0)), (8192, 300, 2, 300, (2.5, 2.0))):
        cls = [_limits_class(lam=lam[0], theta=3.0, out_p0=300.0),
               _limits_class(lam=lam[1], in_p0=40.0, out_p0=500.0, theta=9.0)]
        cfg = _limits_cfg(f"ab-shapes-{N}-{M}-{Bcap}", cls, N=N, M=M, B=Bcap, steps=steps, replications=1,
                          dbuf_cap=2048, queue_cap=8192)
        sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=2)
        t, g = orc.tallies(0)
        if M < 1000:
            assert t[:, TI["AB_P"]].sum() > 500, (N, M)
        if Bcap == 2:
            assert t[:, TI["AB_D"]].sum() > 5000 and g[5] == 1
        assert sim.stats()["overflow"] == bool(g[5])


def test_config5_width_with_abandonment_on_a_sampled_replication(B, oracle_mod):
    """Config 5 at its full width (16 waves, the LDS of a compute unit nearly full) with impatient classes and a
    quarter of its mixed servers, so that the prefill queues hold thousands of requests."""
    cfg = W.config(5, replications=2, mod_period=20000)
    cfg = replace(cfg, M=cfg.M // 4)
    for c in cfg.classes:
        c.theta = 0.5
    sim, orc = run_both(B, oracle_mod, cfg, 2000, oracle_reps=[1], checkpoints=2)
    t, _ = orc.tallies(1)
    assert t[:, TI["AB_P"]].min() > 5000
