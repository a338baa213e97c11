"""GPU parity with a moving mixed/solo split (sim_set_split between runs; paper, online adaptive algorithm)."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_replication_equal, assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy

pytestmark = pytest.mark.gpu


def _run_moves(B, oracle_mod, cfg, moves, reps=None, oracle_reps=None):
    reps = cfg.replications if reps is None else reps
    sim = B.Sim(cfg, max_replications=reps)
    orc = oracle_mod.Oracle(cfg, max_reps=reps)
    if oracle_reps is not None:
        orc.select(oracle_reps)
    for m, steps in moves:
        if m is not None:
            sim.set_split(m); orc.set_split(m)
        sim.run(steps, reps); orc.run(steps, reps)
        for r in (range(reps) if oracle_reps is None else oracle_reps):
            assert_replication_equal(sim, orc, r, what=f"{cfg.name} after M={m}, {steps} steps")
    return sim, orc


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_FCFS])
def test_moves_on_the_overloaded_small_instance(B, oracle_mod, gate):
    cfg = _heavy(gate, queue_cap=4096, dbuf_cap=4096)
    sim, orc = _run_moves(B, oracle_mod, cfg, [(None, 500), (11, 400), (3, 400), (0, 400), (12, 400), (6, 400), (6, 200), (1, 400)])
    assert_stats_equal(sim.stats(), orc.stats())
    cfg = _heavy(gate)   # with the small rings: drops on the way
    _run_moves(B, oracle_mod, cfg, [(None, 300), (9, 500), (2, 500), (12, 300)])


def test_moves_across_bitmap_words_and_workgroup_shapes(B, oracle_mod):
    """The split crosses several 64-server words in both directions while prefills are in service and decode
    rows are full; two-wave and sixteen-wave workgroups."""
    for N, moves in ((1500, [(None, 300), (700, 300), (64, 300), (0, 200), (1500, 200), (130, 300)]),
                     (6000, [(None, 120), (900, 120), (200, 120), (2000, 120)])):
        cls = [_limits_class(lam=2.2, in_p0=900.0, out_p0=60.0), _limits_class(lam=1.8, in_p0=300.0, out_p0=200.0)]
        cfg = _limits_cfg(f"moves-{N}", cls, N=N, M=N // 10, B=8, steps=100, replications=1, dbuf_cap=8192, queue_cap=16384)
        sim, orc = _run_moves(B, oracle_mod, cfg, moves)
        t, _ = orc.tallies(0)
        assert t[:, TI["U_DM"]].sum() > 0 and t[:, TI["M_MS"]].sum() > 0


def test_moves_with_abandonment_and_with_the_randomized_router(B, oracle_mod):
    cfg = _heavy(queue_cap=4096, dbuf_cap=4096)
    cfg.classes = [replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))]
    _run_moves(B, oracle_mod, cfg, [(None, 400), (10, 400), (2, 400), (7, 400)])
    cfg = replace(_heavy(queue_cap=4096, dbuf_cap=4096), route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.8, 0.3, 0.55])
    _run_moves(B, oracle_mod, cfg, [(None, 400), (10, 400), (2, 400), (7, 400)])
    cfg = replace(_heavy(), route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.8, 0.3, 0.55])   # both at once, small rings
    cfg.classes = [replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))]
    _run_moves(B, oracle_mod, cfg, [(None, 400), (10, 400), (2, 400), (7, 400)])


def test_config5_width_with_a_moving_split(B, oracle_mod):
    cfg = W.config(5, replications=2, mod_period=20000)
    m0 = cfg.M
    _run_moves(B, oracle_mod, cfg, [(None, 600), (m0 + 300, 500), (m0 - 500, 500), (m0, 400)], oracle_reps=[0])


def test_a_split_that_does_not_fit_on_chip_is_refused(B):
    cfg = W.config(5, replications=1)
    for c in cfg.classes:
        c.theta = 0.5               # (the abandonment variant keeps a candidate table on chip as well)
    sim = B.Sim(cfg)
    with pytest.raises(B.SimError):
        sim.set_split(cfg.N)        # prompt-token counters for 10000 servers exceed what is left of the LDS
    with pytest.raises(B.SimError):
        sim.set_split(-1)
    sim.set_split(cfg.M + 100)
    sim.run(10)


def test_online_adaptive_loop_in_step_with_the_oracle(B, oracle_mod):
    """The online controller (rolling-window rate estimate, LP re-solve, new targets and split every epoch)
    around the library and around the oracle: the same tallies feed it, so both closed loops stay bit-equal."""
    from paper_2602_02987_amd import online
    cfg = W.config(5, N=512, replications=3, mod_period=6000)
    sim = B.Sim(cfg); orc = oracle_mod.Oracle(cfg)
    la = online.run_online(sim, cfg, 9000, replan_every=1000, window=3000)
    lb = online.run_online(orc, cfg, 9000, replan_every=1000, window=3000)
    assert [pl.M for _, _, pl in la] == [pl.M for _, _, pl in lb] and len({pl.M for _, _, pl in la}) > 1
    for r in range(cfg.replications):
        assert_replication_equal(sim, orc, r, what="online loop")
    assert_stats_equal(sim.stats(), orc.stats())


def test_a_burst_of_completed_prefills_larger_than_one_round(B, oracle_mod):
    """The two-buffer routers take the completed prefills of a step 64 to a wave, in rounds of up to four waves.
    Queues fill while no server admits (M = 0); then many servers turn mixed at once, admit in the same step (several
    gate passes) and end their one-chunk prefills in the same step: 1200 completions in a step for eight-wave
    workgroups (five rounds), 500 for two-wave workgroups (four rounds), also with a decode buffer too small for them,
    with abandonment and with the weighted router."""
    cls = [_limits_class(lam=2.4, out_p0=300.0), _limits_class(lam=2.0, in_p0=40.0, out_p0=500.0)]
    base = _limits_cfg("burst", cls, N=1500, M=0, B=8, steps=100, replications=1, dbuf_cap=4096, queue_cap=8192)
    rr = replace(base, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.6, 0.3])
    ab = replace(rr, classes=[replace(c, theta=th) for c, th in zip(rr.classes, (2.0, 0.5))])
    ws = replace(ab, route_mode=W.ROUTE_WEIGHTED_SPLIT, w_solo=[0.7, 0.3], w_mixed=[0.2, 0.8])
    moves = [(None, 40), (1200, 6), (100, 20), (1400, 8)]
    for cfg in (rr, replace(rr, name="burst-small-buffer", dbuf_cap=512), ab, ws):
        sim, orc = _run_moves(B, oracle_mod, cfg, moves)
        t, _ = orc.tallies(0)
        assert t[:, TI["S_P"]].sum() > 1500, cfg.name   # the bursts went through
    many = replace(rr, name="burst-two-waves", N=600, replications=1500)
    _run_moves(B, oracle_mod, many, [(None, 40), (500, 6), (50, 10)], oracle_reps=[0, 749, 1499])
