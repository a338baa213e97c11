"""Pins of the oracle's moving mixed/solo split (paper, online adaptive algorithm: the split tracks M*(t_k),
existing service is not pre-empted, the new split governs later admissions and placements). CPU only."""
from dataclasses import replace

import numpy as np

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import TI, _heavy


def test_the_same_split_again_changes_nothing(oracle_mod):
    cfg = _heavy()
    a = oracle_mod.Oracle(cfg); a.run(1500)
    b = oracle_mod.Oracle(cfg); b.set_check(1); b.run(700); b.set_split(cfg.M); b.run(800)
    assert b.violations() == (0, 0)
    for r in range(cfg.replications):
        assert a.digest(r) == b.digest(r) and np.array_equal(a.tallies(r)[0], b.tallies(r)[0])


def test_a_split_set_before_the_first_step_is_the_configured_one(oracle_mod):
    for m1, m2 in ((5, 9), (9, 2), (0, 12), (12, 0)):
        a = oracle_mod.Oracle(_heavy(M=m2)); a.run(1200)
        b = oracle_mod.Oracle(_heavy(M=m1)); b.set_split(m2); b.run(1200)
        for r in range(3):
            assert a.digest(r) == b.digest(r) and np.array_equal(a.tallies(r)[0], b.tallies(r)[0])


def test_no_preemption_when_the_mixed_group_shrinks(oracle_mod):
    """M -> 0: the call itself changes no state; no admission follows; the prefills in service run to their end
    and their servers then serve decodes up to B."""
    cfg = _heavy(M=8, queue_cap=4096, dbuf_cap=4096)
    o = oracle_mod.Oracle(cfg); o.set_check(1)
    o.run(900)
    before = [o.digest(r) for r in range(cfg.replications)]
    x0 = [int(o.class_state(r)["X"].sum()) for r in range(cfg.replications)]
    up0 = [int(o.tallies(r)[0][:, TI["U_P"]].sum()) for r in range(cfg.replications)]
    sp0 = [int(o.tallies(r)[0][:, TI["S_P"]].sum()) for r in range(cfg.replications)]
    o.set_split(0)
    assert [o.digest(r) for r in range(cfg.replications)] == before and max(x0) > 0
    o.run(40)
    assert max(o.slots(r)["n_dec"][:8].max() for r in range(cfg.replications)) == cfg.B   # as solo servers they fill to B
    o.run(1460)
    assert o.violations() == (0, 0)
    for r in range(cfg.replications):
        t, _ = o.tallies(r)
        assert int(t[:, TI["U_P"]].sum()) == up0[r]                        # nobody admitted after the move
        assert int(t[:, TI["S_P"]].sum()) == sp0[r] + x0[r]                  # every prefill in service finished
        assert o.class_state(r)["X"].sum() == 0


def test_servers_that_turn_mixed_keep_their_decodes_and_take_no_more_until_below_the_cap(oracle_mod):
    """M: 2 -> 10 on the overloaded instance: servers 2..9 hold B decodes at the move; from then on they get
    prefills, and none of them receives a decode while it holds B-1 or more."""
    cfg = _heavy(M=2, queue_cap=4096, dbuf_cap=4096)
    o = oracle_mod.Oracle(cfg); o.set_check(1)
    o.run(1500)
    assert o.slots(0)["n_dec"][2:10].min() == cfg.B
    o.set_split(10)
    prev = o.slots(0)["n_dec"].copy()
    took_prefill = np.zeros(cfg.N, bool)
    for _ in range(600):
        o.run(1)
        cur = o.slots(0)["n_dec"]
        grew = cur > prev
        assert not np.any(grew[2:10] & (prev[2:10] >= cfg.B - 1))
        took_prefill |= o.servers(0)["rem"] > 0
        prev = cur.copy()
    assert o.violations() == (0, 0)
    assert took_prefill[2:10].all() and not took_prefill[10:].any()


def test_balance_equations_hold_across_repeated_moves(oracle_mod):
    cfg = _heavy(queue_cap=4096, dbuf_cap=4096)
    o = oracle_mod.Oracle(cfg); o.set_check(1)
    for m in (5, 11, 3, 0, 12, 6, 6, 1):
        o.set_split(m)
        o.run(400)
    assert o.violations() == (0, 0)


def test_online_adaptive_loop_follows_the_load(oracle_mod):
    """The controller of the paper's online adaptive algorithm around the oracle, on sinusoidal arrivals: the
    estimated rates follow the modulation (times the safety factor), the split M*(t_k) moves with them, and
    the balance equations hold across every move."""
    from paper_2602_02987_amd import online
    cfg = W.config(5, N=256, replications=2, mod_period=8000)
    o = oracle_mod.Oracle(cfg); o.set_check(25)
    log = online.run_online(o, cfg, 16000, replan_every=1000, window=2000, rho=1.0)
    assert o.violations() == (0, 0)
    lam_total = np.array([lam.sum() for _, lam, _ in log]); ms = np.array([pl.M for _, _, pl in log])
    base = sum(c.lam for c in cfg.classes)
    # window (s-2000, s]: mean of the modulation over it
    steps = np.array([s for s, _, _ in log])
    want = np.array([np.mean(1.0 + cfg.mod_amp * np.sin(2 * np.pi * (np.arange(max(s - 2000, 0), s) % 8000) / 8000)) for s in steps])
    assert np.allclose(lam_total / base, want, rtol=0.06)
    assert ms.max() > ms.min() + 5 and np.corrcoef(ms, lam_total)[0, 1] > 0.8
