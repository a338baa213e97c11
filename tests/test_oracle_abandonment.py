"""Pins of the oracle's abandonment (paper Sec. 2.3: every waiting job has an exponential patience with its
class's rate theta, in the prefill queue and in the decode buffer). CPU only.

What fixes the behaviour: the patience table against the closed-form geometric law; a queue that nobody is
ever admitted from, rebuilt job by job from the random blocks the patience is drawn from (prefill queue and
decode buffer); the exact stationary law of the discrete many-server queue with abandonment (the discrete
Erlang-A chain); the balance equations with the abandonment terms, every step."""
from dataclasses import replace

import numpy as np
import pytest
from scipy import stats

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import GI, TI, _heavy, one_class


@pytest.mark.parametrize("theta,dt", [(0.1, 0.010), (5.0, 0.010), (40.0, 0.010), (2.0, 0.004)])
def test_patience_table_is_geometric_in_steps(oracle_mod, theta, dt):
    """An exponential patience asked at step boundaries: Pr(patience >= m steps) = exp(-theta*dt*(m-1))."""
    t = oracle_mod.patience_table(theta, dt).astype(np.int64)
    assert t.min() == 1 and np.all(np.diff(t) >= 0)
    ks = np.unique(np.concatenate([np.arange(1, 50), np.linspace(1, t.max(), 200).astype(int)]))
    emp = np.searchsorted(t, ks, side="right") / 65536.0
    cdf = 1.0 - np.exp(-theta * dt * ks)
    assert np.max(np.abs(emp - cdf)) <= 1.0 / 65536 + 1e-12
    assert t.mean() == pytest.approx(1.0 / (1.0 - np.exp(-theta * dt)), rel=3e-4)


def _expected_occupancy(joined, pats):
    """joined[s] jobs join at step s with patience pats[s][j]; a job is present at the end of steps
    s .. s+pat-1 and leaves at the start of step s+pat. Returns (present at the end of each step, cumulative leavers)."""
    S = len(joined)
    diff = np.zeros(S + 70000, dtype=np.int64)
    leave = np.zeros(S + 70000, dtype=np.int64)
    for s in range(S):
        for j in range(joined[s]):
            diff[s] += 1
            diff[s + pats[s][j]] -= 1
            leave[s + pats[s][j]] += 1
    return np.cumsum(diff)[:S], np.cumsum(leave)[:S]


def test_prefill_queue_nobody_is_admitted_from(oracle_mod):
    """No mixed server: every arrival waits out its patience. The queue length and the abandonment count at
    every step are rebuilt from the blocks (step, stream 2+k, j, replication) of the accepted arrivals."""
    theta = [5.0, 12.0]
    cls = [replace(one_class(1.1, 100, 10), theta=theta[0]), replace(one_class(0.7, 100, 10), theta=theta[1])]
    cfg = W.SimConfig(name="ab-nogate", K=2, N=24, B=4, C=64, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=0,
                      x_star=[0.1, 0.1], qp_star=[0.0, 0.0], queue_cap=4096, dbuf_cap=16, replications=2, steps=1500,
                      seed=21)
    tabs = [oracle_mod.patience_table(th, cfg.c0).astype(np.int64) for th in theta]
    o = oracle_mod.Oracle(cfg)
    o.set_check(1)
    S = cfg.steps
    qp = np.zeros((cfg.replications, cfg.K, S), dtype=np.int64)
    ab = np.zeros_like(qp); arr = np.zeros_like(qp)
    for s in range(S):
        o.run(1)
        for r in range(cfg.replications):
            t, _ = o.tallies(r)
            qp[r, :, s] = o.class_state(r)["Qp"]
            ab[r, :, s] = t[:, TI["AB_P"]]; arr[r, :, s] = t[:, TI["A"]]
    assert o.violations() == (0, 0)
    for r in range(cfg.replications):
        t, _ = o.tallies(r)
        assert t[:, TI["U_P"]].sum() == 0 and t[:, TI["AB_P"]].sum() > 500
        for k in range(cfg.K):
            joined = np.diff(arr[r, k], prepend=0)
            pats = [[int(tabs[k][int(oracle_mod.philox(cfg.seed, s, 2 + k, j, r)[0]) >> 16]) for j in range(joined[s])]
                    for s in range(S)]
            present, left = _expected_occupancy(joined, pats)
            assert np.array_equal(qp[r, k], present), (r, k)
            assert np.array_equal(ab[r, k], left), (r, k)
            assert int(t[k, TI["SUM_QP"]]) == int(present.sum())
            # what is still waiting: stamps and the steps their patience ends in, oldest first
            want = [(s, s + pats[s][j]) for s in range(S) for j in range(joined[s]) if s + pats[s][j] > S - 1]
            got = list(zip(o.queue(r, k).astype(np.int64).tolist(), o.queue_deadlines(r, k).astype(np.int64).tolist()))
            assert got == want


def test_decode_buffer_nobody_is_routed_from(oracle_mod):
    """One server that is mixed and has B = 1: no decode slot exists, every completed prefill waits in the decode
    buffer until its patience, drawn from block (step, stream 10, server, replication), ends."""
    theta = 8.0
    cls = [replace(one_class(2.0, 60, 5), theta=theta)]
    cfg = W.SimConfig(name="ab-noroute", K=1, N=1, B=1, C=64, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=1,
                      x_star=[0.5], qp_star=[0.0], queue_cap=4096, dbuf_cap=4096, replications=3, steps=6000, seed=4)
    tab = oracle_mod.patience_table(theta, cfg.c0).astype(np.int64)
    o = oracle_mod.Oracle(cfg)
    o.set_check(1)
    S = cfg.steps
    qd = np.zeros((cfg.replications, S), dtype=np.int64); ab = np.zeros_like(qd); sp = np.zeros_like(qd)
    for s in range(S):
        o.run(1)
        for r in range(cfg.replications):
            t, _ = o.tallies(r)
            qd[r, s] = o.class_state(r)["Qd"][0]
            ab[r, s] = t[0, TI["AB_D"]]; sp[r, s] = t[0, TI["S_P"]]
    assert o.violations() == (0, 0)
    for r in range(cfg.replications):
        t, _ = o.tallies(r)
        assert t[0, TI["U_DM"]] + t[0, TI["U_DS"]] == 0 and t[0, TI["S_P"]] > 50
        joined = np.diff(sp[r], prepend=0)
        assert joined.max() == 1
        pats = [[int(tab[int(oracle_mod.philox(cfg.seed, s, 10, 0, r)[0]) >> 16])] * joined[s] for s in range(S)]
        present, left = _expected_occupancy(joined, pats)
        assert np.array_equal(qd[r], present) and np.array_equal(ab[r], left)
        assert int(t[0, TI["SUM_QD"]]) == int(present.sum())
        # with the buffer never drained, prefill-queue abandonment still runs: balance with both terms
        assert int(t[0, TI["A"]]) == int(t[0, TI["U_P"]] + t[0, TI["AB_P"]] + o.class_state(r)["Qp"][0])


def _erlang_a_chain(pa, c, q, pab, nmax=400):
    """Exact stationary law of n' = n + A - Bin(min(n,c), q) - Bin(max(n-c,0), pab): per step the waiting jobs
    of the previous step each leave with probability pab, the jobs in service each finish with probability q,
    and the freed servers are refilled from the queue. Returns (mean queue, abandonments per step)."""
    T = np.zeros((nmax + 1, nmax + 1))
    for n in range(nmax + 1):
        b, w = min(n, c), max(n - c, 0)
        pd = stats.binom.pmf(np.arange(b + 1), b, q)
        pl = stats.binom.pmf(np.arange(w + 1), w, pab)
        out = np.convolve(pd, pl)
        for d, pdv in enumerate(out):
            if pdv < 1e-18:
                continue
            for a, pav in enumerate(pa):
                T[n, min(n - d + a, nmax)] += pdv * pav
    w_, v = np.linalg.eig(T.T)
    pi = np.real(v[:, np.argmin(np.abs(w_ - 1.0))]); pi = pi / pi.sum()
    n = np.arange(nmax + 1)
    queue = np.maximum(n - c, 0)
    return float(pi @ queue), float(pi @ queue) * pab


def test_prefill_stage_is_the_discrete_erlang_a_queue(oracle_mod):
    """Single class, contention off, overloaded (rho = 1.15): the prefill stage is a c-server queue with geometric
    service and geometric patience; its exact stationary mean queue and abandonment rate pin the patience law,
    the instant a job is asked, and the order abandonment - completion - gate within a step."""
    c, N, Cchunk, meanP, theta = 4, 8, 64, 800.0, 3.0
    q = 1.0 - (1.0 - 1.0 / meanP) ** Cchunk
    pab = 1.0 - np.exp(-theta * 0.010)
    rho = 1.15
    lam = rho * c * q / (N * 0.010)
    cls = [W.SimClass(lam=lam, in_law=W.LAW_GEOMETRIC, in_p0=meanP, out_law=W.LAW_CONST, out_p0=1.0, theta=theta)]
    cfg = W.SimConfig(name="erlang-a", K=1, N=N, B=8, C=Cchunk, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=c,
                      x_star=[0.4], qp_star=[0.0], queue_cap=100000, dbuf_cap=64, replications=48, steps=40000, seed=9)
    o = oracle_mod.Oracle(cfg)
    o.run(cfg.steps)
    tl = [o.tallies(r)[0] for r in range(cfg.replications)]
    mq = np.array([t[0, TI["SUM_QP"]] / cfg.steps for t in tl], dtype=np.float64)
    abr = np.array([t[0, TI["AB_P"]] / cfg.steps for t in tl], dtype=np.float64)
    m = lam * 0.010
    p1 = stats.poisson.pmf([0, 1, 2], m); p1 = np.append(p1, 1.0 - p1.sum())
    pa = np.array([1.0])
    for _ in range(N):
        pa = np.convolve(pa, p1)
    exact_q, exact_ab = _erlang_a_chain(pa, c, q, pab)
    for got, want in ((mq, exact_q), (abr, exact_ab)):
        se = got.std(ddof=1) / np.sqrt(got.size)
        assert se / want < 0.03
        assert abs(got.mean() - want) < 4.0 * se
    # overloaded: what is not served abandons, arrivals = served + abandoned in the long run
    st = o.stats()
    assert st["abandon_rate_p"][0] == pytest.approx(st["arrival_rate"][0] - st["tally"][0, TI["U_P"]] /
                                                    (N * st["sim_time"] * cfg.replications), rel=2e-3)
    # a mean-queue estimate that ignored abandonment, or asked new arrivals in their own step, is far off
    wrong_q, _ = _erlang_a_chain(pa, c, q, pab * 1.25)
    assert abs(mq.mean() - wrong_q) > 8.0 * mq.std(ddof=1) / np.sqrt(mq.size)


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_invariants_hold_every_step_with_abandonment(oracle_mod, gate):
    """Balance equations with B_p and B_d (Sec. 2.3), FIFO order, nobody waiting past their patience: every step,
    on the overloaded instance, with one patient class among impatient ones."""
    for over in (dict(), dict(M=1), dict(B=1, M=6), dict(queue_cap=8, name="heavy-prefill")):
        cfg = _heavy(gate, **over)
        cfg.classes = [replace(c, theta=th) for c, th in zip(cfg.classes, (4.0, 0.0, 25.0))]
        o = oracle_mod.Oracle(cfg)
        o.set_check(1)
        o.run(cfg.steps)
        assert o.violations() == (0, 0), over
        t, g = o.tallies(0)
        assert t[1, TI["AB_P"]] == 0 and t[1, TI["AB_D"]] == 0
        assert t[0, TI["AB_P"]] + t[2, TI["AB_P"]] > 0
        if not over:
            assert t[0, TI["AB_D"]] + t[2, TI["AB_D"]] > 0 and t[:, TI["U_DM"]].sum() > 0
        # abandonment shortens the queues
        o0 = oracle_mod.Oracle(_heavy(gate, **over)); o0.run(cfg.steps)
        t0 = o0.tallies(0)[0]
        assert t[:, TI["SUM_QP"]].sum() + t[:, TI["SUM_QD"]].sum() < t0[:, TI["SUM_QP"]].sum() + t0[:, TI["SUM_QD"]].sum()


def test_theta_zero_changes_nothing(oracle_mod):
    """With every theta = 0 the state digest and the tallies are those of the model without abandonment."""
    cfg = _heavy()
    a = oracle_mod.Oracle(cfg); a.run(800)
    t, _ = a.tallies(0)
    assert t[:, TI["AB_P"]].sum() == 0 and t[:, TI["AB_D"]].sum() == 0
    assert np.all(a.queue_deadlines(0, 0) == 0xFFFFFFFF)


def test_overloaded_network_with_abandonment_sits_at_the_fluid_point(oracle_mod):
    """With theta > 0 the fluid LP keeps its optimum (the unserved flow lambda_i - mu_p,i x_i* abandons instead of
    queueing for ever): on the binding-capacity instance the revenue rate approaches R*, and the prefill backlog
    settles where abandonment balances the unserved flow, q_p,i = (lambda_i - mu_p,i x_i*) / theta (per step:
    Q_p,i * (1 - e^(-theta*dt)) = unserved arrivals per step)."""
    from paper_2602_02987_amd import plan as P
    from test_oracle_dynamics import _lp_instance, _window_revenue
    theta = 0.1   # the rate of the paper's own convergence instance
    cfg = _lp_instance(512, 1, 60000, (1024, 3072), (400, 160))
    for c in cfg.classes:
        c.theta = theta
    cfg = W.with_plan(cfg)                                     # the plan now carries backlog targets q_p*
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    assert np.allclose(cfg.qp_star, (np.array([c.lam for c in cfg.classes]) - pl.served) / theta, rtol=1e-9, atol=1e-12)
    o = oracle_mod.Oracle(cfg)
    o.run(20000); s0 = o.stats()
    o.run(40000); s1 = o.stats()
    t = s1["tally"].astype(np.float64) - s0["tally"].astype(np.float64)
    nt = cfg.N * 40000 * cfg.c0
    rev = sum(c.price_in * t[k, TI["TOKP_DEC"]] + c.price_out * t[k, TI["TOKD_DEC"]] for k, c in enumerate(cfg.classes)) / nt
    assert rev == pytest.approx(pl.value, rel=0.03) and rev < pl.value   # (some decode-buffer waiters leave too)
    lam = np.array([c.lam for c in cfg.classes])
    unserved = lam - pl.served                                  # per server and second
    assert np.any(unserved > 0.05)
    qp = t[:cfg.K, TI["SUM_QP"]] / (cfg.N * 40000)              # per server
    want = unserved * cfg.c0 / (1.0 - np.exp(-theta * cfg.c0))
    assert np.allclose(qp, want, rtol=0.08, atol=0.15)
    ab = t[:cfg.K, TI["AB_P"]] / nt
    assert np.allclose(ab, unserved, rtol=0.08, atol=0.02)
