"""Pins of the oracle's dynamics (CPU only): hand-traced example, flow-balance and capacity
invariants, Little's law, the exact discrete M/Geo/c chain with its Erlang-C limit, and
convergence of revenue to the fluid-LP optimum as the number of servers grows."""
import os
from dataclasses import replace

import numpy as np
import pytest
from scipy import stats

from paper_2602_02987_amd import plan as P
from paper_2602_02987_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TI = {n: i for i, n in enumerate(["A", "DROP_P", "U_P", "S_P", "U_DM", "U_DS", "S_DM", "S_DS", "M_SM", "M_MS",
                                  "DROP_D", "TOKP_PRE", "TOKP_DEC", "TOKD_DEC", "TOK_EMIT", "TOK_PREF", "SUM_QP",
                                  "SUM_QD", "SUM_X", "SUM_YM", "SUM_YS", "WAIT_STEPS", "TTFT_SUM", "E2E_SUM",
                                  "TBT_SUM", "AB_P", "AB_D"])}
GI = {n: i for i, n in enumerate(["ITERS_MIX", "ITERS_SOLO", "BUSY_MIX", "BUSY_SOLO", "STEPS", "OVERFLOW"])}


def one_class(lam, P_len, D_len, **kw):
    return W.SimClass(lam=lam, in_law=W.LAW_CONST, in_p0=P_len, out_law=W.LAW_CONST, out_p0=D_len, **kw)


def test_worked_example(oracle_mod):
    """tests/golden/worked_example.txt: one request, every server record at every step."""
    cfg = W.SimConfig(name="worked", K=1, N=2, B=2, C=256, c0=0.010, c_pre=0.00005, c_dec=0.0002,
                      classes=[one_class(2.5, 600, 3)], M=1, x_star=[0.1], qp_star=[0.0], queue_cap=16, dbuf_cap=16)
    # a seed whose only arrival in the first 11 steps falls in step 0
    seed = None
    for cand in range(1, 3000):
        o = oracle_mod.Oracle(cfg, max_reps=1)
        o.run(1, 1, cand)
        if o.tallies(0)[0][0, TI["A"]] != 1:
            continue
        o.run(10, 1, cand)
        if o.tallies(0)[0][0, TI["A"]] == 1:
            seed = cand
            break
    assert seed is not None
    rows, final = {}, None
    for line in open(os.path.join(GOLDEN, "worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        if f[0] == "T":
            final = [int(v) for v in f[1:]]
        else:
            rows.setdefault(int(f[0]), []).append([int(v) for v in f[1:]])
    o = oracle_mod.Oracle(cfg, max_reps=1)
    o.set_check(1)
    for s in range(11):
        o.run(1, 1, seed)
        sv = o.servers(0)
        sl = o.slots(0)
        for g, t_next, it, rem, nd in rows.get(s, []):
            got_t = -1 if sv["t_next"][g] == np.iinfo(np.int64).max else int(sv["t_next"][g])
            assert (got_t, int(sv["iter"][g]), int(sv["rem"][g]), int(sl["n_dec"][g])) == (t_next, it, rem, nd), (s, g)
    assert o.violations() == (0, 0)
    t, g = o.tallies(0)
    got = [t[0, TI["TTFT_SUM"]], t[0, TI["E2E_SUM"]], t[0, TI["TBT_SUM"]], t[0, TI["TOK_EMIT"]],
           t[0, TI["TOKP_DEC"]], t[0, TI["TOKD_DEC"]], g[GI["ITERS_MIX"]] + g[GI["ITERS_SOLO"]]]
    assert [int(v) for v in got] == final
    st = o.stats()
    assert st["rev_bundled_total"] == pytest.approx(603.0 / (2 * 0.11), rel=1e-12)   # (P + D) tokens at price 1
    assert st["ttft_mean"][0] == pytest.approx(0.060, rel=1e-12)
    assert st["tbt_mean"][0] == pytest.approx(0.0102, rel=1e-12)
    assert (t[0, TI["S_P"]], t[0, TI["S_DS"]], t[0, TI["S_DM"]], t[0, TI["U_DS"]]) == (1, 1, 0, 1)


def _heavy(gate=W.GATE_OCCUPANCY, **over):
    """Small overloaded instance that exercises every path: full slots, decode buffer, queue overflow."""
    cls = [W.SimClass(lam=1.6, in_law=W.LAW_GEOMETRIC, in_p0=300.0, out_law=W.LAW_GEOMETRIC, out_p0=40.0, priority=0.2),
           W.SimClass(lam=1.2, in_law=W.LAW_LOGNORMAL, in_p0=90.0, in_p1=0.8, out_law=W.LAW_LOGNORMAL, out_p0=150.0,
                      out_p1=1.0, priority=1.5, bundled=0, price_in=0.5, price_out=2.0),
           W.SimClass(lam=0.8, in_law=W.LAW_CONST, in_p0=513.0, out_law=W.LAW_GEOMETRIC, out_p0=20.0, priority=0.9)]
    cfg = W.SimConfig(name="heavy", K=3, N=12, B=4, C=128, c0=0.010, c_pre=0.00005, c_dec=0.0002, classes=cls, M=5,
                      x_star=[0.2, 0.15, 0.05], qp_star=[0.5, 0.0, 0.1], queue_cap=40, dbuf_cap=12, gate_mode=gate,
                      replications=3, steps=4000, seed=11)
    return replace(cfg, **over)


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_invariants_hold_every_step(oracle_mod, gate):
    """Balance equations, capacity constraints (Sec. 2.3), token conservation, FIFO order, every step."""
    for cfg in (_heavy(gate), _heavy(gate, M=0), _heavy(gate, M=12), _heavy(gate, B=1, M=6),
                _heavy(gate, name="heavy-prefill", M=1, queue_cap=8), W.config(1, replications=2, steps=3000)):
        o = oracle_mod.Oracle(cfg)
        o.set_check(1)
        o.run(cfg.steps)
        assert o.violations() == (0, 0), cfg.name
        t, g = o.tallies(0)
        if cfg.name == "heavy" and 0 < cfg.M < 12 and cfg.B > 1:
            assert g[GI["OVERFLOW"]] == 1 and t[:, TI["DROP_D"]].sum() > 0      # the overflow path was exercised
            assert t[:, TI["U_DM"]].sum() > 0 and t[:, TI["M_SM"]].sum() > 0 and t[:, TI["SUM_QD"]].sum() > 0
        if cfg.name == "heavy-prefill":
            assert g[GI["OVERFLOW"]] == 1 and t[:, TI["DROP_P"]].sum() > 0


# What oracle_poke can perturb (first argument after the replication) and the checker's codes: 130-134 recount of
# X, Y_m, Y_s, Q_d, Q_p from the servers and queues; 140-144 the balance equations of Sec. 2.3 (eq:bal-Qp, eq:bal-X,
# eq:bal-Qd, eq:bal-Ym, eq:bal-Ys); 150/151 token conservation; 103 decode count of a server; 106 a mixed-group
# server holds at most B-1 decodes; 121 the aggregate form of it, Y_m <= (B-1) X (eq:cap-Ym); 108/109 prefill state;
# 112 a running iteration ends after the current boundary; 101 finish index of a decode.
_POKE = dict(Qp=0, X=1, Qd=2, Ym=3, Ys=4, tally=5, n_dec=6, pf_rem=7, t_next=8, fin=9, extra_slot=10)


def test_checker_detects_a_planted_imbalance(oracle_mod):
    """The invariant checker fires, with the code of the violated relation, when one number of a consistent state
    is perturbed: each balance equation, each recounted aggregate, token conservation, the per-server capacity
    constraint and its aggregate form. Every "invariants hold" pin rests on this."""
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, replications=1)
    K, NT = cfg.K, len(TI)

    def fresh(steps):
        o = oracle_mod.Oracle(cfg)
        o.run(steps)
        assert o.check() == 0 and o.violations() == (0, 0)
        return o

    def planted(o, what, i, delta, expect, also=()):
        o.clear_violations()
        o.poke(0, _POKE[what], i, delta)
        n = o.check()
        codes = o.violation_codes()
        assert n > 0 and o.violations()[1] == expect and set(also) <= set(codes), (what, i, delta, n, codes)
        o.poke(0, _POKE[what], i, -delta)          # undo: the state is consistent again
        o.clear_violations()
        assert o.check() == 0, (what, i, "undo")

    o = fresh(700)
    for k in range(K):
        # counting processes: each perturbs exactly the balance equations it appears in (the first one is reported first)
        planted(o, "tally", k * NT + TI["A"], 1, 140)
        planted(o, "tally", k * NT + TI["U_P"], 1, 140, also=(141,))
        planted(o, "tally", k * NT + TI["S_P"], 1, 141, also=(142,))
        planted(o, "tally", k * NT + TI["U_DS"], 1, 142, also=(144,))
        planted(o, "tally", k * NT + TI["U_DM"], 1, 142, also=(143,))
        planted(o, "tally", k * NT + TI["S_DM"], 1, 143)
        planted(o, "tally", k * NT + TI["S_DS"], 1, 144)
        planted(o, "tally", k * NT + TI["M_SM"], 1, 143, also=(144,))
        planted(o, "tally", k * NT + TI["M_MS"], -1, 143, also=(144,))
        planted(o, "tally", k * NT + TI["TOK_EMIT"], 1, 150)
        planted(o, "tally", k * NT + TI["TOKD_DEC"], 1, 150)
        planted(o, "tally", k * NT + TI["TOK_PREF"], -1, 151)
        # state counters against the recount from the servers and queues, and against the balance equations
        planted(o, "X", k, 1, 130, also=(141,))
        planted(o, "Ym", k, -1, 131, also=(143,))
        planted(o, "Ys", k, 1, 132, also=(144,))
        planted(o, "Qd", k, 1, 133, also=(142,))
        planted(o, "Qp", k, -1, 134, also=(140,))
    sl, sv = o.slots(0), o.servers(0)
    g_busy = int(np.nonzero(sl["n_dec"] > 0)[0][0])
    planted(o, "n_dec", g_busy, 1, 103)
    planted(o, "fin", g_busy, 40000, 101)                       # a decode that would outlive its D tokens
    planted(o, "t_next", g_busy, -10**12, 112)                  # an iteration that should already have completed
    g_pf = int(np.nonzero(sv["rem"] > 0)[0][0])
    planted(o, "pf_rem", g_pf, 40000, 109, also=(151,))         # more prompt tokens left than the prompt has
    g_solo = cfg.M + int(np.nonzero(sl["n_dec"][cfg.M:] > 0)[0][0])
    planted(o, "pf_rem", g_solo, 1, 108, also=(130,))           # a prefill on a solo-group server
    # capacity (Sec. 2.3): a mixed-group server with B decodes beside its prefill; with every mixed server full,
    # the aggregate constraint Y_m <= (B-1) X fails too
    o = oracle_mod.Oracle(cfg)
    for _ in range(3000):
        o.run(1)
        sl, sv = o.slots(0), o.servers(0)
        if np.all(sv["rem"][:cfg.M] > 0) and np.all(sl["n_dec"][:cfg.M] == cfg.B - 1):
            break
    else:
        raise AssertionError("the mixed group never filled up")
    assert o.check() == 0
    o.poke(0, _POKE["extra_slot"], 0, 0)
    assert o.check() > 0
    assert {103, 106, 121} <= set(o.violation_codes()), o.violation_codes()


def test_little_law_exact_identity(oracle_mod):
    """sum_s Q_p,k(s) = sum over admitted jobs of (admission step - arrival step)
    + sum over still-waiting jobs of (S - arrival step): exact integers."""
    for cfg in (_heavy(queue_cap=100000), W.config(1, replications=2, steps=5000)):
        o = oracle_mod.Oracle(cfg)
        o.run(cfg.steps)
        S = cfg.steps
        for r in range(cfg.replications):
            t, _ = o.tallies(r)
            for k in range(cfg.K):
                waiting = o.queue(r, k).astype(np.int64)
                assert int(t[k, TI["SUM_QP"]]) == int(t[k, TI["WAIT_STEPS"]]) + int((S - waiting).sum())


def test_little_law_whole_system(oracle_mod):
    """L = lambda W for the whole network, time-averaged (long underloaded run)."""
    cfg = W.config(1, N=16, replications=4, steps=60000)
    o = oracle_mod.Oracle(cfg)
    o.run(cfg.steps)
    st = o.stats()
    t = st["tally"]
    for k in range(cfg.K):
        L = sum(int(t[k, TI[n]]) for n in ("SUM_QP", "SUM_X", "SUM_QD", "SUM_YM", "SUM_YS")) / (cfg.steps * cfg.replications)
        lam = int(t[k, TI["A"]]) / (cfg.steps * cfg.replications)           # per step
        Wt = st["e2e_mean"][k] / cfg.c0                                      # in steps
        assert L == pytest.approx(lam * Wt, rel=0.03)


def _mgc_chain_mean_queue(pa, c, q, nmax=600):
    """Exact stationary mean queue of n' = n + A - Bin(min(n,c), q), queue = max(n-c,0)."""
    T = np.zeros((nmax + 1, nmax + 1))
    for n in range(nmax + 1):
        b = min(n, c)
        pd = stats.binom.pmf(np.arange(b + 1), b, q)
        for d, pdv in enumerate(pd):
            for a, pav in enumerate(pa):
                T[n, min(n - d + a, nmax)] += pdv * pav
    w, v = np.linalg.eig(T.T)
    pi = np.real(v[:, np.argmin(np.abs(w - 1.0))]); pi = pi / pi.sum()
    n = np.arange(nmax + 1)
    return float(pi @ np.maximum(n - c, 0))


def test_prefill_stage_is_the_discrete_mgc_queue_and_tends_to_erlang_c(oracle_mod):
    """Single class, contention off (every iteration lasts one step): the prefill stage is a
    c-server queue with geometric service; its exact stationary mean queue pins the gate, the
    FIFO and the start/complete timing; Erlang-C is its continuous-time limit."""
    c, N, Cchunk, meanP = 4, 8, 64, 800.0
    q = 1.0 - (1.0 - 1.0 / meanP) ** Cchunk                     # ceil(P/C) is geometric(q)
    rho = 0.8
    lam_step_total = rho * c * q
    lam = lam_step_total / (N * 0.010)
    cls = [W.SimClass(lam=lam, in_law=W.LAW_GEOMETRIC, in_p0=meanP, out_law=W.LAW_CONST, out_p0=1.0)]
    cfg = W.SimConfig(name="mgc", K=1, N=N, B=8, C=Cchunk, c0=0.010, c_pre=0.0, c_dec=0.0, classes=cls, M=c,
                      x_star=[0.4], qp_star=[0.0], queue_cap=100000, dbuf_cap=64, replications=48, steps=60000, seed=5)
    o = oracle_mod.Oracle(cfg)
    o.run(cfg.steps)
    per_rep = np.array([o.tallies(r)[0][0, TI["SUM_QP"]] / cfg.steps for r in range(cfg.replications)], dtype=np.float64)
    # arrivals per step: sum over N servers of the truncated Poisson the sampler draws
    m = lam * 0.010
    p1 = stats.poisson.pmf([0, 1, 2], m); p1 = np.append(p1, 1.0 - p1.sum())
    pa = np.array([1.0])
    for _ in range(N):
        pa = np.convolve(pa, p1)
    exact = _mgc_chain_mean_queue(pa, c, q)
    se = per_rep.std(ddof=1) / np.sqrt(per_rep.size)
    assert se / exact < 0.05
    assert abs(per_rep.mean() - exact) < 4.0 * se
    a = rho * c
    erl = P.erlang_c(c, a) * rho / (1.0 - rho)                  # M/M/c mean queue length
    assert exact == pytest.approx(erl, rel=3.0 * q)             # discretisation term O(1/E[service steps])
    assert per_rep.mean() == pytest.approx(erl, rel=3.0 * q + 4.0 * se / exact)


def _lp_instance(N, reps, steps, Pl, Dl, overload=1.3):
    """Overloaded two-class instance shaped like the EC's synthetic convergence study: a decode-heavy
    and a prefill-heavy class, constant lengths that are multiples of the chunk, iteration times of the
    paper's calibration (tau_solo = 8.9 ms, tau_mix = 33.3 ms at C = 256), arrivals 30 % above capacity."""
    cls = [one_class(1.0, Pl[0], Dl[0], price_in=0.1, price_out=0.2), one_class(1.0, Pl[1], Dl[1], price_in=0.1, price_out=0.2)]
    cfg = W.SimConfig(name="lp", K=2, N=N, B=16, C=256, c0=0.0089, c_pre=(0.0333 - 0.0089) / 256, c_dec=0.0,
                      classes=cls, queue_cap=400000, dbuf_cap=1 << 20, replications=reps, steps=steps, seed=3)
    s = P.capacity_scale(cfg, [0.5, 0.5])
    for c in cfg.classes:
        c.lam = overload * s * 0.5
    return W.with_plan(cfg)


def _window_revenue(o, cfg, warm, steps):
    o.run(warm); s0 = o.stats()
    o.run(steps); s1 = o.stats()
    t = s1["tally"].astype(np.float64) - s0["tally"].astype(np.float64)
    nt = cfg.N * cfg.replications * steps * cfg.c0
    rev = sum(c.price_in * t[k, TI["TOKP_DEC"]] + c.price_out * t[k, TI["TOKD_DEC"]] for k, c in enumerate(cfg.classes)) / nt
    x = t[:cfg.K, TI["SUM_X"]] / (cfg.N * cfg.replications * steps)
    return rev, x


def test_revenue_converges_to_fluid_lp_optimum(oracle_mod):
    """Asymptotic optimality (Theorem 2): per-server bundled revenue of gate-and-route tends to the
    LP optimum R* as n grows, in the binding-capacity case (prefill and decode both saturated)."""
    errs = {}
    for N, reps in ((8, 16), (128, 2), (512, 1)):
        cfg = _lp_instance(N, reps, 90000, (1024, 3072), (400, 160))
        pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
        lam = np.array([c.lam for c in cfg.classes])
        assert np.all(pl.served <= lam + 1e-9) and np.any(pl.served < lam - 1e-3)   # capacity binds
        assert 0 < cfg.M < cfg.N and pl.ys.sum() > 1.0 and pl.ym.sum() > 1.0          # both decode pools in use
        o = oracle_mod.Oracle(cfg)
        rev, x = _window_revenue(o, cfg, 30000, 60000)
        errs[N] = (rev - pl.value) / pl.value
        if N == 512:
            assert np.allclose(x, pl.x, rtol=0.04)       # prefill occupancy tracks x* (EC, occupancy convergence)
    assert abs(errs[512]) < 0.02
    assert abs(errs[512]) < abs(errs[128]) + 0.005 < abs(errs[8]) + 0.01
    assert all(e < 0.01 for e in errs.values())         # the fluid optimum is an upper bound (up to noise)


def test_prefill_bound_revenue_equals_lp_optimum(oracle_mod):
    """Short outputs: only the prefill capacity binds, every server is mixed, and the revenue rate equals
    R* = sum_i w_i mu_p,i x_i* at any n once the gate holds the class mix at x*."""
    cfg = _lp_instance(32, 4, 50000, (1024, 3072), (40, 16))
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    assert cfg.M == cfg.N and pl.x.sum() == pytest.approx(1.0)
    o = oracle_mod.Oracle(cfg)
    rev, x = _window_revenue(o, cfg, 10000, 40000)
    assert rev == pytest.approx(pl.value, rel=2e-3)
    assert np.allclose(x, pl.x, rtol=1e-2)


def test_underloaded_throughput_and_revenue(oracle_mod):
    """Underloaded case: every request is served, so the revenue rate is sum_i lambda_i w_i and the
    prefill occupancy is lambda_i times the mean prefill service time (LP flow balance with theta = 0)."""
    cfg = W.config(2, N=64, replications=4, steps=60000)
    o = oracle_mod.Oracle(cfg)
    o.run(10000); s0 = o.stats()
    o.run(50000); s1 = o.stats()
    t = (s1["tally"].astype(np.float64) - s0["tally"].astype(np.float64))
    nt = cfg.N * cfg.replications * 50000 * cfg.c0
    r = P.rates(cfg)
    for k, c in enumerate(cfg.classes):
        assert t[k, TI["A"]] / nt == pytest.approx(c.lam, rel=0.03)
        assert (t[k, TI["S_DM"]] + t[k, TI["S_DS"]]) / nt == pytest.approx(c.lam, rel=0.03)
        assert t[k, TI["TOKD_DEC"]] / (t[k, TI["S_DM"]] + t[k, TI["S_DS"]]) == pytest.approx(r["ED"][k], rel=0.03)
        assert t[k, TI["TOKP_PRE"]] / t[k, TI["S_P"]] == pytest.approx(r["EP"][k], rel=0.03)
    sep = sum(c.price_in * t[k, TI["TOKP_PRE"]] + c.price_out * t[k, TI["TOKD_DEC"]] for k, c in enumerate(cfg.classes)) / nt
    want = sum(c.lam * (c.price_in * r["EP"][k] + c.price_out * r["ED"][k]) for k, c in enumerate(cfg.classes))
    assert sep == pytest.approx(want, rel=0.03)
    # mean prefill occupancy = lambda * (E ceil(P/C) * c0 + c_pre * E P + c_dec * mean co-resident decodes * ...) >= lower bound
    x_lo = np.array([c.lam * (r["ECH"][k] * cfg.c0 + cfg.c_pre * r["EP"][k]) for k, c in enumerate(cfg.classes)])
    x_sim = t[:2, TI["SUM_X"]] / (cfg.N * cfg.replications * 50000)
    assert np.all(x_sim > 0.97 * x_lo) and np.all(x_sim < 1.25 * x_lo)


def test_arrival_rates_and_counts(oracle_mod):
    cfg = W.config(1, N=32, replications=8, steps=20000)
    o = oracle_mod.Oracle(cfg)
    o.run(cfg.steps)
    tot = cfg.N * cfg.replications * cfg.steps
    A = o.stats()["tally"][:2, TI["A"]].astype(np.float64)
    for k, c in enumerate(cfg.classes):
        m = c.lam * cfg.c0
        assert abs(A[k] / tot - m) < 4.0 * np.sqrt(m / tot)


def test_resume_subset_and_digest(oracle_mod):
    cfg = _heavy()
    a = oracle_mod.Oracle(cfg); a.run(700)
    b = oracle_mod.Oracle(cfg); b.run(300); b.run(400)
    c = oracle_mod.Oracle(cfg); c.select([2]); c.run(700)
    for r in range(cfg.replications):
        assert a.digest(r) == b.digest(r)
        assert np.array_equal(a.tallies(r)[0], b.tallies(r)[0])
    assert a.digest(2) == c.digest(2) and a.digest(0) != a.digest(1)
    assert np.array_equal(a.tallies(2)[0], c.tallies(2)[0])
    for k in range(3):
        assert np.array_equal(a.hist(2, k), c.hist(2, k))
    d0 = a.digest(0); a.run(1); assert a.digest(0) != d0


def test_percentiles_from_histogram(oracle_mod):
    cfg = W.config(1, replications=4, steps=10000)
    o = oracle_mod.Oracle(cfg)
    o.run(cfg.steps)
    st = o.stats()
    h = sum(o.hist(r, 2) for r in range(cfg.replications))
    for k in range(cfg.K):
        n = int(h[k].sum()); assert n == int(st["tally"][k, TI["TOK_EMIT"]])
        cum = np.cumsum(h[k])
        b95 = int(np.searchsorted(cum, -(-95 * n // 100)))
        assert st["tbt_p95"][k] == pytest.approx(oracle_mod.hedge(b95) * 1e-9, rel=1e-12)
        assert oracle_mod.hedge(oracle_mod.hbin(10_000_000)) * 1e-9 <= st["tbt_p50"][k] <= st["tbt_p95"][k] <= st["tbt_p99"][k] <= 0.0492


def test_rate_estimate_and_replanning():
    """Rolling-window estimate (Eq. main-online-arrival-estimate) by hand, and the re-solved LP keeps the
    prefill occupancy inside the split it was given."""
    from paper_2602_02987_amd import plan
    lam = plan.estimate_rates([130, 40], [10, 40], n_servers=20, t_now=12.0, window=30.0, rho=3.0, lam_min=1e-6)
    assert lam[0] == 3.0 * 120 / (20 * 12.0) and lam[1] == 1e-6      # window cut at t, floor for a silent class
    lam = plan.estimate_rates([130, 40], [100, 10], n_servers=20, t_now=100.0, window=30.0)
    assert np.allclose(lam, [3.0 * 30 / 600.0, 3.0 * 30 / 600.0])
    cfg = W.config(3, N=64, replications=1)
    base = np.array([c.lam for c in cfg.classes])
    p = plan.replan(cfg, 3.0 * base)
    assert p.x.sum() <= cfg.M / cfg.N + 1e-9 and p.x.sum() > 0.5 * cfg.M / cfg.N
    q = plan.replan(cfg, 0.1 * base)
    assert q.x.sum() < p.x.sum() and np.all(q.x > 0)                 # light load: every class served, little prefill occupancy
    assert np.allclose(q.served, 0.1 * base, rtol=1e-6)


def test_targets_can_move_between_runs(oracle_mod):
    """New targets change the gate's order from then on and nothing else: the state carries over, the
    invariants hold, and a run whose targets are set to the values it already has is unchanged."""
    cfg = _heavy()
    a = oracle_mod.Oracle(cfg); a.set_check(1); a.run(600); a.set_targets(cfg.x_star, cfg.qp_star); a.run(600)
    b = oracle_mod.Oracle(cfg); b.run(1200)
    assert a.violations() == (0, 0)
    assert all(a.digest(r) == b.digest(r) for r in range(cfg.replications))
    # where the prefill slots are the bottleneck the admission mix follows the targets
    cfg = _heavy(name="heavy-prefill", M=1, queue_cap=8)
    a = oracle_mod.Oracle(cfg); a.run(2000)
    c = oracle_mod.Oracle(cfg); c.set_check(1); c.run(600); c.set_targets([0.02, 0.4, 0.3], [0.0, 2.0, 0.0]); c.run(1400)
    assert c.violations() == (0, 0)
    ta, tc = a.tallies(0)[0], c.tallies(0)[0]
    assert np.array_equal(ta[:, TI["A"]] + ta[:, TI["DROP_P"]], tc[:, TI["A"]] + tc[:, TI["DROP_P"]])   # same arrivals
    assert not np.array_equal(ta[:, TI["U_P"]], tc[:, TI["U_P"]])                                       # another admission mix
    assert tc[1, TI["U_P"]] > 10 * ta[1, TI["U_P"]]                                                     # the class whose target was raised
