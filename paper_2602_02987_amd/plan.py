"""Host-side static planning: the steady-state fluid LP and the server partition.

The LP (paper Sec. 3.2, the steady-state fluid control problem) is solved once per
configuration with scipy/HiGHS; its solution (x*, y_m*, y_s*) and the mixed-server
count M = ceil(n * sum_i x_i*) (paper Sec. 4, "Static Planning") are *inputs* of the
simulation library. Nothing here runs on the device and nothing here is on the
simulation's hot path.

Service rates follow the paper's definition (Sec. 2.3, service-rate display):
mu_p = 1/(prefill service time), mu_m = 1/(D tau_mix), mu_s = 1/(D tau_solo), with the
token-level refinements needed because lengths are random and the last chunk of a
prompt is short: the prefill service time of class i is
E[ceil(P_i/C)] * (c0 + c_dec * n_m) + c_pre * E[P_i].
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
from scipy.optimize import linprog
from scipy.special import erfc

LAW_GEOMETRIC, LAW_LOGNORMAL, LAW_CONST, LAW_TABLE = 0, 1, 2, 3
LMAX = 32768


def length_pmf(law: int, p0: float, p1: float = 0.0, table=None) -> np.ndarray:
    """pmf over lengths 1..LMAX (index k-1) of the integer-valued, clamped length law."""
    k = np.arange(1, LMAX + 1, dtype=np.float64)
    if law == LAW_CONST:
        pmf = np.zeros(LMAX)
        pmf[int(min(max(round(p0), 1), LMAX)) - 1] = 1.0
        return pmf
    if law == LAW_TABLE:
        t = np.asarray(table, dtype=np.int64)
        return np.bincount(t - 1, minlength=LMAX).astype(np.float64) / t.size
    if law == LAW_GEOMETRIC:
        p = 1.0 / p0
        cdf = np.ones(LMAX) if p >= 1.0 else -np.expm1(k * math.log1p(-p))
    elif law == LAW_LOGNORMAL:
        z = (np.log(k + 0.5) - math.log(p0)) / p1
        cdf = 0.5 * erfc(-z / math.sqrt(2.0))
    else:
        raise ValueError("unknown law")
    cdf[-1] = 1.0  # clamp: the tail mass sits on LMAX
    return np.diff(np.concatenate([[0.0], cdf]))


def length_moments(law: int, p0: float, p1: float, C: int, table=None):
    """(E[L], E[ceil(L/C)]) under the clamped integer law."""
    pmf = length_pmf(law, p0, p1, table)
    k = np.arange(1, LMAX + 1, dtype=np.float64)
    return float(pmf @ k), float(pmf @ np.ceil(k / C))


@dataclass
class Plan:
    x: np.ndarray          # prefill occupancy targets x_i* (per server)
    ym: np.ndarray         # mixed decode occupancy y_m,i*
    ys: np.ndarray         # solo decode occupancy y_s,i*
    served: np.ndarray     # planned prefill throughput mu_p,i x_i* (per server per unit time)
    value: float           # LP optimum R* (per server per unit time)
    M: int                 # mixed servers
    mu_p: np.ndarray
    mu_m: np.ndarray
    mu_s: np.ndarray
    tau_mix: float
    tau_solo: float
    EP: np.ndarray
    ED: np.ndarray
    info: dict = field(default_factory=dict)


def rates(cfg, n_mixed_decodes=None, n_solo_decodes=None):
    """Class service rates for the LP from the iteration-time law t = c0 + c_pre*ptok + c_dec*n."""
    K, B, C = cfg.K, cfg.B, cfg.C
    nm = (B - 1) if n_mixed_decodes is None else n_mixed_decodes
    nsd = B if n_solo_decodes is None else n_solo_decodes
    tau_mix = cfg.c0 + cfg.c_pre * C + cfg.c_dec * nm
    tau_solo = cfg.c0 + cfg.c_dec * nsd
    EP = np.zeros(K); ECH = np.zeros(K); ED = np.zeros(K)
    for i, c in enumerate(cfg.classes):
        EP[i], ECH[i] = length_moments(c.in_law, c.in_p0, c.in_p1, C, c.in_table)
        ED[i], _ = length_moments(c.out_law, c.out_p0, c.out_p1, C, c.out_table)
    sp = ECH * (cfg.c0 + cfg.c_dec * nm) + cfg.c_pre * EP
    return dict(mu_p=1.0 / sp, mu_m=1.0 / (ED * tau_mix), mu_s=1.0 / (ED * tau_solo),
                tau_mix=tau_mix, tau_solo=tau_solo, EP=EP, ED=ED, ECH=ECH)


def solve_lp(cfg, lam, objective="bundled", tbt_mixed_share=None, served_floor=None,
             n_mixed_decodes=None, n_solo_decodes=None, max_mixed_fraction=None) -> Plan:
    """Steady-state fluid LP with theta = 0 and q_d = 0 (decode-buffer elimination, Prop. 1).

    Variables per class: x_i, y_m,i, y_s,i. The prefill flow balance is relaxed to
    mu_p,i x_i <= lambda_i (the theta -> 0+ limit of the paper's constraint: an overloaded
    class keeps an unbounded prefill backlog instead of abandoning).
    Optional SLI rows (paper Sec. 5.2): `tbt_mixed_share` bounds, per class, the share of
    decode tokens emitted in mixed iterations; `served_floor` is a lower bound on every
    class's served fraction mu_p,i x_i / lambda_i (max-min fairness floor).
    `max_mixed_fraction` caps sum_i x_i (replanning with the mixed/solo split held where it is).
    """
    K, B = cfg.K, cfg.B
    lam = np.asarray(lam, dtype=np.float64)
    r = rates(cfg, n_mixed_decodes, n_solo_decodes)
    mu_p, mu_m, mu_s = r["mu_p"], r["mu_m"], r["mu_s"]
    pin = np.array([c.price_in for c in cfg.classes]); pout = np.array([c.price_out for c in cfg.classes])
    w = pin * r["EP"] + pout * r["ED"]
    nv = 3 * K
    ix, im, isx = (lambda i: i), (lambda i: K + i), (lambda i: 2 * K + i)
    cost = np.zeros(nv)
    for i in range(K):
        if objective == "bundled":
            cost[im(i)] -= w[i] * mu_m[i]; cost[isx(i)] -= w[i] * mu_s[i]
        else:
            cost[ix(i)] -= pin[i] * r["EP"][i] * mu_p[i]
            cost[im(i)] -= pout[i] * r["ED"][i] * mu_m[i]; cost[isx(i)] -= pout[i] * r["ED"][i] * mu_s[i]
    A_ub, b_ub, A_eq, b_eq = [], [], [], []
    row = np.zeros(nv); row[:K] = 1; A_ub.append(row); b_ub.append(1.0 if max_mixed_fraction is None else float(max_mixed_fraction))
    row = np.zeros(nv); row[K:2 * K] = 1; row[:K] = -(B - 1); A_ub.append(row); b_ub.append(0.0)
    row = np.zeros(nv); row[2 * K:] = 1; row[:K] = B; A_ub.append(row); b_ub.append(float(B))
    for i in range(K):
        row = np.zeros(nv); row[ix(i)] = mu_p[i]; A_ub.append(row); b_ub.append(lam[i])
        row = np.zeros(nv); row[ix(i)] = mu_p[i]; row[im(i)] = -mu_m[i]; row[isx(i)] = -mu_s[i]
        A_eq.append(row); b_eq.append(0.0)
        if tbt_mixed_share is not None:
            a = tbt_mixed_share
            row = np.zeros(nv); row[im(i)] = (1 - a) / r["tau_mix"]; row[isx(i)] = -a / r["tau_solo"]
            A_ub.append(row); b_ub.append(0.0)
        if served_floor is not None:
            row = np.zeros(nv); row[ix(i)] = -mu_p[i]; A_ub.append(row); b_ub.append(-served_floor * lam[i])
    res = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub), A_eq=np.array(A_eq), b_eq=np.array(b_eq),
                  bounds=[(0, None)] * nv, method="highs")
    if res.status != 0:
        raise RuntimeError(f"fluid LP failed: {res.message}")
    x = np.maximum(res.x[:K], 0.0); ym = np.maximum(res.x[K:2 * K], 0.0); ys = np.maximum(res.x[2 * K:], 0.0)
    M = int(min(cfg.N, math.ceil(cfg.N * float(x.sum()) - 1e-9)))
    return Plan(x=x, ym=ym, ys=ys, served=mu_p * x, value=-float(res.fun), M=M, mu_p=mu_p, mu_m=mu_m, mu_s=mu_s,
                tau_mix=r["tau_mix"], tau_solo=r["tau_solo"], EP=r["EP"], ED=r["ED"])


def solo_probabilities(plan: Plan) -> np.ndarray:
    """p_s,i = mu_s,i y_s,i* / (mu_m,i y_m,i* + mu_s,i y_s,i*), 1 where the denominator vanishes: the share of
    class-i decode service the plan gives to solo servers (paper Sec. 5.2, randomized decode router)."""
    a = plan.mu_s * plan.ys
    b = plan.mu_m * plan.ym
    return np.where(a + b > 0.0, a / np.where(a + b > 0.0, a + b, 1.0), 1.0)


def selection_weights(plan: Plan):
    """(varpi_s, varpi_m): the class shares of the planned decode completion rate of the solo and of the mixed pool,
    varpi_s,i = mu_s,i y_s,i* / sum_j mu_s,j y_s,j* and likewise for the mixed pool, 0/0 = 0 (paper EC, "General
    SLI-aware Extension")."""
    a = plan.mu_s * plan.ys
    b = plan.mu_m * plan.ym
    return (a / a.sum() if a.sum() > 0.0 else np.zeros_like(a)), (b / b.sum() if b.sum() > 0.0 else np.zeros_like(b))


def capacity_scale(cfg, mix, tbt_mixed_share=None, **kw) -> float:
    """Largest s such that arrivals s*mix are served in full by the fluid LP (all classes at 100 %),
    under the optional per-class bound on the share of decode tokens emitted in mixed iterations."""
    K, B = cfg.K, cfg.B
    mix = np.asarray(mix, dtype=np.float64)
    r = rates(cfg, kw.get("n_mixed_decodes"), kw.get("n_solo_decodes"))
    mu_p, mu_m, mu_s = r["mu_p"], r["mu_m"], r["mu_s"]
    nv = 3 * K + 1  # + s
    cost = np.zeros(nv); cost[-1] = -1.0
    A_ub, b_ub, A_eq, b_eq = [], [], [], []
    row = np.zeros(nv); row[:K] = 1; A_ub.append(row); b_ub.append(1.0)
    row = np.zeros(nv); row[K:2 * K] = 1; row[:K] = -(B - 1); A_ub.append(row); b_ub.append(0.0)
    row = np.zeros(nv); row[2 * K:3 * K] = 1; row[:K] = B; A_ub.append(row); b_ub.append(float(B))
    for i in range(K):
        row = np.zeros(nv); row[i] = mu_p[i]; row[-1] = -mix[i]; A_eq.append(row); b_eq.append(0.0)
        row = np.zeros(nv); row[i] = mu_p[i]; row[K + i] = -mu_m[i]; row[2 * K + i] = -mu_s[i]
        A_eq.append(row); b_eq.append(0.0)
        if tbt_mixed_share is not None:
            a = tbt_mixed_share
            row = np.zeros(nv); row[K + i] = (1 - a) / r["tau_mix"]; row[2 * K + i] = -a / r["tau_solo"]
            A_ub.append(row); b_ub.append(0.0)
    res = linprog(cost, A_ub=np.array(A_ub), b_ub=np.array(b_ub), A_eq=np.array(A_eq), b_eq=np.array(b_eq),
                  bounds=[(0, None)] * nv, method="highs")
    if res.status != 0:
        raise RuntimeError(f"capacity LP failed: {res.message}")
    return float(res.x[-1])


def estimate_rates(arrivals_now, arrivals_before, n_servers, t_now, window, rho=3.0, lam_min=1e-6, eps=1e-9):
    """Conservative per-server class arrival rates from a rolling window (paper, online adaptive algorithm,
    Eq. main-online-arrival-estimate): N_i = A_i(t) - A_i((t - W)^+), W_eff = min{W, max{t, eps}},
    lambda_i = max{rho * N_i / (n * W_eff), lam_min}. `arrivals_*` are cumulative counts per class at t and at
    (t - W)^+; times in seconds."""
    n_i = np.asarray(arrivals_now, dtype=np.float64) - np.asarray(arrivals_before, dtype=np.float64)
    w_eff = min(float(window), max(float(t_now), float(eps)))
    return np.maximum(float(rho) * n_i / (float(n_servers) * w_eff), float(lam_min))


def replan(cfg, lam_hat, hold_split=True, **kw) -> Plan:
    """Re-solves the fluid LP for new rate estimates (paper, online adaptive algorithm: the LP is re-solved with
    the estimates in place of lambda_i). The plan's x are the gate's new occupancy targets. With `hold_split`
    the mixed/solo split stays at cfg.M servers (sum_i x_i <= M/N); without it the plan's M is the new split
    M*(t_k) = ceil(n sum_i x_i*(t_k)) (Eq. main-online-mixed-target)."""
    if hold_split:
        return solve_lp(cfg, lam_hat, max_mixed_fraction=cfg.M / cfg.N, **kw)
    return solve_lp(cfg, lam_hat, **kw)


def erlang_c(c: int, a: float) -> float:
    """Erlang-C delay probability for c servers and offered load a < c."""
    s = 0.0; term = 1.0
    for k in range(c):
        if k: term *= a / k
        s += term
    last = term * a / c if c else 1.0
    last = last / (1.0 - a / c)
    return last / (s + last)
