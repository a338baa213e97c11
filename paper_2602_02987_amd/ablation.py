"""Component ablation on synthetic instances (paper EC, "Additional Ablation Studies on Synthetic Workloads").

Five policies are run on the same seeded instances and compared by their revenue rate relative to the fluid
optimum R* of the instance. A policy is a prefill rule, a decode rule and a planning rule:

    GG-SP   occupancy gate, solo-first router, planned mixed/solo split   (the full gate-and-route policy)
    FG-SP   FCFS admission, solo-first router, planned split
    GF-WSP  occupancy gate, least-loaded router over all servers, no split (every server may prefill)
    GI-WSP  occupancy gate, decode continues on the prefill's server, no split
    FI-WSP  FCFS admission, decode continues on the prefill's server, no split

The instances follow the ranges the paper states (mixed-iteration intercept alpha in [0.02, 0.15] s, slope beta in
[1e-5, 1e-3] s per chunk token, solo token rate gamma in [10, 50] per s, mean lengths in [200, 3000], arrival
rates in [0.25, 0.5] per server, n = 500); what it does not state is chosen here: two classes, geometric lengths,
batch size B in {8, 16, 32}, chunk 256, patience rate 0.1, bundled prices 0.1 / 0.2 per token.
This module only builds configurations and reads tallies; the simulation runs in the library.
"""
from __future__ import annotations

from dataclasses import replace

import numpy as np

from . import plan as _plan
from . import workloads as W

POLICIES = ("GG-SP", "FG-SP", "GF-WSP", "GI-WSP", "FI-WSP")


def instances(count: int, seed: int = 20260301, n: int = 500, seeds: int = 3):
    """`count` seeded instances (planned with the occupancy LP; the plan's split M is what "SP" keeps)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        alpha, beta = rng.uniform(0.02, 0.15), float(np.exp(rng.uniform(np.log(1e-5), np.log(1e-3))))
        gamma = rng.uniform(10.0, 50.0)
        tau_solo, tau_mix, C = 1.0 / gamma, alpha + beta * 256, 256
        if tau_mix < tau_solo:        # the iteration-time law here has one intercept: a chunk cannot make it shorter
            continue
        P = rng.uniform(200.0, 3000.0, 2); D = rng.uniform(200.0, 3000.0, 2)
        lam = rng.uniform(0.25, 0.5, 2)
        B = int(rng.choice([8, 16, 32]))
        cls = [W.SimClass(lam=float(lam[i]), in_p0=float(P[i]), out_p0=float(D[i]), price_in=0.1, price_out=0.2,
                          bundled=1, theta=0.1, priority=float(D[i] / P[i])) for i in range(2)]
        dt = min(tau_solo, 0.04 / float(lam.sum()))          # at most 0.04 arrivals per server-step
        cfg = W.SimConfig(name=f"ablation-{len(out)}", K=2, N=n, B=B, C=C, c0=tau_solo, dt=dt,
                          c_pre=(tau_mix - tau_solo) / C, c_dec=0.0, classes=cls, replications=seeds, seed=1 + len(out),
                          queue_cap=1 << 14, dbuf_cap=1 << 14)
        out.append(W.with_plan(cfg, objective="bundled"))
    return out


def policies(cfg):
    """The five policies as configurations of the same instance."""
    full = replace(cfg, gate_mode=W.GATE_OCCUPANCY, route_mode=W.ROUTE_SOLO_FIRST)
    return {"GG-SP": full,
            "FG-SP": replace(full, gate_mode=W.GATE_FCFS),
            "GF-WSP": replace(full, M=cfg.N),
            "GI-WSP": replace(full, route_mode=W.ROUTE_IMMEDIATE, M=cfg.N),
            "FI-WSP": replace(full, gate_mode=W.GATE_FCFS, route_mode=W.ROUTE_IMMEDIATE, M=cfg.N)}


def revenue_rate(make_sim, cfg, warm_time: float, measure_time: float):
    """Per-server bundled revenue per unit time of every replication, after a warm-up (`make_sim(cfg)` returns an
    object with run(steps) and stats(); tallies are read per replication)."""
    from .binding import TALLY
    ti = {n: i for i, n in enumerate(TALLY)}
    dt = cfg.dt if cfg.dt > 0.0 else cfg.c0
    warm, meas = int(round(warm_time / dt)), int(round(measure_time / dt))
    sim = make_sim(cfg)
    sim.run(warm)
    t0 = np.stack([sim.tallies(r)[0][:cfg.K].astype(np.float64) for r in range(cfg.replications)])
    sim.run(meas)
    t1 = np.stack([sim.tallies(r)[0][:cfg.K].astype(np.float64) for r in range(cfg.replications)])
    t = t1 - t0
    pin = np.array([c.price_in for c in cfg.classes]); pout = np.array([c.price_out for c in cfg.classes])
    return (t[:, :, ti["TOKP_DEC"]] * pin + t[:, :, ti["TOKD_DEC"]] * pout).sum(axis=1) / (cfg.N * meas * dt)


def study(make_sim, count: int = 8, warm_time: float = 1500.0, measure_time: float = 3000.0, **kw):
    """Revenue of every policy on every instance, relative to the instance's R*: array [instance][policy]."""
    rows = []
    for cfg in instances(count, **kw):
        r_star = cfg.notes["lp_value"]
        rows.append([float(revenue_rate(make_sim, c, warm_time, measure_time).mean()) / r_star
                     for c in policies(cfg).values()])
    return np.array(rows)


def main():
    from . import binding
    res = study(binding.Sim)
    print("instance  " + "  ".join(f"{p:>7s}" for p in POLICIES))
    for i, row in enumerate(res):
        print(f"{i:8d}  " + "  ".join(f"{v:7.3f}" for v in row))
    print("    mean  " + "  ".join(f"{v:7.3f}" for v in res.mean(axis=0)))
    print("     std  " + "  ".join(f"{v:7.3f}" for v in res.std(axis=0)))


if __name__ == "__main__":
    main()
