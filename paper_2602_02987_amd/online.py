"""Host-side loop of the paper's online adaptive algorithm (trace-driven online policy evaluation, "Online adaptive
algorithm"): every replanning epoch the class arrival rates are re-estimated from a rolling window
(Eq. main-online-arrival-estimate), the fluid LP is re-solved, and the gate's targets and the mixed/solo split
M*(t_k) (Eq. main-online-mixed-target) are handed to the simulation, which goes on from its current state.

The loop drives anything that offers run / stats / set_targets / set_split; none of the simulation's arithmetic
is here. The paper's settings are a 30 s window, replanning every 10 s and a safety factor rho = 3.
"""
from __future__ import annotations

import numpy as np

from . import plan as _plan

_A = 0   # index of the arrival count among the per-class tallies


def run_online(sim, cfg, steps, replan_every, window, rho=3.0, lam_min=1e-6, eps=1e-9, move_split=True,
               on_epoch=None, **lp_options):
    """Runs `steps` steps in epochs of `replan_every` steps; `window` (steps) should be a multiple of the epoch.
    Returns the list of (step, lambda_hat, plan) the controller went through."""
    dt = cfg.dt if cfg.dt > 0 else cfg.c0
    K, reps = cfg.K, cfg.replications
    seen = {0: np.zeros(K)}
    log = []
    done = 0
    while done < steps:
        n = min(replan_every, steps - done)
        sim.run(n)
        done += n
        seen[done] = sim.stats()["tally"][:K, _A].astype(np.float64) / reps
        back = max(done - window, 0)
        back = max(s for s in seen if s <= back)
        lam_hat = _plan.estimate_rates(seen[done], seen[back], cfg.N, done * dt, window * dt, rho, lam_min, eps)
        plan = _plan.replan(cfg, lam_hat, hold_split=not move_split, **lp_options)
        sim.set_targets([float(v) for v in plan.x], [0.0] * K)
        if move_split:
            sim.set_split(plan.M)
        log.append((done, lam_hat, plan))
        if on_epoch is not None:
            on_epoch(done, lam_hat, plan)
    return log
