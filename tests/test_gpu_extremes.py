"""GPU parity at the edges of the parameter ranges: a step far shorter than an iteration, one-token chunks,
patience of one step and patience beyond the table's clamp, arrival rates modulated down to zero, iterations
that span dozens of steps, and classes the plan never admits."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, _limits_cfg, _limits_class, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import TI, _heavy

pytestmark = pytest.mark.gpu


def _cases():
    h = _heavy()
    yield "short-step", replace(h, dt=h.c0 / 40.0, classes=[replace(c, lam=c.lam * 8.0) for c in h.classes]), 40000
    yield "one-token-chunks", replace(h, C=1, classes=[replace(c, in_law=W.LAW_GEOMETRIC, in_p0=6.0) for c in h.classes]), 4000
    yield "patience-one-step", replace(h, classes=[replace(c, theta=1000.0) for c in h.classes]), 3000
    yield "patience-clamped", replace(h, classes=[replace(c, theta=1e-6) for c in h.classes]), 3000
    calm = [replace(c, lam=c.lam * 0.45) for c in h.classes]     # (the peak rate stays within the sampler's range)
    yield "rate-to-zero", replace(h, mod_amp=1.0, mod_period=7, classes=calm), 3000
    yield "rate-to-zero-slow", replace(h, mod_amp=-1.0, mod_period=1500, classes=calm), 4000
    yield "long-iterations", replace(h, c0=0.001, c_pre=0.0, c_dec=0.005, dt=0.0, classes=[replace(c, lam=c.lam * 0.2) for c in h.classes]), 20000
    yield "never-admitted", replace(h, x_star=[0.0, 0.3, 0.0], queue_cap=25), 3000
    yield "nobody-admitted", replace(h, x_star=[0.0, 0.0, 0.0]), 1500
    yield "all-random-split-mixed", replace(h, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.0, 0.0, 0.0]), 3000
    yield "all-random-split-solo", replace(h, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[1.0, 1.0, 1.0]), 3000


@pytest.mark.parametrize("name,cfg,steps", list(_cases()), ids=[c[0] for c in _cases()])
def test_extreme_parameters(B, oracle_mod, name, cfg, steps):
    cfg = replace(cfg, name=name)
    sim, orc = run_both(B, oracle_mod, cfg, steps, checkpoints=3)
    ss, os_ = sim.stats(), orc.stats()
    assert_stats_equal(ss, os_)
    assert ss["overflow"] == bool(os_["glob"][5])
    t = os_["tally"]
    if name == "patience-one-step":
        assert t[:, TI["AB_P"]].sum() > 20 and t[:, TI["AB_D"]].sum() > 100   # nobody waits a second step
    if name == "patience-clamped":
        assert t[:, TI["AB_P"]].sum() == 0 and t[:, TI["AB_D"]].sum() == 0
    if name == "nobody-admitted":
        assert t[:, TI["U_P"]].sum() == 0 and t[:, TI["A"]].sum() > 0
    if name == "never-admitted":
        assert t[0, TI["U_P"]] == 0 and t[2, TI["U_P"]] == 0 and t[1, TI["U_P"]] > 0 and t[0, TI["DROP_P"]] > 0
    if name == "one-token-chunks":
        assert t[:, TI["TOK_PREF"]].sum() == os_["glob"][0] > 1000          # one prompt token per mixed iteration
