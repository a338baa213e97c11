"""Config 5 at its full size, in the launch shape the benchmark times, checked by what holds at any size (the
oracle cannot follow 256 replications of 10000 servers): the balance equations of Sec. 2.3 as exact integer
identities between the cumulative tallies and the state, the capacity constraints, buffer contents against the
class counters, token conservation — for the base policy and for the most involved variant (abandonment with the
weighted router)."""
import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from test_gpu_parity import B  # noqa: F401  (fixture)
from test_oracle_dynamics import TI

pytestmark = pytest.mark.gpu


def _check(sim, cfg, reps):
    K = cfg.K
    st = sim.stats()
    assert not st["overflow"]
    for r in reps:
        t = sim.tallies(r)[0][:K].astype(np.int64)
        sn = sim.snapshot(r)
        g = lambda n: t[:, TI[n]]   # noqa: E731
        assert np.array_equal(g("A") - g("DROP_P") - g("U_P") - g("AB_P"), sn["Qp"][:K]), (r, "Q_p")
        assert np.array_equal(g("U_P") - g("S_P"), sn["X"][:K]), (r, "X")
        assert np.array_equal(g("S_P") - g("DROP_D") - g("U_DM") - g("U_DS") - g("AB_D"), sn["Qd"][:K]), (r, "Q_d")
        assert np.array_equal(g("U_DM") + g("M_SM") - g("M_MS") - g("S_DM"), sn["Ym"][:K]), (r, "Y_m")
        assert np.array_equal(g("U_DS") - g("M_SM") + g("M_MS") - g("S_DS"), sn["Ys"][:K]), (r, "Y_s")
        nd, rem = sn["n_dec"], sn["rem"]
        assert (rem > 0).sum() == sn["X"][:K].sum() and (rem[cfg.M:] > 0).sum() == 0       # prefills on mixed servers only
        assert nd.max() <= cfg.B and nd[:cfg.M].max() <= cfg.B - 1                       # decode slots per server
        assert nd.sum() == (sn["Ym"][:K] + sn["Ys"][:K]).sum()
        assert nd[rem > 0].sum() == sn["Ym"][:K].sum()                                  # mixed decodes sit beside a prefill
        assert len(sn["dbuf"]) + len(sn["dbuf_m"]) == sn["Qd"][:K].sum()
        for k in range(K):
            assert len(sn["queues"][k]) == sn["Qp"][k]
            assert np.all(np.diff(sn["queues"][k].astype(np.int64)) >= 0)                # FCFS: arrival stamps in order
        # tokens: every completed decode emitted its whole output; emitted >= completed outputs
        assert g("TOK_EMIT").sum() >= g("TOKD_DEC").sum() and g("TOK_PREF").sum() >= g("TOKP_PRE").sum()
    # the replications are different sample paths of one law: their completion counts agree to a few percent
    done = np.array([sim.tallies(r)[0][:K, TI["S_DS"]].sum() + sim.tallies(r)[0][:K, TI["S_DM"]].sum() for r in reps], dtype=np.float64)
    assert done.std() / done.mean() < 0.05 and len(set(done)) > 1


def test_base_policy(B):
    cfg = W.config(5)
    sim = B.Sim(cfg)
    for _ in range(12):
        sim.run(2000)
    _check(sim, cfg, range(0, cfg.replications, 32))


def test_abandonment_with_the_weighted_router(B):
    base = W.config(5)
    cfg = W.with_weighted_split(base, lam_plan=[c.lam / 0.95 for c in base.classes])
    for c in cfg.classes:
        c.theta = 0.1
    sim = B.Sim(cfg)
    for _ in range(12):
        sim.run(2000)
    _check(sim, cfg, range(5, cfg.replications, 32))
    t = sim.stats()["tally"]
    assert t[:, TI["AB_P"]].sum() > 0
