"""Element-by-element comparison of the HIP library's state with the oracle's (test helper)."""
import numpy as np

from oracle.binding import canonical_slots

IDLE = np.iinfo(np.int64).max


def assert_replication_equal(sim, orc, r, ro=None, what=""):
    """Integer state, tallies, histograms and digest of replication r: bit-exact."""
    ro = r if ro is None else ro
    cfg = sim.cfg
    tag = f"{what} rep {r}"
    s = sim.snapshot(r)
    oc = orc.class_state(ro)
    for name in ("Qp", "X", "Qd", "Ym", "Ys"):
        assert np.array_equal(s[name], oc[name]), (tag, name, s[name], oc[name])
    osv = orc.servers(ro)
    for name in ("t_next", "iter", "rem", "ptok", "pfjob", "n_cls", "n_join"):
        if not np.array_equal(s[name], osv[name]):
            bad = np.nonzero(np.any((s[name] != osv[name]).reshape(cfg.N, -1), axis=1))[0]
            raise AssertionError((tag, name, "servers", bad[:8], s[name][bad[:4]], osv[name][bad[:4]]))
    osl = orc.slots(ro)
    ssl = canonical_slots(s["fin"], s["job"], s["n_dec"])
    assert np.array_equal(ssl["n_dec"], osl["n_dec"]), (tag, "n_dec")
    assert np.array_equal(ssl["fin"], osl["fin"]), (tag, "slot fin")
    assert np.array_equal(ssl["job"], osl["job"]), (tag, "slot job")
    for k in range(cfg.K):
        assert np.array_equal(s["queues"][k], orc.queue(ro, k)), (tag, "queue", k)
        assert np.array_equal(s["queue_dl"][k], orc.queue_deadlines(ro, k)), (tag, "queue deadlines", k)
    assert np.array_equal(s["dbuf"], orc.queue(ro, -1)), (tag, "decode buffer")
    assert np.array_equal(s["dbuf_dl"], orc.queue_deadlines(ro, -1)), (tag, "decode buffer deadlines")
    assert np.array_equal(s["dbuf_m"], orc.queue(ro, -2)), (tag, "decode buffer of the mixed group")
    st, sg = sim.tallies(r)
    ot, og = orc.tallies(ro)
    assert np.array_equal(st, ot), (tag, "tallies", np.nonzero(st != ot), st[st != ot], ot[st != ot])
    assert np.array_equal(sg, og), (tag, "global tallies", sg, og)
    for which in range(3):
        assert np.array_equal(sim.hist(r, which), orc.hist(ro, which)), (tag, "hist", which)
    assert sim.digest(r) == orc.digest(ro), (tag, "digest")


def assert_stats_equal(ss, os_, rel=1e-12):
    """Totals bit-exact; derived fp64 figures within `rel`."""
    for name, ov in os_.items():
        sv = ss[name]
        if name in ("tally", "glob", "K", "replications", "steps"):
            assert np.array_equal(np.asarray(sv), np.asarray(ov)), name
        else:
            assert np.allclose(np.asarray(sv, dtype=np.float64), np.asarray(ov, dtype=np.float64), rtol=rel, atol=0.0), name
