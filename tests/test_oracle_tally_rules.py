"""Pin of the oracle's tallies (paper Sec. 2.3 revenue recognition and counting processes; latency indicators of
the experiments): every step's increments of the token, latency, busy-time and revenue tallies are recomputed in
Python from the previous snapshot (which servers were due, which batch they had frozen, which requests they held)
and the requests that left, and must equal the oracle's increments exactly. CPU only."""
import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import GI, TI, _heavy

IDLE = np.iinfo(np.int64).max


def _unpack(jw):
    jw = int(jw)
    return dict(stamp=jw & ((1 << 29) - 1), cls=(jw >> 29) & 7, P=((jw >> 32) & 0xFFFF) + 1, D=((jw >> 48) & 0xFFFF) + 1)


@pytest.mark.parametrize("over", [dict(), dict(M=12), dict(M=2, B=3)])
def test_tally_increments_replayed_step_by_step(oracle_mod, over):
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, replications=1, **over)
    c0, cpre, cdec = (int(round(v * 1e9)) for v in (cfg.c0, cfg.c_pre, cfg.c_dec))
    dt = c0
    K = cfg.K
    o = oracle_mod.Oracle(cfg)
    prev = None
    prev_t = np.zeros((K, len(TI)), dtype=np.int64); prev_g = np.zeros(len(GI), dtype=np.int64)
    seen = dict(ttft=0, e2e=0, tbt=0)
    for s in range(1500):
        o.run(1)
        sv, sl = o.servers(0), o.slots(0)
        t, g_ = o.tallies(0)
        t = t.astype(np.int64); g_ = g_.astype(np.int64)
        cur = dict(t=sv["t_next"].copy(), rem=sv["rem"].copy(), ptok=sv["ptok"].copy(), pfjob=sv["pfjob"].copy(),
                   ncls=sv["n_cls"].astype(np.int64), njoin=sv["n_join"].astype(np.int64),
                   jobs={g: [int(v) for v in sl["job"][g, :sl["n_dec"][g]]] for g in range(cfg.N)})
        if prev is not None:
            T = (s + 1) * dt
            want = np.zeros((K, len(TI)), dtype=np.int64); wg = np.zeros(len(GI), dtype=np.int64)
            for g in range(cfg.N):
                if prev["t"][g] == IDLE or prev["t"][g] > T:
                    continue
                tc = int(prev["t"][g])                                      # exact completion time
                emit = prev["ncls"][g] - prev["njoin"][g]                   # the batch frozen at its start
                d = c0 + cpre * int(prev["ptok"][g]) + cdec * int(emit.sum())
                kind = "MIX" if prev["ptok"][g] > 0 else "SOLO"
                wg[GI["ITERS_" + kind]] += 1; wg[GI["BUSY_" + kind]] += d
                want[:, TI["TOK_EMIT"]] += emit[:K]; want[:, TI["TBT_SUM"]] += emit[:K] * d
                a, b = list(prev["jobs"][g]), list(cur["jobs"][g])
                for jw in list(a):
                    if jw in b:
                        a.remove(jw); b.remove(jw)
                for jw in a:                                                # decodes that emitted their last token
                    j = _unpack(jw)
                    mixed = prev["rem"][g] > 0
                    want[j["cls"], TI["S_DM" if mixed else "S_DS"]] += 1
                    want[j["cls"], TI["TOKP_DEC"]] += j["P"]; want[j["cls"], TI["TOKD_DEC"]] += j["D"]
                    want[j["cls"], TI["E2E_SUM"]] += tc - (j["stamp"] + 1) * dt
                    seen["e2e"] += 1
                if prev["ptok"][g] > 0:
                    j = _unpack(prev["pfjob"][g])
                    want[j["cls"], TI["TOK_PREF"]] += int(prev["ptok"][g])
                    if prev["rem"][g] == prev["ptok"][g]:                   # the last chunk: the prefill completes
                        want[j["cls"], TI["S_P"]] += 1; want[j["cls"], TI["TOKP_PRE"]] += j["P"]
                        want[j["cls"], TI["TTFT_SUM"]] += tc - (j["stamp"] + 1) * dt
                        seen["ttft"] += 1
                seen["tbt"] += int(emit.sum())
            got = t - prev_t
            for name in ("TOK_EMIT", "TBT_SUM", "S_DM", "S_DS", "TOKP_DEC", "TOKD_DEC", "E2E_SUM", "TOK_PREF", "S_P",
                         "TOKP_PRE", "TTFT_SUM"):
                assert np.array_equal(got[:, TI[name]], want[:, TI[name]]), (over, s, name)
            gg = g_ - prev_g
            for name in ("ITERS_MIX", "ITERS_SOLO", "BUSY_MIX", "BUSY_SOLO"):
                assert gg[GI[name]] == wg[GI[name]], (over, s, name)
            # end-of-step sums
            cs = o.class_state(0)
            for name, key in (("SUM_QP", "Qp"), ("SUM_QD", "Qd"), ("SUM_X", "X"), ("SUM_YM", "Ym"), ("SUM_YS", "Ys")):
                assert np.array_equal(got[:, TI[name]], cs[key]), (over, s, name)
        prev = cur; prev_t = t; prev_g = g_
    assert seen["ttft"] > 300 and seen["e2e"] > 300 and seen["tbt"] > 5000
    # revenue figures of sim_stats from the token sums (bundled: at completion; separate: prompt tokens at prefill end)
    st = o.stats()
    nt = cfg.N * st["sim_time"]
    for k, c in enumerate(cfg.classes):
        assert st["rev_bundled"][k] == pytest.approx((c.price_in * t[k, TI["TOKP_DEC"]] + c.price_out * t[k, TI["TOKD_DEC"]]) / nt, rel=1e-12)
        assert st["rev_separate"][k] == pytest.approx((c.price_in * t[k, TI["TOKP_PRE"]] + c.price_out * t[k, TI["TOKD_DEC"]]) / nt, rel=1e-12)
        assert st["ttft_mean"][k] == pytest.approx(t[k, TI["TTFT_SUM"]] * 1e-9 / max(t[k, TI["S_P"]], 1), rel=1e-12)
