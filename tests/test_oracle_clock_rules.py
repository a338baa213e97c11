"""Pin of the oracle's iteration clock (paper Sec. 2.2: an iteration lasts c0 + c_pre * prefill tokens of its chunk
+ c_dec * decodes in the batch; readings: the batch is frozen when the iteration starts, a server that completes an
iteration restarts back to back from its own clock, an idle server that gets work starts at the step boundary, a
decode placed in mid-iteration does not change the running iteration). Replayed for every server and step from
consecutive snapshots. CPU only."""
import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import _heavy

IDLE = np.iinfo(np.int64).max


@pytest.mark.parametrize("over", [dict(), dict(M=12), dict(M=1, B=2), dict(dt=0.004)])
def test_clocks_replayed_step_by_step(oracle_mod, over):
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, replications=1, **over)
    c0, cpre, cdec = (int(round(v * 1e9)) for v in (cfg.c0, cfg.c_pre, cfg.c_dec))
    dt = int(round(cfg.dt * 1e9)) if cfg.dt > 0 else c0
    o = oracle_mod.Oracle(cfg)
    prev = None
    restarts = starts = joins = 0
    for s in range(1500):
        o.run(1)
        sv, sl = o.servers(0), o.slots(0)
        T = (s + 1) * dt
        cur = dict(t=sv["t_next"].copy(), it=sv["iter"].copy(), rem=sv["rem"].copy(), ptok=sv["ptok"].copy(), nd=sl["n_dec"].copy())
        if prev is not None:
            for g in range(cfg.N):
                was_busy = prev["t"][g] != IDLE
                due = was_busy and prev["t"][g] <= T
                has_work = cur["nd"][g] > 0 or cur["rem"][g] > 0
                if was_busy and not due:                       # the running iteration goes on, whatever was placed
                    assert cur["t"][g] == prev["t"][g] and cur["it"][g] == prev["it"][g] and cur["ptok"][g] == prev["ptok"][g]
                    joins += int(cur["nd"][g] > prev["nd"][g])
                    continue
                assert cur["it"][g] == prev["it"][g] + (1 if due else 0)
                if not has_work:
                    assert cur["t"][g] == IDLE and cur["ptok"][g] == 0
                    continue
                chunk = min(cfg.C, int(cur["rem"][g]))
                assert cur["ptok"][g] == chunk
                base = int(prev["t"][g]) if due else T
                assert cur["t"][g] == base + c0 + cpre * chunk + cdec * int(cur["nd"][g]), (over, s, g)
                restarts += int(due); starts += int(not due)
        prev = cur
    assert restarts > 2000 and starts > 5 and (joins > 0 or cfg.B <= 2)


def test_every_decode_runs_exactly_its_output_length(oracle_mod):
    """A request with D output tokens leaves its server when the server has completed exactly D iterations
    that had it in the batch: iterations are counted from the restart that follows the placement (one more
    if the server was in mid-iteration when the request arrived)."""
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, replications=1)
    dt = int(round(cfg.c0 * 1e9))
    o = oracle_mod.Oracle(cfg)
    prev_jobs = {g: [] for g in range(cfg.N)}
    prev_t = np.full(cfg.N, IDLE, dtype=np.int64)
    born = {}
    checked = mid_seen = 0
    for s in range(2500):
        o.run(1)
        sv, sl = o.servers(0), o.slots(0)
        T = (s + 1) * dt
        for g in range(cfg.N):
            now = [int(v) for v in sl["job"][g, :sl["n_dec"][g]]]
            was_mid = prev_t[g] != IDLE and prev_t[g] > T
            a, b = list(prev_jobs[g]), list(now)
            for jw in list(a):
                if jw in b:
                    a.remove(jw); b.remove(jw)
            for jw in a:                                    # left in this step
                it0, mid = born.pop((g, jw))
                D = (jw >> 48) + 1
                assert int(sv["iter"][g]) == it0 + D + mid, (s, g, jw)
                checked += 1
            for jw in b:                                    # placed in this step
                born[(g, jw)] = (int(sv["iter"][g]), int(was_mid))
                mid_seen += int(was_mid)
            prev_jobs[g] = now
        prev_t = sv["t_next"].copy()
    assert checked > 500 and mid_seen > 5
