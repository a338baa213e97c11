"""Pin of the oracle's decode router (paper Sec. 4, decode routing: solo group first, then the mixed group, else
the FCFS decode buffer; here with the least-loaded feasible server, lowest index on ties). The rule is re-stated in
Python and replayed on every step's inputs, which follow from two consecutive snapshots: the decodes that left,
the prefills that completed (in server order, behind the buffer's content), and the loads the router saw.
CPU only."""
import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import TI, _heavy


def _route(cfg, loads, jobs):
    """Sequential rule: every job to the least-loaded server of the solo group with a free slot (cap B), else of
    the mixed group (cap B-1), lowest index on ties; the first job that fits nowhere stops the step."""
    placed = {}
    loads = loads.copy()
    n = 0
    for jw in jobs:
        dst = -1
        for lo, hi, cap in ((cfg.M, cfg.N, cfg.B), (0, cfg.M, cfg.B - 1)):
            cand = [g for g in range(lo, hi) if loads[g] < cap]
            if cand:
                dst = min(cand, key=lambda g: (loads[g], g))
                break
        if dst < 0:
            break
        placed.setdefault(dst, []).append(jw)
        loads[dst] += 1
        n += 1
    return placed, loads, jobs[n:]


@pytest.mark.parametrize("over", [dict(), dict(M=1), dict(M=11), dict(B=1, M=6), dict(M=0), dict(M=12)])
def test_placements_replayed_step_by_step(oracle_mod, over):
    cfg = _heavy(queue_cap=100000, dbuf_cap=100000, replications=1, **over)
    o = oracle_mod.Oracle(cfg)
    prev_sl = {g: [] for g in range(cfg.N)}
    prev_sv = dict(rem=np.zeros(cfg.N, np.int32), pfjob=np.zeros(cfg.N, np.uint64))
    buf = []
    used_mixed = waited = 0
    for s in range(1500):
        o.run(1)
        sl, sv = o.slots(0), o.servers(0)
        now = {g: sorted(int(v) for v in sl["job"][g, :sl["n_dec"][g]]) for g in range(cfg.N)}
        # prefills that completed in this step, in server order: they join the buffer behind what waited
        done = [int(prev_sv["pfjob"][g]) for g in range(cfg.N)
                if prev_sv["rem"][g] > 0 and (sv["rem"][g] == 0 or sv["pfjob"][g] != prev_sv["pfjob"][g])]
        jobs = buf + done
        # decodes that stayed: what is there now and was there before (request words are unique: stamp, lengths, class
        # may coincide in rare cases, so multisets are compared)
        stayed = {}
        for g in range(cfg.N):
            a, b = list(prev_sl[g]), list(now[g])
            keep = []
            for jw in a:
                if jw in b:
                    b.remove(jw); keep.append(jw)
            stayed[g] = keep
        loads = np.array([len(stayed[g]) for g in range(cfg.N)])
        placed, after, left = _route(cfg, loads, jobs)
        for g in range(cfg.N):
            assert sorted(stayed[g] + placed.get(g, [])) == now[g], (over, s, g)
        assert [int(v) for v in o.queue(0, -1)] == left, (over, s)
        used_mixed += sum(len(v) for g, v in placed.items() if g < cfg.M)
        waited += len(left) > 0
        buf = left
        prev_sl = now
        prev_sv = dict(rem=sv["rem"].copy(), pfjob=sv["pfjob"].copy())
    if not over:
        assert used_mixed > 50 and waited > 50     # both groups and the buffer were in play
