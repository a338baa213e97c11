"""Pins of the oracle's prefill gate (paper Sec. 4, "Dynamic control": admit the waiting class with the smallest
occupancy deviation (X_i - n x_i*)/x_i*, ties by the larger backlog deviation Q_p,i - n q_p,i*; Sec. 5.1: the class
with the largest static priority index; and the FCFS ablation). The rule is re-stated here in a few lines of
Python and replayed on the gate's inputs of every step, which are known from the end-of-step state and the
step's counts: Q_p before the gate = previous Q_p + arrivals, X before the gate = previous X - prefill
completions, idle prefill slots = M - sum X. CPU only."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

from test_oracle_dynamics import TI, _heavy


def _admissions(mode, cfg, qp, x, fifo, n_slots):
    """Admissions per class of one step: one idle slot after the other, state updated in between."""
    K, N = cfg.K, cfg.N
    out = np.zeros(K, dtype=np.int64)
    qp = qp.copy(); x = x.copy()
    for _ in range(n_slots):
        waiting = [i for i in range(K) if qp[i] > 0]
        if mode == W.GATE_OCCUPANCY:
            waiting = [i for i in waiting if cfg.x_star[i] > 0.0]
        if not waiting:
            break
        if mode == W.GATE_OCCUPANCY:
            key = lambda i: ((float(x[i]) - N * cfg.x_star[i]) * (1.0 / cfg.x_star[i]), -(float(qp[i]) - N * cfg.qp_star[i]), i)
        elif mode == W.GATE_PRIORITY:
            key = lambda i: (-cfg.classes[i].priority, i)
        else:
            key = lambda i: (fifo[i][0], i)
        k = min(waiting, key=key)
        out[k] += 1; qp[k] -= 1; x[k] += 1
        fifo[k].pop(0)
    return out


@pytest.mark.parametrize("mode", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_gate_decisions_replayed_step_by_step(oracle_mod, mode):
    for over in (dict(), dict(M=9, x_star=[0.2, 0.0, 0.05]), dict(M=12, qp_star=[3.0, 0.0, 0.4], x_star=[0.1, 0.1, 0.1])):
        cfg = _heavy(mode, queue_cap=100000, dbuf_cap=100000, replications=1, **over)
        if mode == W.GATE_PRIORITY:
            cfg.classes = [replace(c, priority=p) for c, p in zip(cfg.classes, (0.9, 1.5, 0.9))]   # a tie in the index
        o = oracle_mod.Oracle(cfg)
        fifo = [[] for _ in range(cfg.K)]
        prev_t = np.zeros((cfg.K, len(TI)), dtype=np.int64)
        prev = dict(Qp=np.zeros(cfg.K, np.int64), X=np.zeros(cfg.K, np.int64))
        decided = 0
        for s in range(3000):
            o.run(1)
            t = o.tallies(0)[0].astype(np.int64)
            d = t - prev_t
            arr, sp, up = d[:, TI["A"]], d[:, TI["S_P"]], d[:, TI["U_P"]]
            for k in range(cfg.K):
                fifo[k] += [s] * int(arr[k])
            qp_in = prev["Qp"] + arr
            x_in = prev["X"] - sp
            want = _admissions(mode, cfg, qp_in, x_in, fifo, cfg.M - int(x_in.sum()))
            assert np.array_equal(up, want), (over, s, up, want)
            decided += int(want.sum() > 0 and (qp_in > 0).sum() > 1)
            cs = o.class_state(0)
            prev = dict(Qp=cs["Qp"].copy(), X=cs["X"].copy())
            assert np.array_equal(prev["Qp"], qp_in - want) and np.array_equal(prev["X"], x_in + want)
            prev_t = t
        assert decided > 50      # steps in which the gate really had to choose between classes
        if mode == W.GATE_OCCUPANCY and "x_star" in over and over["x_star"][1] == 0.0:
            assert t[1, TI["U_P"]] == 0 and t[1, TI["A"]] > 0   # a class without a target is never admitted
