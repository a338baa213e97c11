"""GPU parity with the smallest rings: class queues and decode buffers that hold one or two requests, so every
append, admission, staging pass and compaction wraps around, in every kernel variant."""
from dataclasses import replace

import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B, run_both  # noqa: F401  (B is a fixture)
from test_oracle_dynamics import _heavy

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("caps", [(1, 1), (2, 1), (1, 2), (3, 2)])
def test_rings_of_one_or_two_entries(B, oracle_mod, caps):
    qc, dc = caps
    for gate in (W.GATE_OCCUPANCY, W.GATE_FCFS):
        base = _heavy(gate, queue_cap=qc, dbuf_cap=dc, name=f"tiny-{qc}-{dc}")
        impatient = replace(base, classes=[replace(c, theta=th) for c, th in zip(base.classes, (4.0, 0.0, 25.0))])
        for cfg in (base,
                    impatient,
                    replace(base, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.8, 0.3, 0.55]),
                    replace(impatient, route_mode=W.ROUTE_RANDOM_SPLIT, p_solo=[0.8, 0.3, 0.55]),
                    replace(base, route_mode=W.ROUTE_WEIGHTED_SPLIT, p_solo=[0.8, 0.3, 0.55], w_solo=[0.5, 0.3, 0.2], w_mixed=[0.1, 0.6, 0.3]),
                    replace(impatient, route_mode=W.ROUTE_WEIGHTED_SPLIT, p_solo=[0.8, 0.3, 0.55], w_solo=[0.5, 0.0, 0.5], w_mixed=[0.1, 0.6, 0.3]),
                    replace(base, route_mode=W.ROUTE_IMMEDIATE),
                    replace(impatient, M=base.N, route_mode=W.ROUTE_IMMEDIATE)):
            sim, orc = run_both(B, oracle_mod, cfg, 1500, checkpoints=3)
            ss, os_ = sim.stats(), orc.stats()
            assert_stats_equal(ss, os_)
            assert ss["overflow"] == bool(os_["glob"][5])
