"""GPU test of sim_create_static, the entry point for callers that cannot allocate device memory: a handle whose
workspace is the library's static device array must behave exactly like one on a caller-allocated workspace.
Two calls in a row, the second with a smaller configuration (the array keeps what the first one left); compared
bit by bit: state, tallies, histograms, digests; derived figures within 1e-12."""
import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_stats_equal
from test_gpu_parity import B  # noqa: F401  (fixture)
from test_oracle_dynamics import _heavy

pytestmark = pytest.mark.gpu


def _same(a, b, cfg):
    for r in range(cfg.replications):
        sa, sb = a.snapshot(r), b.snapshot(r)
        for name in sa:
            if isinstance(sa[name], list):
                assert len(sa[name]) == len(sb[name]) and all(np.array_equal(x, y) for x, y in zip(sa[name], sb[name])), (r, name)
            else:
                assert np.array_equal(sa[name], sb[name]), (r, name)
        ta, ga = a.tallies(r); tb, gb = b.tallies(r)
        assert np.array_equal(ta, tb) and np.array_equal(ga, gb), r
        for which in range(3):
            assert np.array_equal(a.hist(r, which), b.hist(r, which)), (r, which)
        assert a.digest(r) == b.digest(r), r
    assert_stats_equal(a.stats(), b.stats(), rel=1e-12)


def test_static_workspace_matches_a_caller_workspace(B):
    first = W.config(3, N=300, replications=4)          # about 3 MiB of state: several ballot words, lognormal lengths
    second = _heavy()                                   # smaller: 12 servers, rings that overflow, the decode buffer in use
    assert B.sim_workspace_bytes(second, second.replications) < B.sim_workspace_bytes(first, first.replications)
    for cfg, steps in ((first, 1500), (second, 2500)):
        ref = B.Sim(cfg)
        sta = B.Sim(cfg, static_workspace=True)
        assert sta.workspace is None
        for n in (steps // 3, steps - steps // 3):       # in two runs: the second resumes from the state the array holds
            ref.run(n)
            sta.run(n)
        _same(sta, ref, cfg)
        sta.run(200, seed=cfg.seed + 1)                 # another seed restarts from the empty system
        ref.run(200, seed=cfg.seed + 1)
        _same(sta, ref, cfg)
        sta.close()
        ref.close()
    with pytest.raises(B.SimError) as err:              # config 2 needs 206 MiB: beyond the static array
        B.Sim(W.config(2), static_workspace=True)
    assert err.value.code == -2 and "static workspace" in str(err.value)
