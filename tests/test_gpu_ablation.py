"""The paper's component ablation (EC "Additional Ablation Studies on Synthetic Workloads") on the HIP library:
five policies on seeded instances at n = 500. The paper reports a bar chart only, so this checks what the method
itself fixes: the full policy earns the fluid optimum R* on every instance with little spread; dropping the gate
(FCFS admission) or the split (every server mixed, least-loaded routing) loses revenue on overloaded instances;
no policy beats R* by more than the plan's own rounding of chunk lengths allows. One policy set is also compared
with the oracle bit by bit at a small size."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import ablation as A
from test_gpu_parity import B, run_both  # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


def test_policies_against_the_fluid_optimum(B):
    res = A.study(B.Sim, count=4, warm_time=500.0, measure_time=1000.0)
    col = {p: res[:, i] for i, p in enumerate(A.POLICIES)}
    assert res.shape == (4, 5) and np.all(res > 0.2) and np.all(res < 1.01), res
    assert np.all(col["GG-SP"] > 0.98) and col["GG-SP"].std() < 0.01, col["GG-SP"]
    assert col["FG-SP"].mean() < 0.95 and col["GF-WSP"].mean() < 0.85 and col["FI-WSP"].mean() < 0.97, res.mean(axis=0)
    assert np.all(col["GG-SP"] >= col["FG-SP"]) and np.all(col["GG-SP"] >= col["GF-WSP"]), res
    assert np.all(col["GI-WSP"] >= col["FI-WSP"]), res            # the gate helps with either decode rule


def test_policy_set_bit_by_bit(B, oracle_mod):
    cfg = A.instances(2, n=40, seeds=2)[1]
    for name, c in A.policies(cfg).items():
        run_both(B, oracle_mod, replace(c, name=f"{cfg.name}-{name}"), 6000, checkpoints=2)
