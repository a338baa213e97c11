"""CPU-only checks of the library's host side: it loads, exports every declared symbol, validates
configurations, and builds the same sampler tables as the oracle (independent code, same definition)."""
import ctypes
import os
import re
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_02987_amd import binding
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "gnr_sim.h")).read()
    names = set(re.findall(r"^(?:int|const char \*)\s*\*?(sim_[a-z_]+)\(", header, flags=re.M))
    assert {"sim_workspace_bytes", "sim_create", "sim_run", "sim_stats", "sim_snapshot", "sim_destroy",
            "sim_strerror", "sim_tallies", "sim_hist", "sim_digest", "sim_kernel_time", "sim_set_targets",
            "sim_patience_table", "sim_set_split"} <= names
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert B.lib().sim_strerror(-4).decode().startswith("a prefill queue")
    sizes = (ctypes.c_size_t * 4)()
    assert L.sim_abi_sizes(sizes) == 0
    assert list(sizes) == [ctypes.sizeof(B.SimClassC), ctypes.sizeof(B.SimConfigC), ctypes.sizeof(B.SimStatsC),
                           ctypes.sizeof(B.SimStateC)]


def test_tables_match_the_oracle(B, oracle_mod):
    for law, p0, p1 in [(0, 512.0, 0.0), (0, 64.0, 0.0), (0, 1.0, 0.0), (1, 256.0, 0.8), (1, 4096.0, 1.0),
                        (1, 8192.0, 1.0), (2, 600.0, 0.0)]:
        assert np.array_equal(B.sim_length_table(law, p0, p1), oracle_mod.length_table(law, p0, p1)), (law, p0, p1)
    for theta, dt in [(0.1, 0.010), (0.1, 10000000 * 1e-9), (5.0, 0.010), (40.0, 0.010), (2.0, 0.004), (1e-3, 0.010)]:
        assert np.array_equal(B.sim_patience_table(theta, dt), oracle_mod.patience_table(theta, dt)), (theta, dt)
    rng = np.random.default_rng(11)
    for _ in range(50):
        seed = int(rng.integers(0, 2**63)); c = [int(v) for v in rng.integers(0, 2**32, 4)]
        assert np.array_equal(B.sim_philox(seed, *c), oracle_mod.philox(seed, *c))
    for n in (1, 3, 5):
        cfg = W.config(n, N=64, replications=1)
        rows = max(cfg.mod_period, 1)
        arr, cth = B.sim_thresholds(cfg, rows)
        o = oracle_mod.Oracle(cfg)
        _, _, o_cth, o_arr = o.tables(0, rows=rows)
        assert np.array_equal(arr, o_arr)
        assert np.array_equal(cth[:cfg.K - 1], o_cth[:cfg.K - 1])


def test_invalid_configurations_are_rejected(B):
    good = W.config(1)
    assert B.sim_workspace_bytes(good, 16) > 0
    bad = [replace(good, K=9), replace(good, N=0), replace(good, N=20000), replace(good, B=129), replace(good, B=0),
           replace(good, C=0), replace(good, M=9), replace(good, M=-1), replace(good, dt=0.02), replace(good, c0=0.0),
           replace(good, queue_cap=0), replace(good, dbuf_cap=0), replace(good, gate_mode=7), replace(good, route_mode=4),
           replace(good, route_mode=1, p_solo=[0.5, 1.2]), replace(good, route_mode=1, p_solo=[-0.1, 0.5]),
           replace(good, x_star=[-0.1, 0.1]), replace(good, mod_amp=2.0)]
    heavy = W.config(1); heavy.classes[0].lam = 6.0
    theta = W.config(1); theta.classes[1].theta = -0.1
    for cfg in bad + [heavy, theta]:
        with pytest.raises(B.SimError) as e:
            B.sim_workspace_bytes(cfg, 16)
        assert e.value.code == -1
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(good, 0)
    # replications are bounded, so that no size of the workspace layout can wrap around 2^64: a ring of 2^30
    # entries for each of 2^31 - 1 replications would
    with pytest.raises(B.SimError) as e:
        B.sim_workspace_bytes(good, (1 << 20) + 1)
    assert e.value.code == -1
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(replace(good, queue_cap=1 << 30), (1 << 31) - 1)
    big = B.sim_workspace_bytes(replace(good, queue_cap=1 << 30, dbuf_cap=1 << 30), 1 << 20)   # the largest rings allowed
    assert (1 << 20) * (good.K * 4 + 8) * (1 << 30) < big < (1 << 55)


def test_patience_adds_deadline_rings_and_calendars_to_the_workspace(B):
    cfg = W.config(2)
    plain = B.sim_workspace_bytes(cfg, 4)
    cfg.classes[1].theta = 0.1          # longest patience 11783 steps -> calendars of 16384 entries
    longest = int(B.sim_patience_table(0.1, cfg.c0)[-1])
    assert 8192 < longest < 16384
    extra = B.sim_workspace_bytes(cfg, 4) - plain
    want = 4 * (cfg.K * cfg.queue_cap * 4 + cfg.dbuf_cap * 4 + 2 * cfg.K * 16384 * 4) + cfg.K * 65536 * 2
    assert want <= extra <= want + 8 * 256


def test_workspace_size_scales_with_replications(B):
    cfg = W.config(2)
    a, b = B.sim_workspace_bytes(cfg, 8), B.sim_workspace_bytes(cfg, 16)
    per_rep = cfg.N * (8 + 4 + 4 + 8 + 8 + 8 + cfg.B * 12) + cfg.K * cfg.queue_cap * 4 + cfg.dbuf_cap * 8
    assert b > a and (b - a) >= 8 * per_rep


def test_plan_of_config_1_matches_its_closed_forms():
    """Underloaded two-class instance: the fluid LP serves everything, so R* = sum_i lambda_i w_i = 460.8 token-prices
    per server and second, x*_i = lambda_i * (prefill service time), M = ceil(n sum x*); tau_mix = 29 ms,
    tau_solo = 16.4 ms, and the solo pool is the faster one per slot (gamma * tau >= (B-1)/B)."""
    from paper_2602_02987_amd import plan as P
    cfg = W.config(1)
    pl = P.solve_lp(cfg, [c.lam for c in cfg.classes])
    r = P.rates(cfg)
    assert pl.tau_mix == pytest.approx(0.029, rel=1e-12) and pl.tau_solo == pytest.approx(0.0164, rel=1e-12)
    assert pl.tau_mix / pl.tau_solo >= (cfg.B - 1) / cfg.B
    assert pl.value == pytest.approx(0.6 * (512 + 64) + 0.3 * (128 + 256), rel=1e-9)
    service = r["ECH"] * (cfg.c0 + cfg.c_dec * (cfg.B - 1)) + cfg.c_pre * r["EP"]
    assert np.allclose(pl.x, np.array([0.6, 0.3]) * service, rtol=1e-9)
    assert r["EP"] == pytest.approx([512.0, 128.0], rel=2e-5) and r["ED"] == pytest.approx([64.0, 256.0], rel=2e-5)
    # E ceil(P/C) of a geometric P: 1 / (1 - (1-p)^C)
    assert r["ECH"] == pytest.approx([1.0 / (1.0 - (1.0 - 1.0 / m) ** 256) for m in (512.0, 128.0)], rel=1e-4)
    assert cfg.M == pl.M == 1 and W.config(2).M == int(np.ceil(256 * pl.x.sum()))


def test_ablation_policies_are_switches_on_one_instance():
    """The five policies of the component ablation differ only in gate rule, decode rule and split; the instances
    stay within the ranges the paper states and are the same on every call."""
    from paper_2602_02987_amd import ablation as A
    a, b = A.instances(3, n=100), A.instances(3, n=100)
    for x, y in zip(a, b):
        assert x.M == y.M and x.x_star == y.x_star and [c.lam for c in x.classes] == [c.lam for c in y.classes]
    for cfg in a:
        assert 10.0 <= 1.0 / cfg.c0 <= 50.0 and 0.0 < cfg.dt <= cfg.c0 and cfg.c_pre >= 0.0
        assert 0.02 + 256e-5 <= cfg.c0 + cfg.c_pre * 256 <= 0.15 + 0.256 + 1e-12
        assert all(0.25 <= c.lam <= 0.5 and 200 <= c.in_p0 <= 3000 and 200 <= c.out_p0 <= 3000 for c in cfg.classes)
        assert sum(c.lam for c in cfg.classes) * cfg.dt <= 0.04 + 1e-12
        pol = A.policies(cfg)
        assert tuple(pol) == A.POLICIES
        want = {"GG-SP": (W.GATE_OCCUPANCY, W.ROUTE_SOLO_FIRST, cfg.M), "FG-SP": (W.GATE_FCFS, W.ROUTE_SOLO_FIRST, cfg.M),
                "GF-WSP": (W.GATE_OCCUPANCY, W.ROUTE_SOLO_FIRST, cfg.N), "GI-WSP": (W.GATE_OCCUPANCY, W.ROUTE_IMMEDIATE, cfg.N),
                "FI-WSP": (W.GATE_FCFS, W.ROUTE_IMMEDIATE, cfg.N)}
        for name, c in pol.items():
            assert (c.gate_mode, c.route_mode, c.M) == want[name]
            assert c.x_star == cfg.x_star and c.classes is cfg.classes and c.seed == cfg.seed


def test_on_chip_memory_bounds_the_number_of_servers():
    """The library refuses, on the host, a configuration whose per-server records do not fit a compute unit's
    on-chip memory, and says how much a configuration needs."""
    from paper_2602_02987_amd import binding as B
    need5, limit = B.sim_onchip_bytes(W.config(5))
    assert limit == 160 * 1024 and 140_000 < need5 < limit
    cfg = W.config(5, replications=1)
    small = replace(cfg, N=2000, M=400)
    assert B.sim_onchip_bytes(small)[0] < need5 - 80_000           # about 11.4 bytes per server
    ab = W.config(5, replications=1)
    for c in ab.classes:
        c.theta = 0.1
    assert B.sim_onchip_bytes(ab)[0] == need5 + 6 * 256 * 4         # the gate's table of waiting requests
    B.sim_workspace_bytes(replace(cfg, N=11000, M=2377), 1)
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(replace(cfg, N=12200, M=2377), 1)
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(replace(cfg, N=12289, M=0), 1)


def test_frozen_configurations_are_the_generated_ones():
    """The text copies under configs/ hold what workloads.config(n) generates here: seeded hyper-parameters and
    sizes exactly, rates and LP outputs to the solver's reproducibility; a run from the frozen copy of config 1 is
    the run from the generated one, bit for bit."""
    for n in range(1, 6):
        a, b = W.config(n), W.frozen_config(n)
        for f in ("name", "K", "N", "B", "C", "c0", "c_pre", "c_dec", "M", "gate_mode", "route_mode", "mod_amp",
                  "mod_period", "queue_cap", "dbuf_cap", "replications", "steps", "seed"):
            assert getattr(a, f) == getattr(b, f), (n, f)
        assert np.allclose(a.x_star, b.x_star, rtol=1e-9, atol=1e-15) and np.allclose(a.qp_star, b.qp_star, rtol=1e-9, atol=1e-15)
        for ca, cb in zip(a.classes, b.classes):
            for f in ("in_law", "in_p0", "in_p1", "out_law", "out_p0", "out_p1", "price_in", "price_out", "bundled", "priority", "theta"):
                assert getattr(ca, f) == getattr(cb, f), (n, f)
            assert ca.lam == pytest.approx(cb.lam, rel=1e-9)
    assert W.to_plain(W.from_plain(W.to_plain(W.config(4)))) == W.to_plain(W.config(4))


def test_frozen_config1_runs_like_the_generated_one(oracle_mod):
    a = oracle_mod.Oracle(W.config(1)); a.run(3000)
    b = oracle_mod.Oracle(W.frozen_config(1)); b.run(3000)
    for r in range(16):
        assert a.digest(r) == b.digest(r)


def test_every_configuration_is_in_the_regime_without_a_decode_buffer():
    """Prop. 1 (decode-buffer elimination) needs gamma * tau >= (B-1)/B, i.e. tau_mix / tau_solo >= (B-1)/B: true of
    the five configurations, the convergence instance and the ablation instances, whose plans all set q_d* = 0."""
    from paper_2602_02987_amd import ablation as A
    cfgs = [W.config(n) for n in range(1, 6)] + [W.convergence_instance(50)] + A.instances(4, n=50)
    for cfg in cfgs:
        assert cfg.notes["tau_mix"] / cfg.notes["tau_solo"] >= (cfg.B - 1) / cfg.B, cfg.name


def test_null_handles_and_null_outputs_are_refused():
    """Every entry point that takes a handle returns SIM_EINVAL for a null one (before it touches the GPU), the
    host helpers for null outputs; sim_strerror names every code."""
    from paper_2602_02987_amd import binding as B
    L = B.lib()
    null = None
    EINVAL = -1
    assert L.sim_run(null, ctypes.c_int64(1), 1, ctypes.c_uint64(1), null) == EINVAL
    assert L.sim_stats(null, null, null) == EINVAL
    assert L.sim_set_targets(null, null, null, null) == EINVAL
    assert L.sim_set_split(null, 0, null) == EINVAL
    assert L.sim_snapshot(null, 0, null, null) == EINVAL
    assert L.sim_tallies(null, 0, null, null) == EINVAL
    assert L.sim_hist(null, 0, 0, null, null) == EINVAL
    assert L.sim_digest(null, 0, null, null) == EINVAL
    assert L.sim_kernel_time(null, null, null, 0, null) == EINVAL
    assert L.sim_launch_shape(null, null, null) == EINVAL
    assert L.sim_destroy(null) == EINVAL
    assert L.sim_workspace_bytes(null, 1, null) == EINVAL
    assert L.sim_onchip_bytes(null, null, null) == EINVAL
    assert L.sim_length_table(0, ctypes.c_double(10.0), ctypes.c_double(0.0), null) == EINVAL
    assert L.sim_patience_table(ctypes.c_double(1.0), ctypes.c_double(0.01), null) == EINVAL
    assert L.sim_abi_sizes(null) == EINVAL
    L.sim_strerror.restype = ctypes.c_char_p
    names = {L.sim_strerror(c) for c in (0, -1, -2, -3, -4)}
    assert len(names) == 5 and L.sim_strerror(-99) not in names


def test_modulation_period_is_bounded_and_the_weighted_router_counts_its_tables():
    """A modulation period beyond what a run can reach is refused (not a host allocation of its size); the on-chip
    need reported for the weighted router includes its selection tables."""
    from dataclasses import replace
    from paper_2602_02987_amd import binding as B, workloads as W
    cfg = W.config(5, N=300, replications=1)
    assert B.sim_workspace_bytes(cfg, 1) > 0
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(replace(cfg, mod_period=(1 << 29) + 1), 1)
    with pytest.raises(B.SimError):
        B.sim_workspace_bytes(replace(cfg, mod_period=1 << 60), 1)
    base, _ = B.sim_onchip_bytes(cfg)
    ws = W.with_weighted_split(W.config(5, N=300, replications=1), lam_plan=[c.lam / 0.95 for c in cfg.classes])
    rr = W.with_random_split(W.config(5, N=300, replications=1), lam_plan=[c.lam / 0.95 for c in cfg.classes])
    need_ws, _ = B.sim_onchip_bytes(ws)
    need_rr, _ = B.sim_onchip_bytes(rr)
    assert need_rr == base + 4 * 8              # the group words of four chunks of completed prefills
    # (the figure is for the largest workgroup the library would launch, here 512 threads) the deadline rings'
    # candidate table (K x 256 words), 256 x (4 + 2 + 2) bytes of class selections, 8 words of per-class counts
    assert need_ws == need_rr + cfg.K * 256 * 4 + 256 * 8 + 8 * 4


def test_launch_shape_follows_the_replications():
    """A replication is one workgroup that lives for the whole launch: the library takes the largest workgroup that
    keeps the rounds of workgroups lowest (256 compute units, four waves a SIMD at most, LDS) and the roomy form of
    the kernel (two waves a SIMD) unless the dense one saves a round. Without a device 256 compute units are assumed."""
    from paper_2602_02987_amd import binding as B, workloads as W
    plan = lambda n, **over: B.sim_launch_plan(W.config(n, **over))
    assert plan(1)[0::2] == (64, 2)                        # 8 servers: one block, one wave
    assert plan(2)[0::2] == (128, 2)                       # 4 blocks, 1024 replications: a block a wave would not pay for the dense form
    assert plan(2, replications=2048)[0::2] == (128, 4)    # eight two-wave workgroups per compute unit
    assert plan(2, replications=256)[0::2] == (256, 2)     # one per compute unit: room for the form with more registers
    assert plan(3)[0::2] == (128, 4) and plan(3)[1] == 20112
    assert plan(3, replications=1024)[0::2] == (256, 4)
    assert plan(3, replications=512)[0::2] == (512, 4)
    assert plan(3, replications=256)[0::2] == (512, 2)
    assert plan(4)[0::2] == (256, 4)
    assert plan(4, replications=2048)[0::2] == (256, 4)    # the LDS holds four per compute unit: two rounds either way
    assert plan(4, replications=256)[0::2] == (1024, 4)    # a compute unit each: sixteen waves, two blocks a wave
    assert plan(4, replications=257)[0::2] == (512, 4)
    assert plan(5) == (1024, 148368, 4)
    for n in (1, 2, 3, 4, 5):                              # eight of the smallest workgroups share a compute unit
        t, lds, w = plan(n)
        assert lds <= 160 * 1024 and t in (64, 128, 256, 512, 1024) and w in (2, 4)
    # what a handle is created with is what the plan says (no device: compared through the on-chip need)
    assert B.sim_onchip_bytes(W.config(3))[0] == B.sim_launch_plan(W.config(3), 1)[1]
