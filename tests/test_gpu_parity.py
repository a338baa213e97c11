"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs, through the C ABI.
Integer state, tallies, histograms and digests are compared bit-exactly; derived fp64 figures
(rates, revenue, latency means) within 1e-12 relative."""
import os
from dataclasses import replace

import numpy as np
import pytest

from paper_2602_02987_amd import workloads as W
from parity import assert_replication_equal, assert_stats_equal
from test_oracle_dynamics import _heavy, _lp_instance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2602_02987_amd import binding
    binding.lib()
    return binding


def run_both(B, oracle_mod, cfg, steps, reps=None, seed=None, oracle_reps=None, checkpoints=1):
    reps = cfg.replications if reps is None else reps
    sim = B.Sim(cfg, max_replications=reps)
    orc = oracle_mod.Oracle(cfg, max_reps=reps)
    if oracle_reps is not None:
        orc.select(oracle_reps)
    done = 0
    for c in range(checkpoints):
        n = (steps * (c + 1)) // checkpoints - done
        sim.run(n, reps, seed)
        orc.run(n, reps, seed)
        done += n
        for r in (range(reps) if oracle_reps is None else oracle_reps):
            assert_replication_equal(sim, orc, r, what=f"{cfg.name} after {done} steps")
    return sim, orc


def test_config1_full(B, oracle_mod):
    cfg = W.config(1)
    sim, orc = run_both(B, oracle_mod, cfg, cfg.steps, checkpoints=4)
    assert_stats_equal(sim.stats(), orc.stats())
    assert not sim.stats()["overflow"]


@pytest.mark.parametrize("gate", [W.GATE_OCCUPANCY, W.GATE_PRIORITY, W.GATE_FCFS])
def test_heavy_small_instances(B, oracle_mod, gate):
    """Full slots, decode buffer in use, ring overflow, empty groups, B = 1."""
    for cfg in (_heavy(gate), _heavy(gate, M=0), _heavy(gate, M=12), _heavy(gate, B=1, M=6),
                _heavy(gate, name="heavy-prefill", M=1, queue_cap=8), _heavy(gate, N=1, M=1, B=3),
                _heavy(gate, N=1, M=0, B=3)):
        sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=5)
        ss, os_ = sim.stats(), orc.stats()
        assert_stats_equal(ss, os_)
        assert ss["overflow"] == bool(os_["glob"][5])


def test_several_tiles_and_ragged_tail(B, oracle_mod):
    """N spans several 64-server ballot words and several servers per thread, with a ragged tail."""
    for N, M, reps, steps in ((100, 30, 3, 1500), (1500, 400, 2, 800), (2500, 700, 1, 500)):
        cfg = W.config(3, N=N, replications=reps)
        cfg = replace(cfg, M=M)
        run_both(B, oracle_mod, cfg, steps, checkpoints=2)


def test_binding_capacity_instance(B, oracle_mod):
    cfg = _lp_instance(64, 2, 6000, (1024, 3072), (400, 160))
    sim, orc = run_both(B, oracle_mod, cfg, 6000, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())


def test_modulated_arrivals_and_many_classes(B, oracle_mod):
    cfg = W.config(5, N=300, replications=2, mod_period=700)
    run_both(B, oracle_mod, cfg, 2000, checkpoints=2)
    cfg = W.config(4, N=256, replications=2)
    sim, orc = run_both(B, oracle_mod, cfg, 1500)
    assert_stats_equal(sim.stats(), orc.stats())


def test_two_handles_on_two_streams_at_once(B, oracle_mod):
    """Two handles of different configurations (two variants of the step kernel) advance in turns, each on a stream
    of its own with no synchronisation in between, so that their launches overlap on the device; every handle has
    its own workspace and the library keeps no state between them: both match the oracle."""
    import torch
    cfgs = [W.config(3, N=300, replications=3), replace(_heavy(W.GATE_OCCUPANCY), name="heavy-beside")]
    cfgs[0].classes[1].theta = 0.05
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sims = [B.Sim(c, max_replications=c.replications) for c in cfgs]
    for _ in range(6):
        for sim, st in zip(sims, streams):
            with torch.cuda.stream(st):
                sim.run(250)
    for sim, st, cfg in zip(sims, streams, cfgs):
        orc = oracle_mod.Oracle(cfg, max_reps=cfg.replications)
        orc.run(1500, cfg.replications, None)
        with torch.cuda.stream(st):
            for r in range(cfg.replications):
                assert_replication_equal(sim, orc, r, what=cfg.name + " beside another handle")
            assert_stats_equal(sim.stats(), orc.stats())


def test_resume_and_restart(B, oracle_mod):
    cfg = _heavy()
    a = B.Sim(cfg); a.run(900)
    b = B.Sim(cfg); b.run(1); b.run(499); b.run(400)
    for r in range(cfg.replications):
        assert a.digest(r) == b.digest(r)
        assert np.array_equal(a.tallies(r)[0], b.tallies(r)[0])
    b.run(300, seed=77)                       # another seed restarts from the empty system
    orc = oracle_mod.Oracle(cfg); orc.run(300, seed=77)
    for r in range(cfg.replications):
        assert_replication_equal(b, orc, r, what="restart")


def test_full_size_configs_on_sampled_replications(B, oracle_mod):
    """Configs 2-5 at their full N and replication count, in the launch shape the benchmark times,
    for a prefix of steps; the oracle recomputes a sample of replications (first, second, last)."""
    for n, steps in ((2, 3000), (3, 1200), (4, 700), (5, 300)):
        cfg = W.config(n)
        sample = [0, 1, cfg.replications - 1]
        run_both(B, oracle_mod, cfg, steps, oracle_reps=sample)


def test_roomy_and_dense_forms_of_the_smaller_size_classes(B, oracle_mod):
    """The library compiles its one- to eight-wave workgroups twice, for two and for four waves per SIMD, and takes
    the denser form when the launch then needs fewer rounds of workgroups. Both forms of both classes against the
    oracle on sampled replications: N = 3000 runs sixteen waves while every replication has a compute unit of its own
    and 512 threads in the dense form beyond that (two workgroups per compute unit); N = 1500 and N = 600 run 512
    threads roomy with few replications; N = 600 with 1500 replications runs 128 threads dense (six workgroups per
    compute unit)."""
    for N, M, reps, steps in ((3000, 800, 40, 400), (3000, 800, 300, 400), (1500, 400, 40, 500), (600, 150, 64, 600), (600, 150, 1500, 600)):
        cfg = replace(W.config(3, N=N, replications=reps), M=M)
        sim, _ = run_both(B, oracle_mod, cfg, steps, oracle_reps=[0, reps // 2, reps - 1], checkpoints=2)
        threads, lds, per_simd = B.sim_launch_plan(cfg)
        assert sim.launch_shape() == (threads, lds)
        assert (threads, per_simd) == {(3000, 40): (1024, 4), (3000, 300): (512, 4), (1500, 40): (512, 2), (600, 64): (512, 2),
                                       (600, 1500): (128, 4)}[(N, reps)]


def test_results_do_not_depend_on_the_launch_shape(B):
    """The same replications under handles created for few and for many replications (other workgroup sizes and
    kernel forms): identical digests, tallies and histograms."""
    cfg = replace(W.config(3, N=600, replications=8), M=150)
    shapes, outs = set(), []
    for max_reps in (8, 600, 1500, 2400):
        sim = B.Sim(cfg, max_replications=max_reps)
        sim.run(700, 8)
        shapes.add(sim.launch_shape())
        outs.append(([sim.digest(r) for r in range(8)], [sim.tallies(r)[0].copy() for r in range(8)], [np.concatenate([sim.hist(r, w).ravel() for w in range(3)]) for r in range(8)]))
        sim.close()
    assert len(shapes) >= 3
    for o in outs[1:]:
        assert o[0] == outs[0][0]
        assert all(np.array_equal(a, b) for a, b in zip(o[1], outs[0][1]))
        assert all(np.array_equal(a, b) for a, b in zip(o[2], outs[0][2]))


def test_config5_full_size_in_the_state_the_benchmark_times(B, oracle_mod):
    """Config 5 unmodified (N = 10000, 256 replications, modulation period 100000 steps) advanced in 1000-step
    runs as the benchmark issues them, through the peak of the arrival rate (step 25000) into the state the
    benchmark times: it starts its timed region after 31000 steps and ends it, with its default flags, at 36000.
    The oracle follows one replication all the way (about a minute on one host core); state, tallies, histograms
    and digest are compared at 10000, 25000, 31000 and 36000 steps."""
    cfg = W.config(5)
    assert (cfg.N, cfg.replications, cfg.mod_period) == (10000, 256, 100000)
    rep = 137
    sim = B.Sim(cfg)
    orc = oracle_mod.Oracle(cfg, max_reps=cfg.replications)
    orc.select([rep])
    done = 0
    for stop in (10000, 25000, 31000, 36000):
        while done < stop:
            sim.run(1000)
            done += 1000
        orc.run(stop - int(orc.steps_done()), cfg.replications, cfg.seed)
        assert_replication_equal(sim, orc, rep, what=f"config 5 after {stop} steps")
    sn = sim.snapshot(rep)
    assert sn["Qp"].sum() > 1000 and sn["n_dec"][cfg.M:].mean() > cfg.B - 2      # the loaded state: long queues, solo servers full
    assert not sim.stats()["overflow"]


def _limits_class(**kw):
    base = dict(lam=1.0, in_law=W.LAW_CONST, in_p0=64.0, out_law=W.LAW_GEOMETRIC, out_p0=4.0)
    base.update(kw)
    return W.SimClass(**base)


def _limits_cfg(name, classes, N, M, B, steps, x_star=None, **kw):
    K = len(classes)
    return W.SimConfig(name=name, K=K, N=N, B=B, C=256, c0=0.010, c_pre=0.00005, c_dec=0.0002, classes=classes, M=M,
                       x_star=x_star or [0.3 / K] * K, qp_star=[0.0] * K, queue_cap=kw.pop("queue_cap", 4096),
                       dbuf_cap=kw.pop("dbuf_cap", 4096), replications=kw.pop("replications", 2), steps=steps,
                       seed=kw.pop("seed", 5), **kw)


def test_rows_with_more_than_64_decodes(B, oracle_mod):
    """B = 128 and an overloaded decode side: slot rows fill past 64 and up to the cap, so both halves of a row
    are scanned, decodes leave from either half, and the last slot of a full row is reused."""
    cls = [_limits_class(lam=2.4, in_p0=200.0, out_p0=3000.0), _limits_class(lam=1.6, in_p0=90.0, out_p0=1500.0)]
    cfg = _limits_cfg("wide-rows", cls, N=48, M=16, B=128, steps=5000)
    sim, orc = run_both(B, oracle_mod, cfg, 5000, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())
    loads = orc.slots(0)["n_dec"]
    assert loads.max() == 128 and (loads > 64).sum() > 20


def test_more_admissions_and_placements_than_one_pass_stages(B, oracle_mod):
    """Several hundred admissions and placements in one step: more than one gate pass decides (256) and more
    requests than a routing pass stages on chip (256)."""
    cls = [_limits_class(lam=2.5), _limits_class(lam=2.0, in_p0=40.0, out_p0=6.0)]
    cfg = _limits_cfg("bursts", cls, N=8192, M=5000, B=8, steps=40, replications=1)
    sim, orc = run_both(B, oracle_mod, cfg, 40, checkpoints=2)
    t, _ = orc.tallies(0)
    from paper_2602_02987_amd.binding import TALLY
    ti = {n: i for i, n in enumerate(TALLY)}
    assert t[:, ti["U_P"]].sum() / 40 > 300 and (t[:, ti["U_DM"]].sum() + t[:, ti["U_DS"]].sum()) / 40 > 280


def test_placements_on_mixed_servers_wait_for_the_last_gate_pass(B, oracle_mod):
    """More idle prefill slots than one gate pass serves (256) while the solo group is full, so that jobs go to
    mixed-group servers in the same steps: such a placement counts as mixed or solo decode by what the whole
    gate of the step admitted, not by what its first pass did."""
    cls = [_limits_class(lam=2.5, out_p0=300.0), _limits_class(lam=2.0, in_p0=40.0, out_p0=500.0)]
    cfg = _limits_cfg("late-passes", cls, N=8192, M=300, B=2, steps=300, replications=1, dbuf_cap=2048, queue_cap=8192)
    sim, orc = run_both(B, oracle_mod, cfg, 300, checkpoints=3)
    t, _ = orc.tallies(0)
    from paper_2602_02987_amd.binding import TALLY
    ti = {n: i for i, n in enumerate(TALLY)}
    assert t[:, ti["U_DM"]].sum() > 100 and t[:, ti["U_DS"]].sum() > 10000


def test_jobs_spread_over_many_load_levels(B, oracle_mod):
    """Three solo servers with unequal loads take several jobs per step: more load levels than one routing
    pass fills (4), then the mixed group once the solo group is full."""
    cls = [_limits_class(lam=1.0, out_p0=2.0)]
    cfg = _limits_cfg("levels", cls, N=1000, M=997, B=128, steps=1500, x_star=[0.5])
    sim, orc = run_both(B, oracle_mod, cfg, 1500, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())
    cls = [_limits_class(lam=4.5, out_p0=40.0)]   # the solo group saturates: the rest goes to the mixed group
    cfg = _limits_cfg("levels-full", cls, N=200, M=197, B=128, steps=1500, x_star=[0.5])
    run_both(B, oracle_mod, cfg, 1500, checkpoints=2)


def test_long_runs_of_identical_iterations(B, oracle_mod):
    """A lone decode of thousands of tokens: its server repeats the same iteration far more often than the
    untallied-iteration counter holds (254), and launches end in the middle of such runs."""
    cls = [_limits_class(lam=0.25, in_p0=100.0, out_law=W.LAW_CONST, out_p0=2000.0)]
    cfg = _limits_cfg("runs", cls, N=8, M=2, B=4, steps=7000, x_star=[0.1])
    sim, orc = run_both(B, oracle_mod, cfg, 7000, checkpoints=3)
    assert_stats_equal(sim.stats(), orc.stats())


def test_config5_width_through_a_load_peak(B, oracle_mod):
    """Config 5 at its full N (157 blocks of 64 servers, 16 waves) with a short modulation period, so that the
    load peak falls inside the run: every solo server then holds more than 64 decodes."""
    cfg = W.config(5, replications=2, mod_period=20000)
    sim, orc = run_both(B, oracle_mod, cfg, 10000, oracle_reps=[0], checkpoints=2)
    assert (orc.slots(0)["n_dec"] > 64).sum() > 5000


def test_targets_moved_between_runs(B, oracle_mod):
    """sim_set_targets between two runs: the gate follows the new targets from the next step on."""
    for cfg, new_x, new_q in ((_heavy(), [0.02, 0.4, 0.3], [0.0, 2.0, 0.0]),
                              (_heavy(name="heavy-prefill", M=1, queue_cap=8), [0.02, 0.4, 0.3], [0.0, 2.0, 0.0]),
                              (W.config(3, N=300, replications=2), [0.3, 0.02, 0.05, 0.1], [0.0, 0.0, 0.5, 0.0])):
        sim = B.Sim(cfg); orc = oracle_mod.Oracle(cfg)
        sim.run(700); orc.run(700)
        sim.set_targets(new_x, new_q); orc.set_targets(new_x, new_q)
        sim.run(900); orc.run(900)
        for r in range(cfg.replications):
            assert_replication_equal(sim, orc, r, what=f"{cfg.name} after new targets")
        sim.set_targets(cfg.x_star, cfg.qp_star); orc.set_targets(cfg.x_star, cfg.qp_star)
        sim.run(400); orc.run(400)
        for r in range(cfg.replications):
            assert_replication_equal(sim, orc, r, what=f"{cfg.name} after the old targets again")
    with pytest.raises(B.SimError):
        sim.set_targets([-1.0] * cfg.K, [0.0] * cfg.K)


def test_largest_class_count_and_batch_together(B, oracle_mod):
    """K = 8 and B = 128 at once (widest class tables, widest time-between-tokens window, full slot rows)."""
    rng = np.random.default_rng(3)
    cls = [_limits_class(lam=0.55, in_p0=float(rng.integers(60, 900)), out_p0=float(rng.integers(200, 2500)))
           for _ in range(8)]
    cfg = _limits_cfg("k8-b128", cls, N=600, M=120, B=128, steps=2500, replications=2)
    sim, orc = run_both(B, oracle_mod, cfg, 2500, checkpoints=2)
    assert_stats_equal(sim.stats(), orc.stats())
    assert orc.slots(0)["n_dec"].max() > 64


def test_degenerate_runs(B, oracle_mod):
    """No arrivals at all; zero steps; one replication out of several allocated; one server."""
    cfg = W.config(1, replications=3)
    for c in cfg.classes:
        c.lam = 0.0
    sim, orc = run_both(B, oracle_mod, cfg, 500)
    assert sim.stats()["tally"].sum() == 0
    cfg = W.config(1, replications=4)
    sim = B.Sim(cfg, max_replications=4); orc = oracle_mod.Oracle(cfg, max_reps=4)
    sim.run(0, 1); orc.run(0, 1)              # nothing simulated yet: the empty system
    assert_replication_equal(sim, orc, 0, what="zero steps")
    sim.run(700, 1); orc.run(700, 1)          # one replication of the four the workspace holds
    assert_replication_equal(sim, orc, 0, what="one of four")
    with pytest.raises(B.SimError):
        sim.run(10, 5)                        # more than the workspace was sized for
    with pytest.raises(B.SimError):
        sim.run(2 ** 29 - 700, 1)             # arrival stamps are kept in 29 bits: a run ends before step 2^29
    sim.run(1, 1); orc.run(1, 1)              # the refused call changed nothing
    assert_replication_equal(sim, orc, 0, what="after a refused run")
    cfg = _heavy(N=1, M=0, B=1)
    run_both(B, oracle_mod, cfg, 800)


def test_maximum_sizes(B, oracle_mod):
    """The documented limits: the most servers a replication of this shape may have (with 1500 mixed ones: found here
    on the host as the largest N whose on-chip records fit a compute unit's LDS, more than 11500) and one more
    refused, the largest chunk (8191 tokens) with the longest prompts and outputs the tables hold (32768 tokens)."""
    from paper_2602_02987_amd.binding import TALLY
    ti = {n: i for i, n in enumerate(TALLY)}
    cls = [_limits_class(lam=2.0, in_p0=300.0, out_p0=40.0), _limits_class(lam=1.5, in_p0=90.0, out_p0=15.0)]
    shape = lambda n: _limits_cfg("most-servers", cls, N=n, M=1500, B=8, steps=120, replications=1, queue_cap=8192)  # noqa: E731
    lo, hi = 8000, 12288                       # fits / does not fit
    while hi - lo > 1:
        mid = (lo + hi) // 2
        need, limit = B.sim_onchip_bytes(shape(mid))
        lo, hi = (mid, hi) if need <= limit else (lo, mid)
    n_max = lo
    assert n_max > 11500
    cfg = shape(n_max)
    need, limit = B.sim_onchip_bytes(cfg)
    assert limit - 64 < need <= limit
    sim, orc = run_both(B, oracle_mod, cfg, 120, checkpoints=2)
    assert orc.tallies(0)[0][:, ti["S_DS"]].sum() > 1000
    for n_bad in (n_max + 1, 12289):
        with pytest.raises(B.SimError):
            B.Sim(_limits_cfg("too-many-servers", cls, N=n_bad, M=1500, B=8, steps=1))
    # every prompt 32768 tokens long, prefilled in chunks of 8191 + 8191 + 8191 + 8191 + 4; outputs of the same length
    cls = [_limits_class(lam=0.8, in_law=W.LAW_CONST, in_p0=32768.0, out_law=W.LAW_CONST, out_p0=32768.0)]
    cfg = _limits_cfg("longest-requests", cls, N=6, M=2, B=4, steps=70000, x_star=[0.3], replications=1)
    cfg.C = 8191
    cfg.c_pre = 1e-7
    sim, orc = run_both(B, oracle_mod, cfg, 70000, checkpoints=2)
    t = orc.tallies(0)[0]
    assert t[0, ti["S_P"]] > 20 and t[0, ti["TOKP_PRE"]] == 32768 * t[0, ti["S_P"]]
    assert t[0, ti["S_DS"]] + t[0, ti["S_DM"]] > 5
    with pytest.raises(B.SimError):
        bad = _limits_cfg("chunk-too-large", cls, N=6, M=2, B=4, steps=1, x_star=[0.3])
        bad.C = 8192
        B.Sim(bad)


def test_configs_2_to_4_at_their_full_length(B, oracle_mod):
    """Configs 2, 3 and 4 exactly as specified — every replication, all 100000 steps — on the GPU; the oracle
    recomputes sampled replications over the whole length (launch boundaries, clock wrap-arounds and ring
    wrap-arounds of a long run included)."""
    for n, sample in ((2, [0, 511, 1023]), (3, [2047]), (4, [512])):
        cfg = W.config(n)
        assert cfg.steps == 100_000
        sim, orc = run_both(B, oracle_mod, cfg, cfg.steps, oracle_reps=sample)
        assert not sim.stats()["overflow"]


@pytest.mark.skipif(os.environ.get("GNR_LONG_TESTS") != "1",
                    reason="about 150 s of oracle time on one host core; set GNR_LONG_TESTS=1 to run")
def test_config5_over_a_whole_modulation_period(B, oracle_mod):
    """Config 5 at its full size over 100000 steps (one period of the arrival modulation: the empty system, the
    load peak with queues of thousands and every solo server full, and the trough); the oracle follows the last
    replication."""
    cfg = W.config(5)
    run_both(B, oracle_mod, cfg, 100_000, oracle_reps=[cfg.replications - 1], checkpoints=10)
