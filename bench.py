#!/usr/bin/env python3
"""Benchmark of the simulator's hot path on one MI355X.

A bench "step" is one sim_run of `--sim-steps` simulation steps over every replication of the
workload (config 5 at its full size: K=6, N=10000 servers, 256 replications, B=128, sinusoidal
arrivals), state resident in HBM. Before timing, the system is brought away from the empty state
by `--preload` untimed simulation steps. Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


# HBM traffic of one step-kernel launch of the default run, from hardware counters (two rocprofv3 --pmc runs:
# FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a device copy of known size), and the
# occupancy rocprofv3 derives for it. These are STORED figures, not taken in this run: they hold for the kernel
# sources whose hash is given (compared with the current sources; on a mismatch the figures read null) and for the
# state named in `state`. The line says so in `roofline.traffic_source` / `roofline.occupancy.source`.
TRAFFIC = {"sources_sha256": "3abd042e65bae0a98324464102efade702e73527a7039320e997bf28af340194",
           "bytes_per_launch": 383860798110, "occupancy_percent": 49.107249,
           "state": "config 5 after 30000 untimed steps, mean of 2 launches of 1000 steps",
           "profile": "profiles/gnr_step_kernel_cfg5_hbm_traffic.md"}


def algorithmic_bytes(t0, g0, t1, g1, slots):
    """Bytes the method moves for the work done between two tally read-outs.

    Per server-step slot: 8 B to read the server's clock (is it due?); for a due server 24 B for the
    rest of its record plus one 4-byte finish word per occupied decode slot, and 32 B to write the
    record back; about 32 B of request words and ring entries per admission, placement and completion.
    With f = executed iterations per slot, n = occupied decode slots per executed iteration and
    e = events per slot this is 8 + f*(24 + 4n) + f*32 + e*32 bytes per slot.

    The second figure is what this kernel has to move given that server clocks, iteration counters and
    decode counts stay in LDS for a whole launch: the finish words of the due servers, the prefill
    word of iterations that carry a chunk, and the event traffic.
    """
    from paper_2602_02987_amd.binding import GLOBAL, TALLY
    ti = {n: i for i, n in enumerate(TALLY)}
    gi = {n: i for i, n in enumerate(GLOBAL)}
    d = (t1.astype("float64") - t0.astype("float64")).sum(axis=0)
    it_mix = float(g1[gi["ITERS_MIX"]]) - float(g0[gi["ITERS_MIX"]])
    iters = it_mix + float(g1[gi["ITERS_SOLO"]]) - float(g0[gi["ITERS_SOLO"]])
    scanned = d[ti["TOK_EMIT"]]   # every occupied decode slot of an executed iteration emits one token
    events = d[ti["U_P"]] + d[ti["S_P"]] + d[ti["U_DM"]] + d[ti["U_DS"]] + d[ti["S_DM"]] + d[ti["S_DS"]]
    total = 8.0 * slots + (24.0 + 32.0) * iters + 4.0 * scanned + 32.0 * events
    on_chip_records = 4.0 * scanned + 16.0 * it_mix + 32.0 * events
    return total, dict(due_fraction=iters / slots, decodes_per_iteration=scanned / max(iters, 1.0),
                       events_per_slot=events / slots, bytes_per_slot=total / slots,
                       bytes_per_slot_with_records_in_lds=on_chip_records / slots)


def sources_hash():
    """sha256 over the library's kernel and host sources, in a fixed order, and the compiler flags they are built with."""
    import hashlib
    from paper_2602_02987_amd import build as _b
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2602_02987_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as fh:
            h.update(name.encode() + b"\0" + fh.read())
    h.update(" ".join(_b.FLAGS).encode())
    return h.hexdigest()


def measured(key):
    """A stored figure of the hardware-counter runs, or None when the sources are no longer the ones they ran on."""
    return TRAFFIC[key] if TRAFFIC["sources_sha256"] == sources_hash() else None


def occupancy(binding, cfg, sim, replications, measured_percent):
    """Waves per SIMD of the launch (256 compute units of 4 SIMDs, 160 KB of LDS). The library says which form of the
    step kernel it launches: the one compiled for four waves per SIMD (128 registers a lane) or, for workgroups of up
    to 512 threads that all find a place at once at that density, the one for two (up to 256 registers)."""
    threads, lds = sim.launch_shape()
    _, _, per_simd = binding.sim_launch_plan(cfg, replications)
    waves = threads // 64
    per_cu = min(160 * 1024 // max(lds, 1), max(4 * per_simd // waves, 1), -(-replications // 256))
    return {"threads_per_workgroup": threads, "lds_bytes_per_workgroup": lds, "workgroups_per_cu": per_cu,
            "waves_per_simd": waves * per_cu / 4.0, "waves_per_simd_the_registers_allow": per_simd,
            "simd_capacity": 8, "measured_percent": measured_percent,
            "source": "launch shape and kernel form from the library; measured_percent " +
                      (f"stored: rocprofv3 counters, {TRAFFIC['state']}, {TRAFFIC['profile']}" if measured_percent is not None
                       else "not available for these sources (null)")}


def measured_traffic():
    return measured("bytes_per_launch")


def policy_variant(W, cfg, theta, split, immediate, weighted=False):
    """The configuration with the optional policy switches of the command line applied."""
    if split:
        cfg = W.with_random_split(cfg, lam_plan=[c.lam / 0.95 for c in cfg.classes])
    if weighted:
        cfg = W.with_weighted_split(cfg, lam_plan=[c.lam / 0.95 for c in cfg.classes])
    if immediate:
        cfg.route_mode = W.ROUTE_IMMEDIATE   # as in the paper's ablation: no static partition, every server may prefill
        cfg.M = cfg.N
    if theta:
        for c in cfg.classes:
            c.theta = theta
    return cfg


def _oracle_worker(args):
    n, N, rep, steps, theta, split, immediate, weighted = args
    sys.path.insert(0, ROOT)
    from oracle import binding as ob
    from paper_2602_02987_amd import workloads as W
    cfg = policy_variant(W, W.config(n, N=N), theta, split, immediate, weighted)
    o = ob.Oracle(cfg, max_reps=cfg.replications)
    o.select([rep])
    t = time.perf_counter()
    o.run(steps, cfg.replications, cfg.seed)
    return time.perf_counter() - t


def cpu_baseline(n, N, steps, theta=0.0, split=False, immediate=False, weighted=False):
    """The oracle as it stands, one replication per host process, on a bounded sample."""
    import multiprocessing as mp
    from oracle import binding as ob
    ob.build()
    cores = min(16, os.cpu_count() or 1)
    t = time.perf_counter()
    with mp.get_context("spawn").Pool(cores) as pool:
        pool.map(_oracle_worker, [(n, N, r, steps, theta, split, immediate, weighted) for r in range(cores)])
    wall = time.perf_counter() - t
    return dict(value=cores * N * steps / wall, unit="server-steps/s", cores=cores, kind="oracle",
                sample=f"replications 0..{cores - 1} of the workload, first {steps} steps from the empty system, "
                       f"one process per replication, wall {wall:.1f} s incl. table build")


def gpu_on_the_baseline_sample(binding, torch, cfg, steps):
    """The library on the CPU baseline's sample (the first `steps` steps from the empty system; all replications,
    since a launch runs them side by side), so that the two figures can be compared like for like."""
    sim = binding.Sim(cfg)
    sim.run(0)                       # the reset kernel
    torch.cuda.synchronize()
    t = time.perf_counter()
    sim.run(steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t
    sim.close()
    return dict(value=cfg.N * cfg.replications * steps / wall, unit="server-steps/s",
                sample=f"all {cfg.replications} replications, first {steps} steps from the empty system, wall {wall * 1e3:.0f} ms")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5, help="timed bench steps (sim_run calls)")
    ap.add_argument("--warmup", type=int, default=1, help="untimed bench steps")
    ap.add_argument("--sim-steps", type=int, default=1000, help="simulation steps per bench step")
    ap.add_argument("--preload", type=int, default=30000, help="untimed simulation steps before anything else")
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--servers", type=int, default=0, help="override N (0 = the configuration's own)")
    ap.add_argument("--replications", type=int, default=0)
    ap.add_argument("--theta", type=float, default=0.0,
                    help="patience rate given to every class (abandonment; 0 = the configuration's own, none)")
    ap.add_argument("--random-split", action="store_true",
                    help="route decodes with the randomized router, solo probabilities from the configuration's plan")
    ap.add_argument("--weighted-split", action="store_true",
                    help="route decodes with the general SLI-aware router: solo probabilities and class selection "
                         "weights from the configuration's plan")
    ap.add_argument("--immediate", action="store_true",
                    help="decode on the server that ran the prefill, no static partition (the ablation without a decode "
                         "router: M = N)")
    ap.add_argument("--oracle-steps", type=int, default=4000, help="0 skips the CPU baseline")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one device-to-device copy of this size before the timed region "
                         "(a kernel of known traffic to scale hardware counters with)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the simulator runs on one GPU only (replications are independent and would shard "
              "across GPUs without communication, but no multi-GPU path is built); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    # The CPU baseline starts worker processes, so it runs before this process touches the GPU.
    from paper_2602_02987_amd import workloads as W
    base = None
    if args.oracle_steps > 0:
        n_servers = args.servers if args.servers else W.config(args.config).N
        base = cpu_baseline(args.config, n_servers, args.oracle_steps, args.theta, args.random_split, args.immediate,
                            args.weighted_split)

    import torch
    from paper_2602_02987_amd import binding
    over = {}
    if args.servers:
        over["N"] = args.servers
    if args.replications:
        over["replications"] = args.replications
    if args.random_split + args.immediate + args.weighted_split > 1:
        ap.error("--random-split, --weighted-split and --immediate are different decode rules")
    cfg = policy_variant(W, W.config(args.config, **over), args.theta, args.random_split, args.immediate, args.weighted_split)
    default_run = (args.config == 5 and not over and not args.theta and not args.random_split and not args.immediate
                   and not args.weighted_split
                   and args.sim_steps == 1000 and args.preload == 30000)
    slots_per_step = cfg.N * cfg.replications * args.sim_steps

    sim = binding.Sim(cfg)
    for _ in range(args.preload // args.sim_steps):   # same launch size as the timed steps
        sim.run(args.sim_steps)
    if args.preload % args.sim_steps:
        sim.run(args.preload % args.sim_steps)
    for _ in range(args.warmup):
        sim.run(args.sim_steps)
    if args.calibration_copy_mib:
        src = torch.zeros(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    sim.run(0)   # (with no preload and no warm-up this is what puts the empty system in place)
    torch.cuda.synchronize()
    sim.kernel_time(reset=True)
    K = cfg.K
    st0 = sim.stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sim.run(args.sim_steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    launches, kernel_ms = sim.kernel_time()
    st1 = sim.stats()

    slots = float(slots_per_step) * args.steps
    tt0 = st0["tally"][:K]; tt1 = st1["tally"][:K]
    total_bytes, shape = algorithmic_bytes(tt0, st0["glob"], tt1, st1["glob"], slots)
    per_launch_ms = kernel_ms / max(launches, 1)
    achieved = total_bytes / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    own_bytes = shape["bytes_per_slot_with_records_in_lds"] * slots
    achieved_own = own_bytes / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    traffic = measured_traffic() if default_run else None
    iters = float(st1["glob"][0] + st1["glob"][1]) - float(st0["glob"][0] + st0["glob"][1])

    out = {
        "metric": "simulated server-iterations/sec on 1 GPU + achieved HBM GB/s (% of peak)",
        "value": slots / wall,
        "unit": "server-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: K={cfg.K} N={cfg.N} R={cfg.replications} B={cfg.B} C={cfg.C} M={cfg.M}"
                               + (f" theta={args.theta}" if args.theta else "")
                               + (" randomized router" if args.random_split else "")
                               + (" weighted router" if args.weighted_split else "")
                               + (" immediate decode" if args.immediate else "") + ", "
                               f"{args.sim_steps} simulation steps per bench step after {args.preload + args.warmup * args.sim_steps} untimed steps",
                   "server_step_slots_per_bench_step": slots_per_step,
                   "executed_iterations_per_s": iters / wall,
                   "overflow": bool(st1["overflow"])},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     # the same with the bytes this kernel has to move (server clocks, iteration counters and decode
                     # counts stay in LDS for a whole launch and are not part of them)
                     "achieved_own_bytes": achieved_own, "frac_own_bytes": achieved_own / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": (f"stored: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, {TRAFFIC['state']}, sources sha256 "
                                        f"{TRAFFIC['sources_sha256'][:12]}, {TRAFFIC['profile']}" if traffic is not None else
                                        "none: no counter run on these sources and this workload (null)"),
                     "occupancy": occupancy(binding, cfg, sim, cfg.replications, measured("occupancy_percent") if default_run else None),
                     "kernel": "gnr_step_kernel", "launches": launches, "avg_launch_ms": per_launch_ms,
                     "algorithmic_bytes_per_launch": total_bytes / max(launches, 1), **shape},
    }
    if base is not None:
        sim.close()
        del sim
        torch.cuda.empty_cache()
        base["gpu_same_sample"] = gpu_on_the_baseline_sample(binding, torch, cfg, args.oracle_steps)
        out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()
