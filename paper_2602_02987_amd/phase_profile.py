"""Where the step kernel's time goes: builds the library once more with its cycle marks compiled in
(-DGNR_PROF, into libgnr_sim_prof.so next to the normal build) and runs a configuration at the benchmark's state.

Every wave reads the cycle counter at each mark and adds the time since its previous mark to the mark's bucket;
the table gives each bucket's share of all wave-cycles and its cycles per wave and step. The marks cost time
themselves (a step takes a few per cent longer than in the normal build), so the shares are a guide, not a
measurement of the normal build.

    python3 -m paper_2602_02987_amd.phase_profile [--config 5] [--theta 0.1] [--random-split | --weighted-split]
"""
from __future__ import annotations

import argparse
import ctypes
import os
import subprocess
import sys
import time

from . import build as _build

# bucket -> what the time up to that mark was spent on
PHASES = [
    (0, "end of the previous step to the top of this one"),
    (1, "completion pass: before the wave's first block"),
    (2, "completion pass: finishing a block (event list), per block"),
    (3, "completion pass: arrivals of a block (one random block per server)"),
    (4, "completion pass: finishing queued servers, set-up of a round"),
    (11, "completion pass: finishing queued servers, per-server part"),
    (12, "completion pass: finishing queued servers, tallies"),
    (18, "completion pass: opening a block, reads of the on-chip records and tally flush"),
    (19, "completion pass: opening a block, restart of its servers"),
    (20, "completion pass: opening a block, due test and list of slot rows"),
    (21, "completion pass: issuing the loads of a block's first slot rows"),
    (22, "completion pass: waiting for and comparing the slot rows of a block"),
    (23, "completion pass: between the drain and the next block"),
    (5, "completion pass: after the wave's last block"),
    (6, "wait at the barrier that closes the completion pass"),
    (7, "arrivals into the class queues, ranks of completions and idle slots, completions into the buffer (two barriers)"),
    (26, "gate, segment A: class counters (with abandonment: the scan of the class queues)"),
    (27, "gate, segment A: admitted slots per bitmap word"),
    (28, "gate, segment A: ranking the candidates"),
    (24, "routing, segment A: levels of the pass from the load histograms"),
    (25, "routing, segment A: between the two"),
    (9, "routing, segment A: servers of each level per bitmap word"),
    (14, "wait at the barrier after segment A"),
    (29, "weighted router, segment B: class draws"),
    (30, "weighted router, segment B: order within the classes"),
    (31, "weighted router, segment B: walk of the buffer ring"),
    (15, "segment B: admissions take their slots, level counts to ranks, staging of the pass's requests"),
    (16, "wait at the barrier after segment B"),
    (10, "segment C: class counters, placements, restart marks"),
    (17, "wait at the barrier after segment C"),
]


def build_marked() -> str:
    lib = os.path.join(_build.HERE, "libgnr_sim_prof.so")
    srcs = [os.path.join(_build.CSRC, f) for f in os.listdir(_build.CSRC)] + [os.path.join(_build.INCLUDE, "gnr_sim.h")]
    if os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(f) for f in srcs):
        return lib                        # built from the sources as they are
    cmd = ([_build.HIPCC] + _build.FLAGS + ["-DGNR_PROF", f"-I{_build.INCLUDE}", f"-I{_build.CSRC}"]
           + [os.path.join(_build.CSRC, s) for s in _build.SOURCES] + ["-o", lib])
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    return lib


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--preload", type=int, default=31000)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--theta", type=float, default=0.0)
    ap.add_argument("--random-split", action="store_true")
    ap.add_argument("--weighted-split", action="store_true")
    args = ap.parse_args()
    _build.LIB = build_marked()          # the binding loads whatever build.LIB names
    import torch
    from . import binding, workloads as W
    cfg = W.config(args.config)
    lam_plan = [c.lam / 0.95 for c in cfg.classes]
    if args.random_split:
        cfg = W.with_random_split(cfg, lam_plan=lam_plan)
    if args.weighted_split:
        cfg = W.with_weighted_split(cfg, lam_plan=lam_plan)
    if args.theta:
        for c in cfg.classes:
            c.theta = args.theta
    L = binding.lib()
    sim = binding.Sim(cfg)
    sim.run(args.preload)
    torch.cuda.synchronize()
    out = (ctypes.c_ulonglong * 32)()
    L.gnr_prof_read(out, 1)              # read and clear
    t0 = time.perf_counter()
    sim.run(args.steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    L.gnr_prof_read(out, 1)
    threads, _ = sim.launch_shape()
    waves = cfg.replications * (threads // 64)
    total = float(sum(out))
    print(f"{cfg.name}: {args.steps} steps after {args.preload}, {wall / args.steps * 1e6:.1f} us per step with the marks in; "
          f"{total / waves / args.steps:.0f} cycles per wave and step")
    print(f"{'share':>7s} {'cycles/wave/step':>17s}  phase")
    for i, name in PHASES:
        if out[i]:
            print(f"{100.0 * out[i] / total:6.1f}% {out[i] / waves / args.steps:17.0f}  {name}")
    rest = total - sum(out[i] for i, _ in PHASES)
    if rest:
        print(f"{100.0 * rest / total:6.1f}% {rest / waves / args.steps:17.0f}  (other marks)")


if __name__ == "__main__":
    sys.exit(main())
