"""Sanitizer builds of the oracle (CPU only). First: the oracle built with the compiler's undefined-behaviour checks (signed overflow, shifts, out-of-range
conversions, misaligned or null accesses abort the process) runs every policy variant on the overloaded small
instance and two of the benchmark configurations. CPU only; runs in a child process so that an abort is a test
failure, not the end of the test session. Second: every policy variant in a program of its own built with
AddressSanitizer as well (heap and stack overruns, use after free, leaks abort it)."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_the_undefined_behaviour_checks(tmp_path):
    script = textwrap.dedent(f"""
        import sys
        sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})
        from dataclasses import replace
        from oracle import binding as ob
        ob.LIB = ob.build_checked({str(tmp_path / 'liboracle_checked.so')!r})
        ob.build = lambda force=False: ob.LIB
        from paper_2602_02987_amd import workloads as W
        from test_oracle_dynamics import _heavy
        base = _heavy()
        impatient = replace(base, classes=[replace(c, theta=t) for c, t in zip(base.classes, (4.0, 0.0, 25.0))])
        split = dict(p_solo=[0.8, 0.3, 0.55], w_solo=[0.5, 0.0, 0.5], w_mixed=[0.1, 0.6, 0.3])
        cases = [base, impatient, replace(base, gate_mode=W.GATE_FCFS), replace(base, gate_mode=W.GATE_PRIORITY),
                 replace(impatient, route_mode=W.ROUTE_RANDOM_SPLIT, **split),
                 replace(impatient, route_mode=W.ROUTE_WEIGHTED_SPLIT, **split),
                 replace(impatient, route_mode=W.ROUTE_IMMEDIATE, M=base.N),
                 replace(base, queue_cap=1, dbuf_cap=1), W.config(1), W.config(5, N=300, replications=1, mod_period=500)]
        for cfg in cases:
            o = ob.Oracle(cfg)
            o.set_check(1)
            o.run(1500)
            o.set_split(cfg.M // 2)
            o.run(500)
            assert o.violations() == (0, 0), cfg.name
            o.stats(); o.digest(0); o.snapshot(0) if hasattr(o, "snapshot") else None
        print("clean")
        """)
    res = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0 and "clean" in res.stdout and "runtime error" not in res.stderr, res.stderr[-2000:]


def test_oracle_runs_clean_under_address_sanitizer(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-Wall", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           os.path.join(ROOT, "tests", "oracle_asan_driver.c"), "-o", exe, "-lm"])
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0 and "clean" in res.stdout and "ERROR" not in res.stderr, (res.stdout[-1000:], res.stderr[-3000:])
