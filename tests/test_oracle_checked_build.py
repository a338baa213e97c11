"""Sanitizer builds of the oracle (CPU only). First: the oracle built with the compiler's undefined-behaviour checks (signed overflow, shifts, out-of-range
conversions, misaligned or null accesses abort the process) runs every policy variant on the overloaded small
instance and two of the benchmark configurations. CPU only; runs in a child process so that an abort is a test
failure, not the end of the test session. Second: every policy variant in a program of its own built with
AddressSanitizer as well (heap and stack overruns, use after free, leaks abort it). Third: the host side of the
simulator's own library (configuration checks, workspace layout, tables, launch plans, error paths) in a program built
with both sanitizers on the host code; it launches nothing and needs no GPU."""
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


def test_library_host_code_runs_clean_under_the_sanitizers(tmp_path):
    """The C ABI's host logic with AddressSanitizer and the undefined-behaviour checks compiled into the host code
    (device code is compiled as always; the step kernel's variants are replaced by stubs, nothing is launched)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    csrc = os.path.join(ROOT, "paper_2602_02987_amd", "csrc")
    stubs = tmp_path / "stubs.hip"
    stubs.write_text(textwrap.dedent("""
        #include <hip/hip_runtime.h>
        #include "gnr_step.h"
        namespace gnr {
        StepKernel step_kernel_plain(int, bool) { return nullptr; }
        StepKernel step_kernel_rr(int, bool) { return nullptr; }
        StepKernel step_kernel_im(int, bool) { return nullptr; }
        StepKernel step_kernel_ab(int, bool) { return nullptr; }
        StepKernel step_kernel_ab_rr(int, bool) { return nullptr; }
        StepKernel step_kernel_ab_im(int, bool) { return nullptr; }
        StepKernel step_kernel_ws(int, bool) { return nullptr; }
        }
        """))
    flags = ["-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-fno-unroll-loops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer",
             f"-I{os.path.join(ROOT, 'include')}", f"-I{csrc}"]
    sources = [os.path.join(csrc, "gnr_kernels.hip"), os.path.join(csrc, "gnr_api.cpp"), os.path.join(csrc, "gnr_tables.cpp"),
               str(stubs), os.path.join(ROOT, "tests", "host_asan_driver.cpp")]
    objs = []
    procs = []
    for i, src in enumerate(sources):
        obj = str(tmp_path / f"o{i}.o")
        objs.append(obj)
        procs.append(subprocess.Popen([hipcc] + flags + ["-c", src, "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for src, pr in zip(sources, procs):
        out, _ = pr.communicate(timeout=600)
        assert pr.returncode == 0, (src, out[-3000:])
    exe = str(tmp_path / "host_asan")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"] + objs + ["-o", exe])
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0 and "clean" in res.stdout and "runtime error" not in res.stderr and "ERROR" not in res.stderr, \
        (res.stdout[-1500:], res.stderr[-3000:])
