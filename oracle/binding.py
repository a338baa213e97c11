"""ctypes wrapper of the CPU oracle (test infrastructure; never imported by the product).

`build()` compiles gnr_oracle.c with gcc; `Oracle(cfg)` takes any object with the
attributes of a workload description (K, N, B, C, c0, c_pre, c_dec, dt, classes, M,
x_star, qp_star, gate_mode, route_mode, mod_amp, mod_period, queue_cap, dbuf_cap).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gnr_oracle.c")
LIB = os.path.join(HERE, "libgnr_oracle.so")
MAXK = 8


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", SRC, "-o", LIB, "-lm"])
    return LIB


def build_checked(path: str) -> str:
    """A copy of the oracle built with the compiler's undefined-behaviour checks (any finding aborts the process)."""
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-fsanitize=undefined", "-fno-sanitize-recover=all", SRC, "-o", path, "-lm"])
    return path


class _Class(C.Structure):
    _fields_ = [("lam", C.c_double), ("in_law", C.c_int), ("out_law", C.c_int),
                ("in_p0", C.c_double), ("in_p1", C.c_double), ("out_p0", C.c_double), ("out_p1", C.c_double),
                ("in_table", C.c_void_p), ("out_table", C.c_void_p),
                ("price_in", C.c_double), ("price_out", C.c_double), ("bundled", C.c_int),
                ("priority", C.c_double), ("theta", C.c_double)]


class _Config(C.Structure):
    _fields_ = [("K", C.c_int), ("N", C.c_int), ("B", C.c_int), ("C", C.c_int),
                ("c0", C.c_double), ("c_pre", C.c_double), ("c_dec", C.c_double), ("dt", C.c_double),
                ("cls", C.c_void_p), ("M", C.c_int), ("x_star", C.c_void_p), ("qp_star", C.c_void_p),
                ("gate_mode", C.c_int), ("route_mode", C.c_int), ("mod_amp", C.c_double),
                ("mod_period", C.c_int64), ("queue_cap", C.c_int64), ("dbuf_cap", C.c_int64),
                ("p_solo", C.c_void_p), ("w_solo", C.c_void_p), ("w_mixed", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_violations.restype = C.c_int64
        _lib.oracle_check.restype = C.c_int64
        _lib.oracle_steps_done.restype = C.c_int64
        _lib.oracle_hedge.restype = C.c_int64
        _lib.oracle_hedge.argtypes = [C.c_int]
        _lib.oracle_hbin.argtypes = [C.c_int64]
        _lib.oracle_philox.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        _lib.oracle_length_table.argtypes = [C.c_int, C.c_double, C.c_double, C.c_void_p]
        _lib.oracle_run.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_uint64]
        _lib.oracle_set_targets.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.oracle_patience_table.argtypes = [C.c_double, C.c_double, C.c_void_p]
        _lib.oracle_poke.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64]
    return _lib


TALLY = ["A", "DROP_P", "U_P", "S_P", "U_DM", "U_DS", "S_DM", "S_DS", "M_SM", "M_MS", "DROP_D", "TOKP_PRE",
         "TOKP_DEC", "TOKD_DEC", "TOK_EMIT", "TOK_PREF", "SUM_QP", "SUM_QD", "SUM_X", "SUM_YM", "SUM_YS",
         "WAIT_STEPS", "TTFT_SUM", "E2E_SUM", "TBT_SUM", "AB_P", "AB_D"]
GLOBAL = ["ITERS_MIX", "ITERS_SOLO", "BUSY_MIX", "BUSY_SOLO", "STEPS", "OVERFLOW"]
NBIN = 720

_D8 = C.c_double * MAXK


class Stats(C.Structure):
    _fields_ = [("K", C.c_int32), ("replications", C.c_int32), ("steps", C.c_int64), ("sim_time", C.c_double),
                ("tally", (C.c_uint64 * len(TALLY)) * MAXK), ("glob", C.c_uint64 * len(GLOBAL)),
                ("arrival_rate", _D8), ("completion_rate", _D8), ("served_fraction", _D8),
                ("tok_rate_prefill", _D8), ("tok_rate_decode", _D8),
                ("rev_bundled", _D8), ("rev_separate", _D8), ("rev_mixed", _D8),
                ("rev_bundled_total", C.c_double), ("rev_separate_total", C.c_double), ("rev_mixed_total", C.c_double),
                ("mean_qp", _D8), ("mean_qd", _D8), ("mean_x", _D8), ("mean_ym", _D8), ("mean_ys", _D8),
                ("ttft_mean", _D8), ("ttft_p50", _D8), ("ttft_p95", _D8), ("ttft_p99", _D8),
                ("e2e_mean", _D8), ("e2e_p50", _D8), ("e2e_p95", _D8), ("e2e_p99", _D8),
                ("tbt_mean", _D8), ("tbt_p50", _D8), ("tbt_p95", _D8), ("tbt_p99", _D8),
                ("mean_wait", _D8), ("fair_gap_x", C.c_double), ("fair_gap_ys", C.c_double),
                ("fair_min_served", C.c_double), ("util_mix", C.c_double), ("util_solo", C.c_double),
                ("iter_rate", C.c_double), ("abandon_rate_p", _D8), ("abandon_rate_d", _D8)]


def stats_to_dict(st) -> dict:
    out = {}
    for name, typ in st._fields_:
        v = getattr(st, name)
        if name == "tally":
            out[name] = np.array([[v[k][t] for t in range(len(TALLY))] for k in range(MAXK)], dtype=np.uint64)
        elif hasattr(v, "__len__"):
            out[name] = np.array(list(v))
        else:
            out[name] = v
    return out


def philox(seed, c0, c1, c2, c3):
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox(seed, c0, c1, c2, c3, out.ctypes.data)
    return out


def length_table(law, p0, p1=0.0):
    out = np.zeros(65536, dtype=np.uint16)
    rc = lib().oracle_length_table(law, float(p0), float(p1), out.ctypes.data)
    if rc:
        raise ValueError("bad length law")
    return out


def patience_table(theta, dt):
    out = np.zeros(65536, dtype=np.uint16)
    if lib().oracle_patience_table(float(theta), float(dt), out.ctypes.data):
        raise ValueError("bad patience rate")
    return out


def hbin(v):
    return lib().oracle_hbin(int(v))


def hedge(b):
    return lib().oracle_hedge(int(b))


class Oracle:
    def __init__(self, cfg, max_reps=None):
        L = lib()
        self.cfg = cfg
        K = cfg.K
        self._keep = []
        cls = (_Class * K)()
        for i, c in enumerate(cfg.classes):
            cls[i].lam = c.lam
            cls[i].in_law, cls[i].out_law = c.in_law, c.out_law
            cls[i].in_p0, cls[i].in_p1, cls[i].out_p0, cls[i].out_p1 = c.in_p0, c.in_p1, c.out_p0, c.out_p1
            for nm in ("in_table", "out_table"):
                t = getattr(c, nm, None)
                if t is not None:
                    t = np.ascontiguousarray(t, dtype=np.uint16)
                    assert t.size == 65536
                    self._keep.append(t)
                    setattr(cls[i], nm, t.ctypes.data)
            cls[i].price_in, cls[i].price_out = c.price_in, c.price_out
            cls[i].bundled = c.bundled
            cls[i].priority = c.priority
            cls[i].theta = c.theta
        xs = (C.c_double * K)(*cfg.x_star)
        qs = (C.c_double * K)(*cfg.qp_star)
        ps = (C.c_double * K)(*(list(getattr(cfg, "p_solo", [])) or [1.0] * K))
        ws = (C.c_double * K)(*(list(getattr(cfg, "w_solo", [])) or [1.0 / K] * K))
        wm = (C.c_double * K)(*(list(getattr(cfg, "w_mixed", [])) or [1.0 / K] * K))
        cc = _Config(K=K, N=cfg.N, B=cfg.B, C=cfg.C, c0=cfg.c0, c_pre=cfg.c_pre, c_dec=cfg.c_dec, dt=cfg.dt,
                     cls=C.addressof(cls), M=cfg.M, x_star=C.addressof(xs), qp_star=C.addressof(qs),
                     gate_mode=cfg.gate_mode, route_mode=cfg.route_mode, mod_amp=cfg.mod_amp,
                     mod_period=cfg.mod_period, queue_cap=cfg.queue_cap, dbuf_cap=cfg.dbuf_cap,
                     p_solo=C.addressof(ps), w_solo=C.addressof(ws), w_mixed=C.addressof(wm))
        self.max_reps = int(max_reps if max_reps is not None else cfg.replications)
        h = C.c_void_p()
        rc = L.oracle_create(C.byref(cc), self.max_reps, C.byref(h))
        if rc:
            raise ValueError(f"oracle_create failed ({rc})")
        self.h = h
        self.L = L

    def __del__(self):
        if getattr(self, "h", None):
            self.L.oracle_destroy(self.h)
            self.h = None

    def select(self, ids):
        arr = (C.c_int * len(ids))(*ids)
        self.L.oracle_select(self.h, arr, len(ids))

    def set_check(self, every):
        self.L.oracle_set_check(self.h, int(every))

    def run(self, steps, replications=None, seed=None):
        reps = self.cfg.replications if replications is None else replications
        seed = self.cfg.seed if seed is None else seed
        rc = self.L.oracle_run(self.h, int(steps), int(reps), int(seed))
        if rc:
            raise RuntimeError(f"oracle_run failed ({rc})")

    def set_targets(self, x_star, qp_star):
        """New gate targets from here on; the state is kept."""
        x = np.ascontiguousarray(x_star, dtype=np.float64); q = np.ascontiguousarray(qp_star, dtype=np.float64)
        assert x.size == self.cfg.K and q.size == self.cfg.K
        if self.L.oracle_set_targets(self.h, x.ctypes.data, q.ctypes.data):
            raise RuntimeError("oracle_set_targets failed")

    def set_split(self, M):
        """Servers 0..M-1 are the mixed group from here on; work in service stays where it is."""
        if self.L.oracle_set_split(self.h, int(M)):
            raise RuntimeError("oracle_set_split failed")

    def violations(self):
        return int(self.L.oracle_violations(self.h)), int(self.L.oracle_first_violation(self.h))

    def check(self):
        return int(self.L.oracle_check(self.h))

    def poke(self, r, what, i, delta):
        """Test hook: adds `delta` to one number of replication r's state (see oracle_poke)."""
        if self.L.oracle_poke(self.h, int(r), int(what), int(i), C.c_int64(int(delta))):
            raise RuntimeError("oracle_poke: nothing to perturb there")

    def clear_violations(self):
        self.L.oracle_clear_violations(self.h)

    def violation_codes(self):
        """The distinct codes the checker has reported since the last clear."""
        out = (C.c_int * 64)()
        n = self.L.oracle_violation_codes(self.h, out, 64)
        return sorted(out[i] for i in range(min(n, 64)))

    def steps_done(self):
        return int(self.L.oracle_steps_done(self.h))

    def class_state(self, r):
        K = self.cfg.K
        out = np.zeros((5, K), dtype=np.int64)
        assert self.L.oracle_get_class_state(self.h, r, out.ctypes.data_as(C.c_void_p)) == 0
        return dict(Qp=out[0], X=out[1], Qd=out[2], Ym=out[3], Ys=out[4])

    def servers(self, r):
        N = self.cfg.N
        t_next = np.zeros(N, np.int64); it = np.zeros(N, np.uint32); rem = np.zeros(N, np.int32)
        ptok = np.zeros(N, np.int32); pf = np.zeros(N, np.uint64)
        ncls = np.zeros((N, MAXK), np.uint8); njoin = np.zeros((N, MAXK), np.uint8)
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        assert self.L.oracle_get_servers(self.h, r, p(t_next), p(it), p(rem), p(ptok), p(pf), p(ncls), p(njoin)) == 0
        return dict(t_next=t_next, iter=it, rem=rem, ptok=ptok, pfjob=pf, n_cls=ncls, n_join=njoin)

    def slots(self, r):
        """Occupied slots per server as (fin, job) sorted lexicographically; unused entries zero."""
        N, B = self.cfg.N, self.cfg.B
        fin = np.zeros((N, B), np.uint32); job = np.zeros((N, B), np.uint64); nd = np.zeros(N, np.int32)
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        assert self.L.oracle_get_slots(self.h, r, p(fin), p(job), p(nd)) == 0
        return canonical_slots(fin, job, nd)

    def queue(self, r, k):
        ln = C.c_int64(0)
        cap = int(max(self.cfg.queue_cap, self.cfg.dbuf_cap))
        out = np.zeros(cap, np.uint64)
        assert self.L.oracle_get_queue(self.h, r, k, out.ctypes.data_as(C.c_void_p), C.c_int64(cap), C.byref(ln)) == 0
        return out[:ln.value].copy()

    def queue_deadlines(self, r, k):
        """Steps at which the entries of queue(r, k) abandon if still waiting (0xFFFFFFFF: never)."""
        ln = C.c_int64(0)
        cap = int(max(self.cfg.queue_cap, self.cfg.dbuf_cap))
        out = np.zeros(cap, np.uint64)
        assert self.L.oracle_get_queue_deadlines(self.h, r, k, out.ctypes.data_as(C.c_void_p), C.c_int64(cap),
                                                 C.byref(ln)) == 0
        return out[:ln.value].copy()

    def tallies(self, r):
        K = self.cfg.K
        out = np.zeros(K * len(TALLY) + len(GLOBAL), np.uint64)
        assert self.L.oracle_get_tallies(self.h, r, out.ctypes.data_as(C.c_void_p)) == 0
        return out[:K * len(TALLY)].reshape(K, len(TALLY)).copy(), out[K * len(TALLY):].copy()

    def hist(self, r, which):
        out = np.zeros((self.cfg.K, NBIN), np.uint64)
        assert self.L.oracle_get_hist(self.h, r, which, out.ctypes.data_as(C.c_void_p)) == 0
        return out

    def tables(self, k, rows=1):
        tin = np.zeros(65536, np.uint16); tout = np.zeros(65536, np.uint16)
        cthr = np.zeros(MAXK, np.uint32); athr = np.zeros((rows, 3), np.uint32)
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        assert self.L.oracle_get_tables(self.h, k, p(tin), p(tout), p(cthr), p(athr), C.c_int64(rows)) == 0
        return tin, tout, cthr, athr

    def digest(self, r):
        d = C.c_uint64(0)
        assert self.L.oracle_digest(self.h, r, C.byref(d)) == 0
        return d.value

    def stats(self):
        st = Stats()
        assert self.L.oracle_stats_size() == C.sizeof(Stats)
        assert self.L.oracle_stats(self.h, C.byref(st)) == 0
        return stats_to_dict(st)


def canonical_slots(fin, job, nd):
    """Sort each server's occupied slots by (fin, job); the slot position carries no meaning."""
    N, B = fin.shape
    fin = fin.copy(); job = job.copy()
    for g in range(N):
        n = int(nd[g])
        if n > 1:
            order = np.lexsort((job[g, :n], fin[g, :n]))
            fin[g, :n] = fin[g, :n][order]; job[g, :n] = job[g, :n][order]
    return dict(fin=fin, job=job, n_dec=nd.copy())


def unpack_job(w):
    w = int(w)
    return dict(stamp=w & ((1 << 29) - 1), cls=(w >> 29) & 7, P=((w >> 32) & 0xFFFF) + 1, D=((w >> 48) & 0xFFFF) + 1)
