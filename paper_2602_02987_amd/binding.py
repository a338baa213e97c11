"""Thin ctypes binding of the simulator's C ABI (include/gnr_sim.h).

Argument marshalling only: every step of the simulation runs in the library's HIP
kernels. PyTorch provides the device workspace (a uint8 tensor) and the stream.
Importing this module fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import lib_path

MAXK, MAXB, NBIN = 8, 128, 720
TALLY = ["A", "DROP_P", "U_P", "S_P", "U_DM", "U_DS", "S_DM", "S_DS", "M_SM", "M_MS", "DROP_D", "TOKP_PRE",
         "TOKP_DEC", "TOKD_DEC", "TOK_EMIT", "TOK_PREF", "SUM_QP", "SUM_QD", "SUM_X", "SUM_YM", "SUM_YS",
         "WAIT_STEPS", "TTFT_SUM", "E2E_SUM", "TBT_SUM", "AB_P", "AB_D"]
GLOBAL = ["ITERS_MIX", "ITERS_SOLO", "BUSY_MIX", "BUSY_SOLO", "STEPS", "OVERFLOW"]
SIM_EOVERFLOW = -4


class SimClassC(C.Structure):
    _fields_ = [("lam", C.c_double), ("in_law", C.c_int), ("out_law", C.c_int),
                ("in_p0", C.c_double), ("in_p1", C.c_double), ("out_p0", C.c_double), ("out_p1", C.c_double),
                ("in_table", C.c_void_p), ("out_table", C.c_void_p),
                ("price_in", C.c_double), ("price_out", C.c_double), ("bundled", C.c_int),
                ("priority", C.c_double), ("theta", C.c_double)]


class SimConfigC(C.Structure):
    _fields_ = [("K", C.c_int), ("N", C.c_int), ("B", C.c_int), ("C", C.c_int),
                ("c0", C.c_double), ("c_pre", C.c_double), ("c_dec", C.c_double), ("dt", C.c_double),
                ("cls", C.c_void_p), ("M", C.c_int), ("x_star", C.c_void_p), ("qp_star", C.c_void_p),
                ("gate_mode", C.c_int), ("route_mode", C.c_int), ("mod_amp", C.c_double),
                ("mod_period", C.c_int64), ("queue_cap", C.c_int64), ("dbuf_cap", C.c_int64),
                ("p_solo", C.c_void_p), ("w_solo", C.c_void_p), ("w_mixed", C.c_void_p)]


_D8 = C.c_double * MAXK


class SimStatsC(C.Structure):
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


class SimStateC(C.Structure):
    _fields_ = [("class_state", C.c_void_p), ("t_next", C.c_void_p), ("iter", C.c_void_p), ("rem", C.c_void_p),
                ("ptok", C.c_void_p), ("pfjob", C.c_void_p), ("n_cls", C.c_void_p), ("n_join", C.c_void_p),
                ("fin", C.c_void_p), ("job", C.c_void_p), ("n_dec", C.c_void_p),
                ("queue", C.c_void_p * MAXK), ("queue_len", C.c_int64 * MAXK),
                ("dbuf", C.c_void_p), ("dbuf_len", C.c_int64),
                ("queue_dl", C.c_void_p * MAXK), ("dbuf_dl", C.c_void_p),
                ("dbuf_m", C.c_void_p), ("dbuf_m_len", C.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # PyTorch ships its own HIP runtime under the same soname as the system one. Loading it first
        # makes this library bind to it, so that the workspace tensor and the stream belong to the
        # runtime the kernels are launched with (two runtimes in one process do not share pointers).
        import torch  # noqa: F401
        L = C.CDLL(lib_path())
        L.sim_strerror.restype = C.c_char_p
        L.sim_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_size_t)]
        L.sim_onchip_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.sim_launch_plan.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
        L.sim_launch_shape.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_size_t)]
        L.sim_create.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
        L.sim_create_static.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_void_p)]
        L.sim_run.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_void_p]
        L.sim_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.sim_snapshot.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.sim_tallies.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.sim_hist.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.sim_digest.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_uint64), C.c_void_p]
        L.sim_set_targets.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sim_set_split.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.sim_kernel_time.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.c_int, C.c_void_p]
        L.sim_destroy.argtypes = [C.c_void_p]
        L.sim_length_table.argtypes = [C.c_int, C.c_double, C.c_double, C.c_void_p]
        L.sim_patience_table.argtypes = [C.c_double, C.c_double, C.c_void_p]
        L.sim_philox.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.sim_thresholds.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


class SimError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {lib().sim_strerror(code).decode()} ({code})")


def _check(rc, where, allow=()):
    if rc != 0 and rc not in allow:
        raise SimError(rc, where)
    return rc


def marshal_config(cfg):
    """(SimConfigC, keep-alive list) from a workload description."""
    K = cfg.K
    keep = []
    cls = (SimClassC * K)()
    for i, c in enumerate(cfg.classes):
        cls[i].lam = c.lam
        cls[i].in_law, cls[i].out_law = c.in_law, c.out_law
        cls[i].in_p0, cls[i].in_p1, cls[i].out_p0, cls[i].out_p1 = c.in_p0, c.in_p1, c.out_p0, c.out_p1
        for nm in ("in_table", "out_table"):
            t = getattr(c, nm, None)
            if t is not None:
                t = np.ascontiguousarray(t, dtype=np.uint16)
                if t.size != 65536:
                    raise ValueError("length tables need 65536 entries")
                keep.append(t)
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
    cc = SimConfigC(K=K, N=cfg.N, B=cfg.B, C=cfg.C, c0=cfg.c0, c_pre=cfg.c_pre, c_dec=cfg.c_dec, dt=cfg.dt,
                    cls=C.addressof(cls), M=cfg.M, x_star=C.addressof(xs), qp_star=C.addressof(qs),
                    gate_mode=cfg.gate_mode, route_mode=cfg.route_mode, mod_amp=cfg.mod_amp,
                    mod_period=cfg.mod_period, queue_cap=cfg.queue_cap, dbuf_cap=cfg.dbuf_cap,
                    p_solo=C.addressof(ps), w_solo=C.addressof(ws), w_mixed=C.addressof(wm))
    keep += [cls, xs, qs, ps, ws, wm]
    return cc, keep


def sim_onchip_bytes(cfg):
    """(bytes needed, limit) of on-chip memory for `cfg`; host only."""
    cc, _keep = marshal_config(cfg)
    n, lim = C.c_size_t(0), C.c_size_t(0)
    _check(lib().sim_onchip_bytes(C.byref(cc), C.byref(n), C.byref(lim)), "sim_onchip_bytes")
    return n.value, lim.value


def sim_launch_plan(cfg, replications=None):
    """(threads per workgroup, LDS bytes per workgroup, waves per SIMD of the kernel form) for a launch; host only."""
    cc, _keep = marshal_config(cfg)
    t, n, w = C.c_int(0), C.c_size_t(0), C.c_int(0)
    _check(lib().sim_launch_plan(C.byref(cc), cfg.replications if replications is None else replications,
                                 C.byref(t), C.byref(n), C.byref(w)), "sim_launch_plan")
    return t.value, n.value, w.value


def sim_workspace_bytes(cfg, max_replications):
    cc, _keep = marshal_config(cfg)
    n = C.c_size_t(0)
    _check(lib().sim_workspace_bytes(C.byref(cc), int(max_replications), C.byref(n)), "sim_workspace_bytes")
    return n.value


def sim_length_table(law, p0, p1=0.0):
    out = np.zeros(65536, np.uint16)
    _check(lib().sim_length_table(int(law), float(p0), float(p1), out.ctypes.data), "sim_length_table")
    return out


def sim_patience_table(theta, dt):
    out = np.zeros(65536, np.uint16)
    _check(lib().sim_patience_table(float(theta), float(dt), out.ctypes.data), "sim_patience_table")
    return out


def sim_philox(seed, c0, c1, c2, c3):
    out = np.zeros(4, np.uint32)
    _check(lib().sim_philox(int(seed), c0, c1, c2, c3, out.ctypes.data), "sim_philox")
    return out


def sim_thresholds(cfg, rows=1):
    cc, _keep = marshal_config(cfg)
    arr = np.zeros((rows, 3), np.uint32)
    cth = np.zeros(MAXK, np.uint32)
    _check(lib().sim_thresholds(C.byref(cc), rows, arr.ctypes.data, cth.ctypes.data), "sim_thresholds")
    return arr, cth


def _stats_dict(st):
    out = {}
    for name, _typ in st._fields_:
        v = getattr(st, name)
        if name == "tally":
            out[name] = np.array([[v[k][t] for t in range(len(TALLY))] for k in range(MAXK)], dtype=np.uint64)
        elif hasattr(v, "__len__"):
            out[name] = np.array(list(v))
        else:
            out[name] = v
    return out


class Sim:
    """sim_create / sim_run / sim_stats on the current CUDA(HIP) device and stream."""

    def __init__(self, cfg, max_replications=None, device="cuda:0", static_workspace=False):
        """`static_workspace`: use the library's own static device array (sim_create_static: nothing is allocated,
        configurations up to 32 MiB of state) instead of a torch tensor."""
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("the simulator needs a GPU: no HIP device is visible")
        self.torch = torch
        self.cfg = cfg
        self.max_reps = int(max_replications if max_replications is not None else cfg.replications)
        self.device = torch.device(device)
        cc, self._keep = marshal_config(cfg)
        nbytes = C.c_size_t(0)
        _check(lib().sim_workspace_bytes(C.byref(cc), self.max_reps, C.byref(nbytes)), "sim_workspace_bytes")
        self.workspace_bytes = nbytes.value
        with torch.cuda.device(self.device):
            h = C.c_void_p()
            if static_workspace:
                self.workspace = None
                _check(lib().sim_create_static(C.byref(cc), self.max_reps, C.byref(h)), "sim_create_static")
            else:
                self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.device)
                ptr = (self.workspace.data_ptr() + 255) & ~255
                _check(lib().sim_create(C.byref(cc), self.max_reps, C.c_void_p(ptr), nbytes.value, C.byref(h)), "sim_create")
        self.h = h

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "h", None):
            lib().sim_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def run(self, steps, replications=None, seed=None):
        reps = self.cfg.replications if replications is None else replications
        seed = self.cfg.seed if seed is None else seed
        with self.torch.cuda.device(self.device):
            _check(lib().sim_run(self.h, int(steps), int(reps), int(seed), self._stream()), "sim_run")

    def set_targets(self, x_star, qp_star):
        """New gate targets x*, q_p* (per server, K values each) for the steps still to run."""
        x = np.ascontiguousarray(x_star, dtype=np.float64); q = np.ascontiguousarray(qp_star, dtype=np.float64)
        if x.size != self.cfg.K or q.size != self.cfg.K:
            raise ValueError("set_targets wants K values each")
        with self.torch.cuda.device(self.device):
            _check(lib().sim_set_targets(self.h, x.ctypes.data, q.ctypes.data, self._stream()), "sim_set_targets")

    def set_split(self, M):
        """Servers 0..M-1 are the mixed group for the steps still to run; work in service stays where it is."""
        with self.torch.cuda.device(self.device):
            _check(lib().sim_set_split(self.h, int(M), self._stream()), "sim_set_split")

    def stats(self):
        st = SimStatsC()
        with self.torch.cuda.device(self.device):
            rc = _check(lib().sim_stats(self.h, C.byref(st), self._stream()), "sim_stats", allow=(SIM_EOVERFLOW,))
        d = _stats_dict(st)
        d["overflow"] = rc == SIM_EOVERFLOW
        return d

    def launch_shape(self):
        """(threads per workgroup, dynamic LDS bytes per workgroup) of the step kernel."""
        t, n = C.c_int(0), C.c_size_t(0)
        _check(lib().sim_launch_shape(self.h, C.byref(t), C.byref(n)), "sim_launch_shape")
        return t.value, n.value

    def kernel_time(self, reset=False):
        n = C.c_int64(0)
        ms = C.c_double(0.0)
        _check(lib().sim_kernel_time(self.h, C.byref(n), C.byref(ms), int(reset), self._stream()), "sim_kernel_time")
        return n.value, ms.value

    def tallies(self, r):
        K = self.cfg.K
        out = np.zeros(K * len(TALLY) + len(GLOBAL), np.uint64)
        _check(lib().sim_tallies(self.h, int(r), out.ctypes.data, self._stream()), "sim_tallies")
        return out[:K * len(TALLY)].reshape(K, len(TALLY)).copy(), out[K * len(TALLY):].copy()

    def hist(self, r, which):
        out = np.zeros((self.cfg.K, NBIN), np.uint64)
        _check(lib().sim_hist(self.h, int(r), int(which), out.ctypes.data, self._stream()), "sim_hist")
        return out

    def digest(self, r):
        d = C.c_uint64(0)
        _check(lib().sim_digest(self.h, int(r), C.byref(d), self._stream()), "sim_digest")
        return d.value

    def snapshot(self, r):
        """Integer state of replication r as numpy arrays (slots as stored, occupied ones first)."""
        cfg = self.cfg
        K, N, B = cfg.K, cfg.N, cfg.B
        a = dict(class_state=np.zeros((5, K), np.int64), t_next=np.zeros(N, np.int64), iter=np.zeros(N, np.uint32),
                 rem=np.zeros(N, np.int32), ptok=np.zeros(N, np.int32), pfjob=np.zeros(N, np.uint64),
                 n_cls=np.zeros((N, MAXK), np.uint8), n_join=np.zeros((N, MAXK), np.uint8),
                 fin=np.zeros((N, B), np.uint32), job=np.zeros((N, B), np.uint64), n_dec=np.zeros(N, np.int32))
        queues = [np.zeros(cfg.queue_cap, np.uint64) for _ in range(K)]
        dbuf = np.zeros(cfg.dbuf_cap, np.uint64)
        queue_dl = [np.zeros(cfg.queue_cap, np.uint64) for _ in range(K)]
        dbuf_dl = np.zeros(cfg.dbuf_cap, np.uint64)
        dbuf_m = np.zeros(cfg.dbuf_cap, np.uint64)
        st = SimStateC()
        for k, v in a.items():
            setattr(st, k, v.ctypes.data)
        for k in range(K):
            st.queue[k] = queues[k].ctypes.data
            st.queue_dl[k] = queue_dl[k].ctypes.data
        st.dbuf = dbuf.ctypes.data
        st.dbuf_dl = dbuf_dl.ctypes.data
        st.dbuf_m = dbuf_m.ctypes.data
        _check(lib().sim_snapshot(self.h, int(r), C.byref(st), self._stream()), "sim_snapshot")
        a["queues"] = [queues[k][:st.queue_len[k]].copy() for k in range(K)]
        a["dbuf"] = dbuf[:st.dbuf_len].copy()
        a["queue_dl"] = [queue_dl[k][:st.queue_len[k]].copy() for k in range(K)]
        a["dbuf_dl"] = dbuf_dl[:st.dbuf_len].copy()
        a["dbuf_m"] = dbuf_m[:st.dbuf_m_len].copy()
        cs = a.pop("class_state")
        a.update(Qp=cs[0], X=cs[1], Qd=cs[2], Ym=cs[3], Ys=cs[4])
        return a
