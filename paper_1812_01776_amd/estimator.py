"""Python binding of the batched Estimator library (include/estimator.h).

Argument marshalling only: every step of the simulation runs in the HIP kernels behind the C ABI.
The library is loaded from the package directory and there is no fallback: without the built
libestimator.so (or without a GPU) construction fails.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libestimator.so")

EST_OK, EST_EINVAL, EST_ENOMEM, EST_EDEVICE, EST_EUNSUPPORTED, EST_EINTERNAL = 0, -1, -2, -3, -4, -5
EST_STATIC_SCRATCH_BYTES = 64 << 20  # fixed scratch of estimator_run_static_dev (include/estimator.h)
_ERR_NAMES = {-1: "EST_EINVAL", -2: "EST_ENOMEM", -3: "EST_EDEVICE", -4: "EST_EUNSUPPORTED", -5: "EST_EINTERNAL"}

CFG_DTYPE = np.dtype([("hw", "u1"), ("batch", "u1"), ("replicas", "<u2")])

SYMBOLS = ["estimator_create", "estimator_run", "estimator_run_dev", "estimator_run_latencies",
           "estimator_run_latencies_dev", "estimator_workspace_bytes", "estimator_last_stats",
           "estimator_last_error", "estimator_destroy", "estimator_plan", "estimator_tuner_handoff",
           "estimator_run_shared_dev", "estimator_run_static_dev", "estimator_profile_tail"]


class EstimatorError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("%s (%d): %s" % (_ERR_NAMES.get(code, "?"), code, text))
        self.code = code


class _Dag(ctypes.Structure):
    _fields_ = [("n_stages", ctypes.c_uint32), ("parent_off", ctypes.POINTER(ctypes.c_uint32)),
                ("parent_idx", ctypes.POINTER(ctypes.c_uint32))]


class _Profiles(ctypes.Structure):
    _fields_ = [("n_hw", ctypes.c_uint32), ("max_batch", ctypes.c_uint32),
                ("lat_us", ctypes.POINTER(ctypes.c_uint32)), ("cost_uusd_hr", ctypes.POINTER(ctypes.c_uint64))]


class _Trace(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint64), ("arrival_us", ctypes.c_void_p), ("visit_mask", ctypes.c_void_p)]


class _Result(ctypes.Structure):
    _fields_ = [("p99_us", ctypes.c_void_p), ("miss_count", ctypes.c_void_p), ("cost_uusd_hr", ctypes.c_void_p)]


class _PlanResult(ctypes.Structure):
    _fields_ = [("feasible", ctypes.c_uint32), ("n_steps", ctypes.c_uint32), ("estimator_calls", ctypes.c_uint32),
                ("p99_us", ctypes.c_uint32), ("candidates", ctypes.c_uint64), ("cost_uusd_hr", ctypes.c_uint64)]


class _PlanStep(ctypes.Structure):
    _fields_ = [("action", ctypes.c_uint32), ("stage", ctypes.c_int32), ("cost_uusd_hr", ctypes.c_uint64)]


class _Handoff(ctypes.Structure):
    _fields_ = [("n_windows", ctypes.c_uint32), ("reserved", ctypes.c_uint32), ("window_us", ctypes.c_uint64 * 32),
                ("max_queries", ctypes.c_uint32 * 32), ("mu_num", ctypes.c_uint64 * 32), ("mu_den", ctypes.c_uint64 * 32),
                ("rho_num", ctypes.c_uint64 * 32), ("rho_den", ctypes.c_uint64 * 32)]


PLAN_ACTIONS = ("init", "batch", "replica", "hw")


class Stats(ctypes.Structure):
    _fields_ = [("n_launches", ctypes.c_uint32), ("n_slots", ctypes.c_uint32), ("sim_ms", ctypes.c_float),
                ("prep_ms", ctypes.c_float), ("stage_visits", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64),
                ("capture_ms", ctypes.c_float), ("ops_run_fraction", ctypes.c_float),
                ("waves_per_candidate", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


def load_library(path=LIB_PATH):
    if not os.path.exists(path):
        raise RuntimeError("the HIP library %s is not built; run `python -c 'import __graft_entry__ as g; g.build()'`" % path)
    # PyTorch ships its own copy of the HIP runtime; load it first so that this library binds to the
    # same runtime instance (two instances in one process do not both see the GPU).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(path)
    lib.estimator_create.restype = ctypes.c_int
    lib.estimator_run.restype = ctypes.c_int
    lib.estimator_run_dev.restype = ctypes.c_int
    lib.estimator_run_latencies.restype = ctypes.c_int
    lib.estimator_run_latencies_dev.restype = ctypes.c_int
    lib.estimator_workspace_bytes.restype = ctypes.c_uint64
    lib.estimator_last_stats.restype = ctypes.c_int
    lib.estimator_last_error.restype = ctypes.c_char_p
    lib.estimator_destroy.restype = None
    lib.estimator_plan.restype = ctypes.c_int
    lib.estimator_tuner_handoff.restype = ctypes.c_int
    lib.estimator_run_shared_dev.restype = ctypes.c_int
    lib.estimator_run_static_dev.restype = ctypes.c_int
    lib.estimator_profile_tail.restype = ctypes.c_int
    return lib


EST_TAIL_PERCENTILE, EST_TAIL_SIGMA = 0, 1


def profile_tail(samples_us, mode, param, lib=None):
    """estimator_profile_tail: samples_us [..., n_samples] uint32 -> the table of tails, shape samples_us.shape[:-1]."""
    lib = lib or load_library()
    x = np.ascontiguousarray(samples_us, dtype=np.uint32)
    out = np.zeros(x.shape[:-1], np.uint32)
    rc = lib.estimator_profile_tail(_ptr(x), ctypes.c_uint64(out.size), ctypes.c_uint32(x.shape[-1]), ctypes.c_uint32(mode),
                                    ctypes.c_uint32(param), _ptr(out))
    if rc != EST_OK:
        raise EstimatorError(rc, "estimator_profile_tail")
    return out


def pack_configs(cfg_hw, cfg_batch, cfg_replicas):
    """[C][S] arrays -> est_stage_cfg_t[C][S]."""
    hw = np.asarray(cfg_hw)
    out = np.zeros(hw.shape, dtype=CFG_DTYPE)
    out["hw"] = hw
    out["batch"] = np.asarray(cfg_batch)
    out["replicas"] = np.asarray(cfg_replicas)
    return np.ascontiguousarray(out)


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


class Estimator:
    """estimator_create / estimator_run / estimator_run_latencies / estimator_run_dev."""

    def __init__(self, parents, lat_us, cost_uusd_hr, _lib=None):
        self._lib = _lib if _lib is not None else load_library()
        self._h = ctypes.c_void_p()
        lat = np.ascontiguousarray(lat_us, dtype=np.uint32)
        cost = np.ascontiguousarray(cost_uusd_hr, dtype=np.uint64)
        S, H, Bmax = lat.shape
        assert cost.shape == (S, H) and len(parents) == S
        self.S = S
        off = np.zeros(S + 1, dtype=np.uint32)
        idx = []
        for s, ps in enumerate(parents):
            idx.extend(int(p) for p in ps)
            off[s + 1] = len(idx)
        idx = np.asarray(idx if idx else [0], dtype=np.uint32)
        dag = _Dag(S, off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
        prof = _Profiles(H, Bmax, lat.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                         cost.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
        rc = self._lib.estimator_create(ctypes.byref(dag), ctypes.byref(prof), ctypes.byref(self._h))
        if rc != EST_OK:
            self._h = ctypes.c_void_p()
            raise EstimatorError(rc, "estimator_create failed")
        self.n_stages = S

    def close(self):
        if self._h:
            self._lib.estimator_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != EST_OK:
            raise EstimatorError(rc, self._lib.estimator_last_error(self._h).decode())

    # ---- host-pointer entry points
    def run(self, arrival_us, visit_mask, configs, slo_us):
        arr = np.ascontiguousarray(arrival_us, dtype=np.uint32)
        msk = np.ascontiguousarray(visit_mask, dtype=np.uint32)
        cfg = np.ascontiguousarray(configs, dtype=CFG_DTYPE)
        C = cfg.shape[0] if cfg.ndim == 2 else 0
        p99 = np.zeros(max(C, 1), np.uint32); miss = np.zeros(max(C, 1), np.uint32); cost = np.zeros(max(C, 1), np.uint64)
        tr = _Trace(arr.shape[0], _ptr(arr), _ptr(msk))
        res = _Result(_ptr(p99), _ptr(miss), _ptr(cost))
        self._check(self._lib.estimator_run(self._h, ctypes.byref(tr), _ptr(cfg), ctypes.c_uint64(C),
                                            ctypes.c_uint32(slo_us), ctypes.byref(res)))
        return {"p99_us": p99[:C], "miss_count": miss[:C], "cost_uusd_hr": cost[:C]}

    def run_latencies(self, arrival_us, visit_mask, configs):
        arr = np.ascontiguousarray(arrival_us, dtype=np.uint32)
        msk = np.ascontiguousarray(visit_mask, dtype=np.uint32)
        cfg = np.ascontiguousarray(configs, dtype=CFG_DTYPE)
        C = cfg.shape[0] if cfg.ndim == 2 else 0
        n = arr.shape[0]
        lat = np.zeros((max(C, 1), max(n, 1)), np.uint32)
        tr = _Trace(n, _ptr(arr), _ptr(msk))
        self._check(self._lib.estimator_run_latencies(self._h, ctypes.byref(tr), _ptr(cfg), ctypes.c_uint64(C), _ptr(lat)))
        return lat[:C, :n]

    def plan(self, arrival_us, visit_mask, slo_us, max_replicas=64, max_steps=4096):
        """estimator_plan: returns None if no feasible configuration exists, else a dict with the
        configuration ([S] records), its cost and P99, the accepted steps and the call counts."""
        arr = np.ascontiguousarray(arrival_us, dtype=np.uint32)
        msk = np.ascontiguousarray(visit_mask, dtype=np.uint32)
        tr = _Trace(arr.shape[0], _ptr(arr), _ptr(msk))
        cfg = np.zeros(self.S, dtype=CFG_DTYPE)
        res = _PlanResult()
        steps = (_PlanStep * max_steps)()
        self._check(self._lib.estimator_plan(self._h, ctypes.byref(tr), ctypes.c_uint32(slo_us), ctypes.c_uint32(max_replicas),
                                             _ptr(cfg), ctypes.byref(res), steps, ctypes.c_uint32(max_steps)))
        if not res.feasible:
            return None
        log = [(PLAN_ACTIONS[steps[i].action], steps[i].stage, steps[i].cost_uusd_hr) for i in range(min(res.n_steps, max_steps))]
        return {"config": cfg, "cost_uusd_hr": res.cost_uusd_hr, "p99_us": res.p99_us, "steps": log, "n_steps": res.n_steps,
                "estimator_calls": res.estimator_calls, "candidates": res.candidates}

    def tuner_handoff(self, arrival_us, visit_mask, config, service_time_us):
        """estimator_tuner_handoff: window widths, the envelope's query counts, and per model the exact
        integer pairs (mu_num, mu_den), (rho_num, rho_den)."""
        arr = np.ascontiguousarray(arrival_us, dtype=np.uint32)
        msk = np.ascontiguousarray(visit_mask, dtype=np.uint32)
        cfg = np.ascontiguousarray(config, dtype=CFG_DTYPE).reshape(-1)
        tr = _Trace(arr.shape[0], _ptr(arr), _ptr(msk))
        out = _Handoff()
        self._check(self._lib.estimator_tuner_handoff(self._h, ctypes.byref(tr), _ptr(cfg), ctypes.c_uint32(service_time_us),
                                                      ctypes.byref(out)))
        k = out.n_windows
        return {"window_us": list(out.window_us[:k]), "max_queries": list(out.max_queries[:k]),
                "mu": [(out.mu_num[s], out.mu_den[s]) for s in range(self.S)],
                "rho": [(out.rho_num[s], out.rho_den[s]) for s in range(self.S)]}

    # ---- device-pointer entry points (torch tensors on the GPU supply memory and the stream)
    def run_dev(self, arrival_t, mask_t, cfg_t, n_cfg, slo_us, workspace_t=None, stream=None):
        """arrival_t, mask_t: int32 CUDA tensors [n] holding the uint32 bit patterns; cfg_t: uint8 CUDA
        tensor of n_cfg*S*4 bytes (est_stage_cfg_t); workspace_t: optional uint8 CUDA tensor.
        Returns int32/int64 CUDA tensors holding the uint32/uint64 results."""
        import torch
        dev = arrival_t.device
        n = arrival_t.numel()
        p99 = torch.empty(max(n_cfg, 1), dtype=torch.int32, device=dev)
        miss = torch.empty(max(n_cfg, 1), dtype=torch.int32, device=dev)
        cost = torch.empty(max(n_cfg, 1), dtype=torch.int64, device=dev)
        tr = _Trace(n, ctypes.c_void_p(arrival_t.data_ptr()), ctypes.c_void_p(mask_t.data_ptr()))
        res = _Result(ctypes.c_void_p(p99.data_ptr()), ctypes.c_void_p(miss.data_ptr()), ctypes.c_void_p(cost.data_ptr()))
        ws_ptr = ctypes.c_void_p(workspace_t.data_ptr()) if workspace_t is not None else ctypes.c_void_p()
        ws_len = workspace_t.numel() if workspace_t is not None else 0
        st = stream if stream is not None else torch.cuda.current_stream(dev)
        self._check(self._lib.estimator_run_dev(self._h, ctypes.byref(tr), ctypes.c_void_p(cfg_t.data_ptr()),
                                                ctypes.c_uint64(n_cfg), ctypes.c_uint32(slo_us), ctypes.byref(res), ws_ptr,
                                                ctypes.c_uint64(ws_len), ctypes.c_void_p(st.cuda_stream)))
        return {"p99_us": p99[:n_cfg], "miss_count": miss[:n_cfg], "cost_uusd_hr": cost[:n_cfg]}

    def run_static_dev(self, arrival_t, mask_t, cfg_t, n_cfg, slo_us, p99_t, miss_t, cost_t, stream=None):
        """run_dev through the entry point that allocates nothing: the caller passes the result tensors
        too (int32 [n_cfg], int32 [n_cfg], int64 [n_cfg], CUDA), the scratch is the library's fixed array."""
        import torch
        tr = _Trace(arrival_t.numel(), ctypes.c_void_p(arrival_t.data_ptr()), ctypes.c_void_p(mask_t.data_ptr()))
        res = _Result(ctypes.c_void_p(p99_t.data_ptr()), ctypes.c_void_p(miss_t.data_ptr()), ctypes.c_void_p(cost_t.data_ptr()))
        st = stream if stream is not None else torch.cuda.current_stream(arrival_t.device)
        self._check(self._lib.estimator_run_static_dev(self._h, ctypes.byref(tr), ctypes.c_void_p(cfg_t.data_ptr()),
                                                       ctypes.c_uint64(n_cfg), ctypes.c_uint32(slo_us), ctypes.byref(res),
                                                       ctypes.c_void_p(st.cuda_stream)))

    def run_shared_dev(self, arrival_t, mask_t, bases_t, n_bases, cfg_t, base_of_t, n_cfg, slo_us, stream=None):
        """run_dev for candidates that share upstream stages with bases: bases_t like cfg_t
        (n_bases*S*4 bytes), base_of_t an int32 CUDA tensor [n_cfg] of base indices.  Same results."""
        import torch
        dev = arrival_t.device
        n = arrival_t.numel()
        p99 = torch.empty(max(n_cfg, 1), dtype=torch.int32, device=dev)
        miss = torch.empty(max(n_cfg, 1), dtype=torch.int32, device=dev)
        cost = torch.empty(max(n_cfg, 1), dtype=torch.int64, device=dev)
        tr = _Trace(n, ctypes.c_void_p(arrival_t.data_ptr()), ctypes.c_void_p(mask_t.data_ptr()))
        res = _Result(ctypes.c_void_p(p99.data_ptr()), ctypes.c_void_p(miss.data_ptr()), ctypes.c_void_p(cost.data_ptr()))
        st = stream if stream is not None else torch.cuda.current_stream(dev)
        self._check(self._lib.estimator_run_shared_dev(
            self._h, ctypes.byref(tr), ctypes.c_void_p(bases_t.data_ptr()), ctypes.c_uint64(n_bases),
            ctypes.c_void_p(cfg_t.data_ptr()), ctypes.c_void_p(base_of_t.data_ptr()), ctypes.c_uint64(n_cfg),
            ctypes.c_uint32(slo_us), ctypes.byref(res), ctypes.c_void_p(st.cuda_stream)))
        return {"p99_us": p99[:n_cfg], "miss_count": miss[:n_cfg], "cost_uusd_hr": cost[:n_cfg]}

    def run_latencies_dev(self, arrival_t, mask_t, cfg_t, n_cfg, workspace_t=None, stream=None):
        import torch
        dev = arrival_t.device
        n = arrival_t.numel()
        lat = torch.empty((max(n_cfg, 1), max(n, 1)), dtype=torch.int32, device=dev)
        tr = _Trace(n, ctypes.c_void_p(arrival_t.data_ptr()), ctypes.c_void_p(mask_t.data_ptr()))
        ws_ptr = ctypes.c_void_p(workspace_t.data_ptr()) if workspace_t is not None else ctypes.c_void_p()
        ws_len = workspace_t.numel() if workspace_t is not None else 0
        st = stream if stream is not None else torch.cuda.current_stream(dev)
        self._check(self._lib.estimator_run_latencies_dev(self._h, ctypes.byref(tr), ctypes.c_void_p(cfg_t.data_ptr()),
                                                          ctypes.c_uint64(n_cfg), ctypes.c_void_p(lat.data_ptr()), ws_ptr,
                                                          ctypes.c_uint64(ws_len), ctypes.c_void_p(st.cuda_stream)))
        return lat[:n_cfg, :n]

    def workspace_bytes(self, n, n_cfg):
        return int(self._lib.estimator_workspace_bytes(self._h, ctypes.c_uint64(n), ctypes.c_uint64(n_cfg)))

    def stats(self):
        s = Stats()
        self._check(self._lib.estimator_last_stats(self._h, ctypes.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}
