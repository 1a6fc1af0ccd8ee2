"""ctypes binding of the CPU oracle (oracle/estimator_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's cpu_baseline leg may
import this module; the GPU library and its Python binding never do.

The oracle is the discrete-event Estimator of arXiv 1812.01776, Section 4.2, written as a
plain single-threaded global-event-queue simulator.  This file only marshals arguments.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "estimator_oracle.c")
_LIB = os.path.join(_HERE, "libestimator_oracle.so")

HORIZON = 2**32 - 1  # production horizon, us


def build(force=False):
    """Compile the oracle with gcc (plain C99, -O2)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    subprocess.check_call(["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_simulate.restype = ctypes.c_int
        _lib.oracle_run.restype = ctypes.c_int
        _lib.oracle_p99.restype = ctypes.c_uint64
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _dag_arrays(parents):
    """parents: list (one entry per stage) of lists of parent indices -> CSR arrays."""
    off = np.zeros(len(parents) + 1, dtype=np.uint32)
    idx = []
    for s, ps in enumerate(parents):
        idx.extend(int(p) for p in ps)
        off[s + 1] = len(idx)
    return off, np.asarray(idx if idx else [0], dtype=np.uint32)


def simulate(parents, lat_us, arrival, mask, hw, batch, replicas, horizon=HORIZON,
             want_stages=False, want_batches=False):
    """One configuration.  Returns dict with 'latency' (uint64[n]) and, on request,
    'ready'/'done' (uint64[S][n]) and 'batches' (uint64[nb][4]: stage, start, end, size)."""
    lib = _load()
    lat_us = np.ascontiguousarray(lat_us, dtype=np.uint32)
    S, H, Bmax = lat_us.shape
    off, idx = _dag_arrays(parents)
    arrival = np.ascontiguousarray(arrival, dtype=np.uint32)
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    n = arrival.shape[0]
    hw = np.ascontiguousarray(hw, dtype=np.uint8)
    batch = np.ascontiguousarray(batch, dtype=np.uint8)
    replicas = np.ascontiguousarray(replicas, dtype=np.uint16)
    assert hw.shape == (S,) and batch.shape == (S,) and replicas.shape == (S,)
    latency = np.zeros(max(n, 1), dtype=np.uint64)
    ready = np.zeros((S, max(n, 1)), dtype=np.uint64) if want_stages else None
    done = np.zeros((S, max(n, 1)), dtype=np.uint64) if want_stages else None
    cap = S * max(n, 1) if want_batches else 0
    blog = np.zeros((max(cap, 1), 4), dtype=np.uint64) if want_batches else None
    nb = ctypes.c_uint64(0)
    rc = lib.oracle_simulate(
        ctypes.c_uint32(S), _p(off, ctypes.c_uint32), _p(idx, ctypes.c_uint32),
        ctypes.c_uint32(H), ctypes.c_uint32(Bmax), _p(lat_us, ctypes.c_uint32),
        ctypes.c_uint64(n), _p(arrival, ctypes.c_uint32), _p(mask, ctypes.c_uint32),
        _p(hw, ctypes.c_uint8), _p(batch, ctypes.c_uint8), _p(replicas, ctypes.c_uint16),
        ctypes.c_uint64(horizon), _p(latency, ctypes.c_uint64), _p(ready, ctypes.c_uint64),
        _p(done, ctypes.c_uint64), _p(blog, ctypes.c_uint64), ctypes.c_uint64(cap),
        ctypes.byref(nb))
    if rc != 0:
        raise ValueError("oracle_simulate failed with code %d" % rc)
    out = {"latency": latency[:n]}
    if want_stages:
        out["ready"] = ready[:, :n]
        out["done"] = done[:, :n]
    if want_batches:
        out["batches"] = blog[:nb.value]
    return out


def p99(latency):
    lib = _load()
    latency = np.ascontiguousarray(latency, dtype=np.uint64)
    return int(lib.oracle_p99(_p(latency, ctypes.c_uint64), ctypes.c_uint64(latency.shape[0])))


def run(parents, lat_us, cost_uusd_hr, arrival, mask, cfg_hw, cfg_batch, cfg_replicas, slo_us,
        horizon=HORIZON, want_latencies=False):
    """Many configurations, one after the other on one thread.
    cfg_* are [C][S].  Returns dict p99_us, miss_count, cost_uusd_hr (uint64[C]) and, on
    request, 'latency' (uint64[C][n])."""
    lib = _load()
    lat_us = np.ascontiguousarray(lat_us, dtype=np.uint32)
    S, H, Bmax = lat_us.shape
    cost = np.ascontiguousarray(cost_uusd_hr, dtype=np.uint64)
    assert cost.shape == (S, H)
    off, idx = _dag_arrays(parents)
    arrival = np.ascontiguousarray(arrival, dtype=np.uint32)
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    n = arrival.shape[0]
    hw = np.ascontiguousarray(cfg_hw, dtype=np.uint8)
    batch = np.ascontiguousarray(cfg_batch, dtype=np.uint8)
    replicas = np.ascontiguousarray(cfg_replicas, dtype=np.uint16)
    C = hw.shape[0]
    assert hw.shape == (C, S) and batch.shape == (C, S) and replicas.shape == (C, S)
    p99_us = np.zeros(max(C, 1), dtype=np.uint64)
    miss = np.zeros(max(C, 1), dtype=np.uint64)
    cost_out = np.zeros(max(C, 1), dtype=np.uint64)
    lat_all = np.zeros((max(C, 1), max(n, 1)), dtype=np.uint64) if want_latencies else None
    rc = lib.oracle_run(
        ctypes.c_uint32(S), _p(off, ctypes.c_uint32), _p(idx, ctypes.c_uint32),
        ctypes.c_uint32(H), ctypes.c_uint32(Bmax), _p(lat_us, ctypes.c_uint32),
        _p(cost, ctypes.c_uint64), ctypes.c_uint64(n), _p(arrival, ctypes.c_uint32),
        _p(mask, ctypes.c_uint32), ctypes.c_uint64(C), _p(hw, ctypes.c_uint8),
        _p(batch, ctypes.c_uint8), _p(replicas, ctypes.c_uint16), ctypes.c_uint64(slo_us),
        ctypes.c_uint64(horizon), _p(p99_us, ctypes.c_uint64), _p(miss, ctypes.c_uint64),
        _p(cost_out, ctypes.c_uint64), _p(lat_all, ctypes.c_uint64))
    if rc != 0:
        raise ValueError("oracle_run failed with code %d" % rc)
    out = {"p99_us": p99_us[:C], "miss_count": miss[:C], "cost_uusd_hr": cost_out[:C]}
    if want_latencies:
        out["latency"] = lat_all[:C, :n]
    return out
