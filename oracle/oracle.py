"""ctypes front end of the CPU checker -- TEST INFRASTRUCTURE ONLY.

Loads `libthemis_oracle.so` (built from the two C files in this directory by
`build()`) and marshals numpy arrays.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this module; the GPU library never
does and shares nothing with it.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libthemis_oracle.so")
_SOURCES = [os.path.join(_HERE, f) for f in ("themis_oracle.c", "themis_bruteforce.c")]
_lib = None


def build(force: bool = True) -> str:
    """Compile the checker with gcc (-O2, no intrinsics, single-threaded code)."""
    if not force and os.path.exists(_LIB_PATH):
        newest = max(os.path.getmtime(s) for s in _SOURCES)
        if os.path.getmtime(_LIB_PATH) >= newest:
            return _LIB_PATH
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared",
           "-o", _LIB_PATH] + _SOURCES
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB_PATH)
        i32, p = ctypes.c_int32, ctypes.c_void_p
        _lib.themis_oracle_candidates.restype = ctypes.c_int
        _lib.themis_oracle_candidates.argtypes = [i32, i32, i32, p, i32, i32, i32, i32,
                                                  p, p, p, p, i32, i32, p, p, p]
        _lib.themis_oracle_solve.restype = ctypes.c_int
        _lib.themis_oracle_solve.argtypes = [i32, i32, i32, p, i32, i32, i32, i32,
                                             p, p, p, p, i32, i32, p, p, p, p]
        _lib.themis_oracle_solve_ex.restype = ctypes.c_int
        _lib.themis_oracle_solve_ex.argtypes = [i32, i32, i32, p, i32, i32, i32, i32,
                                                p, p, p, p, p, i32, i32, p, p, p, p]
        _lib.themis_oracle_vertical_fallback.restype = ctypes.c_int
        _lib.themis_oracle_vertical_fallback.argtypes = [i32, i32, i32, p, i32, i32, i32, i32,
                                                         p, p, p, p, i32, i32,
                                                         p, p, p, p, p, p, p, p, p]
        _lib.themis_oracle_stability.restype = ctypes.c_int
        _lib.themis_oracle_stability.argtypes = [i32, i32, i32, p, i32, i32, i32, i32,
                                                 p, p, p, p, p, i32, i32, p, p, p, p, p]
        _lib.themis_bruteforce_ex.restype = ctypes.c_int
        _lib.themis_bruteforce_ex.argtypes = [i32, i32, i32, p, i32, i32, p, i32, i32, p, p,
                                              p, p, p, p]
        _lib.themis_bruteforce.restype = ctypes.c_int
        _lib.themis_bruteforce.argtypes = [i32, i32, i32, p, i32, i32, p, i32, i32, p,
                                           p, p, p, p]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _common(w):
    # model options are process-wide in the C files: set them for this call
    qm, pf = int(getattr(w, "queue_model", 0)), int(getattr(w, "profile_form", 0))
    if _load().themis_oracle_set_model(qm, pf) or _load().themis_bruteforce_set_model(qm, pf):
        raise ValueError(f"unknown model options {qm}, {pf}")
    assert w.coef.shape[-1] == (6 if pf else 5)
    bs = np.asarray(w.batch_sizes, dtype=np.int32)
    return bs, _i32(w.coef), _i32(w.lam), _i32(w.slo_us), _i32(w.r_fixed)


def candidates(w):
    """Candidate tables (lt, cost, r), each int32 [N][S][K]; -1 marks infeasible."""
    lib = _load()
    bs, coef, lam, slo, rf = _common(w)
    shape = (w.n_inst, w.n_stage, w.n_cand)
    lt = np.empty(shape, np.int32)
    cost = np.empty(shape, np.int32)
    r = np.empty(shape, np.int32)
    rc = lib.themis_oracle_candidates(w.n_stage, w.c_max, len(bs), _ptr(bs), w.r_max,
                                      w.tick_us, w.slo_max_us, int(w.coef_shared),
                                      _ptr(coef), _ptr(lam), _ptr(slo), _ptr(rf),
                                      0, w.n_inst, _ptr(lt), _ptr(cost), _ptr(r))
    if rc != 0:
        raise RuntimeError(f"themis_oracle_candidates failed: {rc}")
    return lt, cost, r


def solve(w, threads: int = 1, c_fixed=None):
    """Solve every instance; returns (status[N], cost[N], ticks[N], cfg[N][S][3]).

    `threads` > 1 only shards the instance range over a thread pool; each
    shard runs the same single-threaded C routine.  `c_fixed` (int [N][S])
    pins each model's cores.
    """
    lib = _load()
    bs, coef, lam, slo, rf = _common(w)
    cfx = _i32(c_fixed)
    n, s = w.n_inst, w.n_stage
    status = np.empty(n, np.int32)
    cost = np.empty(n, np.int32)
    ticks = np.empty(n, np.int32)
    cfg = np.empty((n, s, 3), np.int32)

    def run(lo, hi):
        rc = lib.themis_oracle_solve_ex(s, w.c_max, len(bs), _ptr(bs), w.r_max, w.tick_us,
                                        w.slo_max_us, int(w.coef_shared), _ptr(coef),
                                        _ptr(lam), _ptr(slo), _ptr(rf), _ptr(cfx), lo, hi,
                                        _ptr(status[lo:]), _ptr(cost[lo:]),
                                        _ptr(ticks[lo:]), _ptr(cfg[lo:]))
        if rc != 0:
            raise RuntimeError(f"themis_oracle_solve failed: {rc}")

    threads = max(1, min(threads, n))
    if threads == 1:
        run(0, n)
    else:
        # small shards so that uneven instances still balance
        step = max(1, n // (threads * 16))
        spans = [(lo, min(n, lo + step)) for lo in range(0, n, step)]
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(lambda ab: run(*ab), spans))
    return status, cost, ticks, cfg


def vertical_fallback(w, threads: int = 1):
    """Algorithm 1 with its fallback for every instance of a vertical workload.

    Returns a dict of int32 arrays: status, cost, ticks, cfg (vertical part at
    lambda_v), lambda_v, status_h, cost_h, ticks_h, cfg_h (new instances for the
    remaining lambda - lambda_v, cores pinned to the vertical part's).
    """
    lib = _load()
    bs, coef, lam, slo, rf = _common(w)
    if rf is None:
        raise ValueError("vertical_fallback needs r_fixed")
    n, s = w.n_inst, w.n_stage
    out = {k: np.empty(n, np.int32) for k in
           ("status", "cost", "ticks", "lambda_v", "status_h", "cost_h", "ticks_h")}
    out["cfg"] = np.empty((n, s, 3), np.int32)
    out["cfg_h"] = np.empty((n, s, 3), np.int32)

    def run(lo, hi):
        rc = lib.themis_oracle_vertical_fallback(
            s, w.c_max, len(bs), _ptr(bs), w.r_max, w.tick_us, w.slo_max_us,
            int(w.coef_shared), _ptr(coef), _ptr(lam), _ptr(slo), _ptr(rf), lo, hi,
            _ptr(out["status"][lo:]), _ptr(out["cost"][lo:]), _ptr(out["ticks"][lo:]),
            _ptr(out["cfg"][lo:]), _ptr(out["lambda_v"][lo:]), _ptr(out["status_h"][lo:]),
            _ptr(out["cost_h"][lo:]), _ptr(out["ticks_h"][lo:]), _ptr(out["cfg_h"][lo:]))
        if rc != 0:
            raise RuntimeError(f"themis_oracle_vertical_fallback failed: {rc}")

    threads = max(1, min(threads, n))
    if threads == 1:
        run(0, n)
    else:
        step = max(1, n // (threads * 16))
        spans = [(lo, min(n, lo + step)) for lo in range(0, n, step)]
        with ThreadPoolExecutor(threads) as pool:
            list(pool.map(lambda ab: run(*ab), spans))
    return out


def stability(w, lam_pred, cores=None):
    """Section 5.1.3's stability test for every instance of a joint workload.

    Returns (stable[N], status[N], cost[N], ticks[N], cfg[N][S][3]); the last
    four are the horizontal solve at the current rate w.lam."""
    lib = _load()
    bs, coef, lam, slo, _ = _common(w)
    n, s = w.n_inst, w.n_stage
    lp, cx = _i32(lam_pred), _i32(cores)
    stable, status, cost, ticks = (np.empty(n, np.int32) for _ in range(4))
    cfg = np.empty((n, s, 3), np.int32)
    rc = lib.themis_oracle_stability(s, w.c_max, len(bs), _ptr(bs), w.r_max, w.tick_us,
                                     w.slo_max_us, int(w.coef_shared), _ptr(coef), _ptr(lam),
                                     _ptr(lp), _ptr(slo), _ptr(cx), 0, n, _ptr(stable),
                                     _ptr(status), _ptr(cost), _ptr(ticks), _ptr(cfg))
    if rc != 0:
        raise RuntimeError(f"themis_oracle_stability failed: {rc}")
    return stable, status, cost, ticks, cfg


def bruteforce(w, i: int = 0, c_fixed=None):
    """Exhaustive enumeration for instance i: (status, cost, ticks, cfg[S][3], visited).

    `c_fixed` (int [S]) pins the cores of each model."""
    lib = _load()
    bs, coef, lam, slo, rf = _common(w)
    cf = coef if w.coef_shared else coef[i]
    cf = np.ascontiguousarray(cf)
    rfi = None if rf is None else np.ascontiguousarray(rf[i])
    cost = ctypes.c_int32(0)
    ticks = ctypes.c_int32(0)
    visited = ctypes.c_int64(0)
    cfg = np.zeros((w.n_stage, 3), np.int32)
    cfx = _i32(c_fixed)
    rc = lib.themis_bruteforce_ex(w.n_stage, w.c_max, len(bs), _ptr(bs), w.r_max, w.tick_us,
                               _ptr(cf), int(lam[i]), int(slo[i]), _ptr(rfi), _ptr(cfx),
                               ctypes.byref(cost), ctypes.byref(ticks), _ptr(cfg),
                               ctypes.byref(visited))
    if rc < 0:
        raise RuntimeError(f"themis_bruteforce failed: {rc}")
    return rc, cost.value, ticks.value, cfg, visited.value
