"""Thin Python binding of the C ABI in include/themis.h.

Argument marshalling only: every step of the solve runs in the HIP library.
PyTorch supplies device buffers and the stream.  There is no CPU fallback: if
the library has not been built, importing the binding's functions raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libthemis_hip.so")

MAX_BATCH = 16
OK = 0
SOLVED, INFEASIBLE, INVALID, INTERNAL = 0, 1, 2, 3
ERR_NULL, ERR_SHAPE, ERR_BATCH, ERR_RANGE, ERR_WORKSPACE, ERR_LAUNCH = -1, -2, -3, -4, -5, -6
ERR_TOO_LARGE = -7
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "themis_version", "themis_check_problem", "themis_workspace_bytes",
    "themis_solve_joint", "themis_solve_joint_static", "themis_solve_vertical",
    "themis_solve_horizontal",
    "themis_fallback_workspace_bytes", "themis_solve_vertical_fallback",
    "themis_stability_workspace_bytes", "themis_check_stability",
    "themis_memo_workspace_bytes", "themis_solve_distinct",
    "themis_stage_candidates",
    "themis_stage_minplus", "themis_stage_backtrack", "themis_export_candidates",
    "themis_count_relaxations",
]


class ThemisProblem(ctypes.Structure):
    _fields_ = [
        ("n_inst", ctypes.c_int32), ("n_stage", ctypes.c_int32), ("c_max", ctypes.c_int32),
        ("n_batch", ctypes.c_int32), ("batch_sizes", ctypes.c_int32 * MAX_BATCH),
        ("r_max", ctypes.c_int32), ("tick_us", ctypes.c_int32),
        ("slo_max_us", ctypes.c_int32), ("coef_shared", ctypes.c_int32),
        ("queue_model", ctypes.c_int32), ("profile_form", ctypes.c_int32),
        ("prune", ctypes.c_int32), ("reserved", ctypes.c_int32 * 1),
    ]


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with "
                "`python -m paper_2407_14843_amd.build` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        P, vp, sz = ctypes.POINTER(ThemisProblem), ctypes.c_void_p, ctypes.c_size_t
        L.themis_version.restype = ctypes.c_int
        L.themis_version.argtypes = []
        L.themis_check_problem.restype = ctypes.c_int
        L.themis_check_problem.argtypes = [P]
        L.themis_workspace_bytes.restype = sz
        L.themis_workspace_bytes.argtypes = [P]
        L.themis_solve_joint.restype = ctypes.c_int
        L.themis_solve_joint.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.themis_solve_joint_static.restype = ctypes.c_int
        L.themis_solve_joint_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp]
        L.themis_solve_vertical.restype = ctypes.c_int
        L.themis_solve_vertical.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.themis_solve_horizontal.restype = ctypes.c_int
        L.themis_solve_horizontal.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.themis_fallback_workspace_bytes.restype = sz
        L.themis_fallback_workspace_bytes.argtypes = [P]
        L.themis_solve_vertical_fallback.restype = ctypes.c_int
        L.themis_solve_vertical_fallback.argtypes = (
            [P, vp, vp, vp, vp] + [vp] * 9 + [vp, sz, vp])
        L.themis_stability_workspace_bytes.restype = sz
        L.themis_stability_workspace_bytes.argtypes = [P]
        L.themis_check_stability.restype = ctypes.c_int
        L.themis_check_stability.argtypes = [P] + [vp] * 10 + [vp, sz, vp]
        L.themis_memo_workspace_bytes.restype = sz
        L.themis_memo_workspace_bytes.argtypes = [P]
        L.themis_solve_distinct.restype = ctypes.c_int
        L.themis_solve_distinct.argtypes = [P] + [vp] * 8 + [vp, sz, vp]
        L.themis_stage_candidates.restype = ctypes.c_int
        L.themis_stage_candidates.argtypes = [P, vp, vp, vp, vp, vp, sz, vp]
        L.themis_stage_minplus.restype = ctypes.c_int
        L.themis_stage_minplus.argtypes = [P, vp, sz, vp]
        L.themis_stage_backtrack.restype = ctypes.c_int
        L.themis_stage_backtrack.argtypes = [P, vp, vp, vp, vp, vp, sz, vp]
        L.themis_export_candidates.restype = ctypes.c_int
        L.themis_export_candidates.argtypes = [P, vp, sz, vp, vp, vp]
        L.themis_count_relaxations.restype = ctypes.c_int
        L.themis_count_relaxations.argtypes = [P, vp, sz, vp, vp]
        _lib = L
    return _lib


QUEUE_PER_REPLICA, QUEUE_SHARED, QUEUE_WORST_CASE = 0, 1, 2
PROFILE_5, PROFILE_EQ1 = 0, 1
PRUNE_NONE, PRUNE_DOMINATED, PRUNE_STEPS = 0, 1, 2


def make_problem(n_inst, n_stage, c_max, batch_sizes, r_max, tick_us, slo_max_us,
                 coef_shared=False, queue_model=0, profile_form=0, prune=0) -> ThemisProblem:
    p = ThemisProblem()
    p.n_inst, p.n_stage, p.c_max = int(n_inst), int(n_stage), int(c_max)
    p.n_batch = len(batch_sizes)
    for j, b in enumerate(list(batch_sizes)[:MAX_BATCH]):
        p.batch_sizes[j] = int(b)
    p.r_max, p.tick_us, p.slo_max_us = int(r_max), int(tick_us), int(slo_max_us)
    p.coef_shared = int(bool(coef_shared))
    p.queue_model, p.profile_form, p.prune = int(queue_model), int(profile_form), int(prune)
    return p


def check_problem(p: ThemisProblem) -> int:
    return lib().themis_check_problem(ctypes.byref(p))


def workspace_bytes(p: ThemisProblem) -> int:
    return int(lib().themis_workspace_bytes(ctypes.byref(p)))


def _dp(t: Optional[torch.Tensor], dtype=torch.int32):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class ThemisError(RuntimeError):
    def __init__(self, fn, rc):
        super().__init__(f"{fn} returned {rc}")
        self.rc = rc


def _chk(fn, rc):
    if rc != OK:
        raise ThemisError(fn, rc)


def alloc_workspace(p: ThemisProblem, device="cuda:0") -> torch.Tensor:
    n = workspace_bytes(p)
    if n == 0:
        raise ThemisError("themis_workspace_bytes", check_problem(p))
    return torch.empty(n, dtype=torch.uint8, device=device)


def alloc_outputs(p: ThemisProblem, device="cuda:0"):
    n, s = p.n_inst, p.n_stage
    return (torch.empty(n, dtype=torch.int32, device=device),
            torch.empty(n, dtype=torch.int32, device=device),
            torch.empty(n, dtype=torch.int32, device=device),
            torch.empty((n, s, 3), dtype=torch.int32, device=device))


def themis_solve_joint(p, coef, lam, slo_us, status, cost, ticks, cfg, workspace, stream=None):
    _chk("themis_solve_joint", lib().themis_solve_joint(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(status), _dp(cost), _dp(ticks),
        _dp(cfg), _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def themis_solve_joint_static(p, coef, lam, slo_us, status, cost, ticks, cfg, stream=None):
    _chk("themis_solve_joint_static", lib().themis_solve_joint_static(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(status), _dp(cost), _dp(ticks),
        _dp(cfg), _stream(stream)))


def themis_solve_vertical(p, coef, lam, slo_us, r_fixed, status, cost, ticks, cfg, workspace,
                          stream=None):
    _chk("themis_solve_vertical", lib().themis_solve_vertical(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(r_fixed), _dp(status),
        _dp(cost), _dp(ticks), _dp(cfg), _dp(workspace, torch.uint8), workspace.numel(),
        _stream(stream)))


def themis_solve_horizontal(p, coef, lam, slo_us, cores, status, cost, ticks, cfg, workspace,
                            stream=None):
    _chk("themis_solve_horizontal", lib().themis_solve_horizontal(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(cores), _dp(status),
        _dp(cost), _dp(ticks), _dp(cfg), _dp(workspace, torch.uint8), workspace.numel(),
        _stream(stream)))


def fallback_workspace_bytes(p: ThemisProblem) -> int:
    return int(lib().themis_fallback_workspace_bytes(ctypes.byref(p)))


def themis_solve_vertical_fallback(p, coef, lam, slo_us, r_fixed, status, cost,
                                   ticks, cfg, lambda_v, status_h, cost_h, ticks_h, cfg_h,
                                   workspace, stream=None):
    _chk("themis_solve_vertical_fallback", lib().themis_solve_vertical_fallback(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(r_fixed),
        _dp(status), _dp(cost), _dp(ticks), _dp(cfg), _dp(lambda_v), _dp(status_h),
        _dp(cost_h), _dp(ticks_h), _dp(cfg_h), _dp(workspace, torch.uint8),
        workspace.numel(), _stream(stream)))


def stability_workspace_bytes(p: ThemisProblem) -> int:
    return int(lib().themis_stability_workspace_bytes(ctypes.byref(p)))


def themis_check_stability(p, coef, lam_now, lam_pred, slo_us, cores, stable, status, cost,
                           ticks, cfg, workspace, stream=None):
    _chk("themis_check_stability", lib().themis_check_stability(
        ctypes.byref(p), _dp(coef), _dp(lam_now), _dp(lam_pred), _dp(slo_us), _dp(cores),
        _dp(stable), _dp(status), _dp(cost), _dp(ticks), _dp(cfg),
        _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def memo_workspace_bytes(p: ThemisProblem) -> int:
    return int(lib().themis_memo_workspace_bytes(ctypes.byref(p)))


def themis_solve_distinct(p, coef, lam, slo_us, r_fixed, status, cost, ticks, cfg, workspace,
                          stream=None):
    _chk("themis_solve_distinct", lib().themis_solve_distinct(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(r_fixed), _dp(status), _dp(cost),
        _dp(ticks), _dp(cfg), _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def themis_stage_candidates(p, coef, lam, slo_us, r_fixed, workspace, stream=None):
    _chk("themis_stage_candidates", lib().themis_stage_candidates(
        ctypes.byref(p), _dp(coef), _dp(lam), _dp(slo_us), _dp(r_fixed),
        _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def themis_stage_minplus(p, workspace, stream=None):
    _chk("themis_stage_minplus", lib().themis_stage_minplus(
        ctypes.byref(p), _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def themis_stage_backtrack(p, status, cost, ticks, cfg, workspace, stream=None):
    _chk("themis_stage_backtrack", lib().themis_stage_backtrack(
        ctypes.byref(p), _dp(status), _dp(cost), _dp(ticks), _dp(cfg),
        _dp(workspace, torch.uint8), workspace.numel(), _stream(stream)))


def themis_export_candidates(p, workspace, lt, cost, stream=None):
    _chk("themis_export_candidates", lib().themis_export_candidates(
        ctypes.byref(p), _dp(workspace, torch.uint8), workspace.numel(), _dp(lt), _dp(cost),
        _stream(stream)))


def themis_count_relaxations(p, workspace, count, stream=None):
    if count.numel() < 3:
        raise ValueError("count takes three values: relaxations, table entries, cells formed")
    _chk("themis_count_relaxations", lib().themis_count_relaxations(
        ctypes.byref(p), _dp(workspace, torch.uint8), workspace.numel(),
        _dp(count, torch.int64), _stream(stream)))


# ---------------------------------------------------------------- conveniences
def problem_of(w, prune=0) -> ThemisProblem:
    """Problem description of a workloads.Workload."""
    return make_problem(w.n_inst, w.n_stage, w.c_max, w.batch_sizes, w.r_max, w.tick_us,
                        w.slo_max_us, w.coef_shared, w.queue_model, w.profile_form, prune)


class DeviceBatch:
    """A workload's arrays resident in HBM plus output and workspace buffers."""

    def __init__(self, w, device="cuda:0", prune=0):
        self.w = w
        self.p = problem_of(w, prune)
        self.device = device
        to = lambda a: None if a is None else torch.from_numpy(a).to(device).contiguous()
        self.coef, self.lam, self.slo_us, self.r_fixed = (
            to(w.coef), to(w.lam), to(w.slo_us), to(w.r_fixed))
        self.status, self.cost, self.ticks, self.cfg = alloc_outputs(self.p, device)
        self.workspace = alloc_workspace(self.p, device)

    def solve(self, stream=None):
        """Enqueue the whole solve; does not synchronise."""
        if self.r_fixed is None:
            themis_solve_joint(self.p, self.coef, self.lam, self.slo_us, self.status,
                               self.cost, self.ticks, self.cfg, self.workspace, stream)
        else:
            themis_solve_vertical(self.p, self.coef, self.lam, self.slo_us, self.r_fixed,
                                  self.status, self.cost, self.ticks, self.cfg,
                                  self.workspace, stream)

    def solve_distinct(self, stream=None):
        """Enqueue the solve that handles every distinct instance once (same outputs)."""
        if getattr(self, "memo_workspace", None) is None:
            self.memo_workspace = torch.empty(memo_workspace_bytes(self.p), dtype=torch.uint8,
                                              device=self.device)
        themis_solve_distinct(self.p, self.coef, self.lam, self.slo_us, self.r_fixed, self.status,
                              self.cost, self.ticks, self.cfg, self.memo_workspace, stream)

    def solve_horizontal(self, cores=None, stream=None):
        """Enqueue the horizontal-only solve (cores: numpy int [N][S] or None = one core)."""
        self.cores = None if cores is None else torch.from_numpy(
            cores.astype("int32")).to(self.device).contiguous()
        themis_solve_horizontal(self.p, self.coef, self.lam, self.slo_us, self.cores,
                                self.status, self.cost, self.ticks, self.cfg, self.workspace,
                                stream)

    def check_stability(self, lam_pred, cores=None, stream=None):
        """Enqueue the stability test; returns the device tensor of flags."""
        to = lambda a: None if a is None else torch.from_numpy(
            a.astype("int32")).to(self.device).contiguous()
        self.lam_pred, self.cores = to(lam_pred), to(cores)
        ws = torch.empty(stability_workspace_bytes(self.p), dtype=torch.uint8,
                         device=self.device)
        self.stable = torch.empty(self.p.n_inst, dtype=torch.int32, device=self.device)
        themis_check_stability(self.p, self.coef, self.lam, self.lam_pred, self.slo_us,
                               self.cores, self.stable, self.status, self.cost, self.ticks,
                               self.cfg, ws, stream)
        self.stability_workspace = ws
        return self.stable

    def solve_vertical_fallback(self, stream=None):
        """Enqueue the vertical solve with fallback; results via fallback_results()."""
        if getattr(self, "fb", None) is None:
            n = fallback_workspace_bytes(self.p)
            self.fb_workspace = torch.empty(n, dtype=torch.uint8, device=self.device)
            self.lambda_v = torch.empty(self.p.n_inst, dtype=torch.int32, device=self.device)
            self.fb = alloc_outputs(self.p, self.device)
        themis_solve_vertical_fallback(self.p, self.coef, self.lam, self.slo_us, self.r_fixed,
                                       self.status, self.cost, self.ticks, self.cfg,
                                       self.lambda_v, *self.fb, self.fb_workspace, stream)

    def fallback_results(self):
        torch.cuda.synchronize()
        names = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h",
                 "cfg_h")
        bufs = (self.status, self.cost, self.ticks, self.cfg, self.lambda_v) + tuple(self.fb)
        return {k: b.cpu().numpy() for k, b in zip(names, bufs)}

    def results(self):
        torch.cuda.synchronize()
        return (self.status.cpu().numpy(), self.cost.cpu().numpy(),
                self.ticks.cpu().numpy(), self.cfg.cpu().numpy())

    def candidates(self):
        """Run stage 1 alone and return its (lt, cost) tables as numpy arrays."""
        themis_stage_candidates(self.p, self.coef, self.lam, self.slo_us, self.r_fixed,
                                self.workspace)
        shape = (self.p.n_inst, self.p.n_stage, self.w.n_cand)
        lt = torch.empty(shape, dtype=torch.int32, device=self.device)
        co = torch.empty(shape, dtype=torch.int32, device=self.device)
        themis_export_candidates(self.p, self.workspace, lt, co)
        torch.cuda.synchronize()
        return lt.cpu().numpy(), co.cpu().numpy()
