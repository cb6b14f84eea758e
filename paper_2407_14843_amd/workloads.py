"""Seeded synthetic workloads for the batched autoscaling solve.

This module only draws random integers and packs them into arrays.  It holds
none of the solver's arithmetic (no latency model, no queue delay, no DP), so
both the CPU checker and the GPU library can be fed from it without sharing
any method code.

A workload is a batch of independent instances.  Every instance is one
inference pipeline (a chain of `n_stage` models) observed at one arrival rate
`lam` (requests/s) under one end-to-end latency objective `slo_us`.  Each stage
carries five integer profile coefficients `(a, k, q, p, o)`: they stand in for
the fitted per-model latency profile of Section 4.1 (Eq. 1), which needs the
real models to measure, with `p` the number of cores beyond which a model no
longer speeds up (the hardware/parallelism limit discussed in Section 2).

The five numbered workloads stand in for the paper's trace-driven evaluation
(Section 6: Twitter-trace arrival rates, seven profiled models, pipelines of
two or three stages, SLOs of roughly one to two and a half seconds); neither
the trace nor the models are available offline, so arrival rates, SLOs and
profile coefficients are drawn from the stated ranges instead.
"""

from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

BASE_SEED = 240714843

JOINT = 0
VERTICAL = 1


@dataclass
class Workload:
    """One batch of instances plus the search-space bounds shared by all."""

    name: str
    variant: int                 # JOINT or VERTICAL
    n_inst: int
    n_stage: int
    c_max: int                   # cores per replica range over 1..c_max
    batch_sizes: List[int]       # strictly increasing
    r_max: int                   # replicas range over 1..r_max
    tick_us: int                 # latency-grid resolution
    slo_max_us: int              # upper bound on every slo_us entry
    coef_shared: bool            # True: coef is [S][5]; False: [N][S][5]
    coef: np.ndarray             # int32, order (a, k, q, p, o)
    lam: np.ndarray              # int32 [N]
    slo_us: np.ndarray           # int32 [N]
    r_fixed: Optional[np.ndarray] = None   # int32 [N][S], vertical only
    queue_model: int = 0         # 0 batch fill per replica, 1 Eq. 4, 2 Eq. 3
    profile_form: int = 0        # 0: coefficients (a,k,q,p,o); 1: (a,k,q,p,o,d), Eq. 1's delta
    seed: int = 0
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_cand(self) -> int:
        return self.c_max * len(self.batch_sizes)

    def head(self, n: int) -> "Workload":
        """The first `n` instances (same values as in the full batch)."""
        n = min(n, self.n_inst)
        return self.take(np.arange(n))

    def take(self, idx) -> "Workload":
        """The instances listed in `idx`, in that order."""
        idx = np.asarray(idx, dtype=np.int64)
        return replace(
            self,
            n_inst=int(idx.size),
            coef=self.coef if self.coef_shared else np.ascontiguousarray(self.coef[idx]),
            lam=np.ascontiguousarray(self.lam[idx]),
            slo_us=np.ascontiguousarray(self.slo_us[idx]),
            r_fixed=None if self.r_fixed is None else np.ascontiguousarray(self.r_fixed[idx]),
        )

    def with_r_fixed(self, r_fixed: np.ndarray, r_max: Optional[int] = None) -> "Workload":
        """The same instances as a vertical-only batch with the given replicas."""
        r_fixed = np.ascontiguousarray(r_fixed, dtype=np.int32)
        assert r_fixed.shape == (self.n_inst, self.n_stage)
        return replace(self, variant=VERTICAL, r_fixed=r_fixed,
                       r_max=self.r_max if r_max is None else r_max)


    def with_model(self, queue_model: int = 0, d: Optional[np.ndarray] = None) -> "Workload":
        """The same instances under another queue model and, when `d` is given
        (int array shaped like coef without its last axis), with that sixth
        profile coefficient appended."""
        coef, form = self.coef, self.profile_form
        if d is not None:
            assert form == 0 and d.shape == coef.shape[:-1]
            coef = np.ascontiguousarray(
                np.concatenate([coef, np.asarray(d, np.int32)[..., None]], axis=-1))
            form = 1
        return replace(self, coef=coef, queue_model=queue_model, profile_form=form)


def _pow2_upto(bmax: int) -> List[int]:
    out, b = [], 1
    while b <= bmax:
        out.append(b)
        b *= 2
    return out


def _draw_coef(rng, shape_prefix, a, k, q, p, o):
    """Independent inclusive-uniform integer draws, one column per coefficient."""
    cols = [rng.integers(lo, hi + 1, size=shape_prefix, dtype=np.int64)
            for (lo, hi) in (a, k, q, p, o)]
    return np.ascontiguousarray(np.stack(cols, axis=-1).astype(np.int32))


_BASE_RANGES = dict(a=(2000, 20000), k=(500, 5000), q=(0, 50), o=(100, 1000))


def workload(idx: int, n_inst: Optional[int] = None) -> Workload:
    """Build numbered workload `idx` (0..4).

    The draw order inside each workload is fixed (coefficients, then arrival
    rates, then SLOs, then fixed replicas) so that a given index always yields
    the same arrays.  `n_inst` keeps only the first instances of the full batch.
    """
    seed = BASE_SEED + idx
    rng = np.random.default_rng(seed)
    if idx == 0:
        N, S = 64, 3
        coef = _draw_coef(rng, (N, S), p=(2, 8), **_BASE_RANGES)
        lam = rng.integers(10, 200 + 1, size=N)
        slo_ms = rng.integers(50, 300 + 1, size=N)
        w = Workload("w0-joint-64x3", JOINT, N, S, 8, _pow2_upto(16), 8, 1000,
                     300_000, False, coef, lam.astype(np.int32),
                     (slo_ms * 1000).astype(np.int32), seed=seed)
    elif idx == 1:
        N, S = 4096, 5
        coef = _draw_coef(rng, (N, S), p=(4, 16), **_BASE_RANGES)
        lam = rng.integers(10, 1000 + 1, size=N)
        slo_ms = rng.integers(100, 1000 + 1, size=N)
        w = Workload("w1-joint-4096x5", JOINT, N, S, 16, _pow2_upto(64), 32, 250,
                     1_000_000, False, coef, lam.astype(np.int32),
                     (slo_ms * 1000).astype(np.int32), seed=seed)
    elif idx == 2:
        N, S = 16384, 8
        coef = _draw_coef(rng, (N, S), p=(8, 32), **_BASE_RANGES)
        lam = rng.integers(50, 2000 + 1, size=N)
        slo_ms = rng.integers(200, 2000 + 1, size=N)
        r_fixed = rng.integers(1, 4 + 1, size=(N, S)).astype(np.int32)
        w = Workload("w2-vertical-16384x8", VERTICAL, N, S, 32, _pow2_upto(128), 4, 250,
                     2_000_000, False, coef, lam.astype(np.int32),
                     (slo_ms * 1000).astype(np.int32), r_fixed=r_fixed, seed=seed)
    elif idx == 3:
        N, S = 65536, 8
        coef = _draw_coef(rng, (N, S), a=(4000, 40000), k=(1000, 10000), q=(0, 100),
                          p=(4, 16), o=(200, 2000))
        u = rng.random(size=N)
        lam = np.clip(np.rint(10.0 * np.power(500.0, u)), 10, 5000).astype(np.int64)
        slo_ms = rng.integers(200, 4000 + 1, size=N)
        w = Workload("w3-joint-65536x8", JOINT, N, S, 32, _pow2_upto(128), 64, 250,
                     4_000_000, False, coef, lam.astype(np.int32),
                     (slo_ms * 1000).astype(np.int32), seed=seed)
    elif idx == 4:
        N, S = 86400, 6
        coef = _draw_coef(rng, (S,), p=(4, 16), **_BASE_RANGES)
        # Two-state Markov-modulated Poisson arrivals, one sample per second.
        switch = rng.random(size=N) < 0.002
        state = np.zeros(N, dtype=np.int64)
        cur = 0
        for t in range(N):
            if t > 0 and switch[t]:
                cur ^= 1
            state[t] = cur
        means = np.array([50.0, 800.0])
        lam = np.maximum(1, rng.poisson(means[state])).astype(np.int64)
        slo = np.full(N, 500_000, dtype=np.int64)
        w = Workload("w4-trace-86400x6", JOINT, N, S, 16, _pow2_upto(64), 48, 250,
                     500_000, True, coef, lam.astype(np.int32), slo.astype(np.int32),
                     seed=seed, extra={"state": state})
    else:
        raise ValueError(f"no workload {idx}")
    if n_inst is not None:
        w = w.head(n_inst)
    return w


def replicas_carried_forward(status: np.ndarray, cfg: np.ndarray) -> np.ndarray:
    """Replica counts a vertical-only solve at second t inherits (workload 4).

    Second t runs on whatever the last successful joint decision before it
    deployed: the replicas of second t-1's joint result if that solve found a
    configuration, otherwise whatever second t-1 itself was running on.  The
    first second starts from one replica per stage.  `cfg` is [N][S][3] with the
    replica count in the last column; `status` is 0 where a solve succeeded.
    Pure bookkeeping on solver outputs: no model arithmetic.
    """
    n, s = cfg.shape[0], cfg.shape[1]
    out = np.ones((n, s), dtype=np.int32)
    for t in range(1, n):
        out[t] = cfg[t - 1, :, 2] if status[t - 1] == 0 else out[t - 1]
    return out


def tiny_random(rng: np.random.Generator, variant: int = JOINT, n_inst: int = 1,
                max_stage: int = 4) -> Workload:
    """A tiny random batch whose whole configuration space can be enumerated."""
    S = int(rng.integers(1, max_stage + 1))
    c_max = int(rng.integers(1, 4 + 1))
    nb = int(rng.integers(1, 3 + 1))
    pool = [1, 2, 3, 4, 6, 8]
    bs = sorted(rng.choice(len(pool), size=nb, replace=False).tolist())
    batch_sizes = [pool[j] for j in bs]
    r_max = int(rng.integers(1, 4 + 1))
    tick = int(rng.choice([1, 7, 250, 1000, 3000]))
    coef = _draw_coef(rng, (n_inst, S), a=(0, 20000), k=(0, 5000), q=(0, 50),
                      p=(1, 5), o=(1, 1000))
    lam = rng.integers(1, 300 + 1, size=n_inst).astype(np.int32)
    slo_us = rng.integers(0, 120_000 + 1, size=n_inst).astype(np.int32)
    r_fixed = None
    if variant == VERTICAL:
        r_fixed = rng.integers(1, r_max + 1, size=(n_inst, S)).astype(np.int32)
    return Workload("tiny", variant, n_inst, S, c_max, batch_sizes, r_max, tick,
                    120_000, False, coef, lam, slo_us, r_fixed=r_fixed)


def medium_random(rng: np.random.Generator, variant: int = JOINT) -> Workload:
    """A random batch with a search space of realistic size (up to 32 cores x 8
    batch sizes, up to 9000 grid cells, up to 5 models) that the CPU checker still
    solves in a fraction of a second; every shape parameter is drawn, with no
    regard to what a solver accepts (S * r_max * c_max can exceed a 16-bit total)."""
    n = int(rng.integers(1, 40))
    S = int(rng.integers(1, 6))
    c_max = int(rng.integers(1, 33))
    batch_sizes = sorted(set(int(x) for x in rng.integers(1, 129, int(rng.integers(1, 9)))))
    r_max = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 64, 100, 250, 1000]))
    tick = int(rng.choice([100, 250, 500, 1000]))
    slo_max = int(rng.integers(1, 9000)) * tick
    coef = _draw_coef(rng, (n, S), a=(1000, 40000), k=(100, 10000), q=(0, 100), p=(1, 40),
                      o=(1, 2000))
    lam = rng.integers(1, 6000, n).astype(np.int32)
    slo_us = rng.integers(0, slo_max + 1, n).astype(np.int32)
    r_fixed = None
    if variant == VERTICAL:
        r_fixed = rng.integers(1, r_max + 1, size=(n, S)).astype(np.int32)
    return Workload("medium", variant, n, S, c_max, batch_sizes, r_max, tick, slo_max, False,
                    coef, lam, slo_us, r_fixed=r_fixed)
