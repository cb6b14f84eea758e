"""GPU parity of the min-plus stage with rows kept as step functions
(THEMIS_PRUNE_STEPS), alone and combined with pruning of dominated candidates:
the answers must be the CPU checker's, bit for bit, and so must the rows it
leaves for the reconstruction (checked through the reconstruction itself:
the checker's configurations are only reproduced from exact rows).
"""

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

pytestmark = pytest.mark.gpu

NAMES = ("status", "cost", "ticks", "cfg")


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_14843_amd import themis
    themis.lib()
    return themis


def same(got, want, names=NAMES):
    for name, g, e in zip(names, got, want):
        assert np.array_equal(g, e), f"{name} differs: {int((g != e).sum())} entries"


@pytest.mark.parametrize("prune", [2, 3])
@pytest.mark.parametrize("idx,n", [(0, 64), (1, 300), (2, 120), (3, 100), (4, 200)])
def test_step_rows_match_checker(T, oracle, idx, n, prune):
    w = wl.workload(idx, n)
    if idx == 4:
        rng = np.random.default_rng(4)
        w = w.with_r_fixed(rng.integers(1, 6, size=(w.n_inst, w.n_stage)))
    print(f"[case] step rows workload {idx} N={n} prune={prune}", flush=True)
    b = T.DeviceBatch(w, prune=prune)
    b.solve()
    same(b.results(), oracle.solve(w, threads=8))


def test_step_rows_tiny_random(T, oracle):
    """Shapes of every kind: one model (answer from the starting row), two
    (no row between), budgets of a few ticks, infeasible and invalid ones."""
    rng = np.random.default_rng(31)
    kinds = np.zeros(3, int)
    for rep in range(60):
        w = wl.tiny_random(rng, int(rng.integers(0, 2)), n_inst=int(rng.integers(1, 70)),
                           max_stage=int(rng.integers(1, 6)))
        if w.slo_max_us // w.tick_us > 32767:
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        if rep % 7 == 0:
            w.lam[0] = 0                                   # an invalid instance
        prune = 2 + rep % 2
        print(f"[case] step rows tiny rep {rep} K={w.n_cand} S={w.n_stage} prune={prune}",
              flush=True)
        b = T.DeviceBatch(w, prune=prune)
        b.solve()
        want = oracle.solve(w)
        same(b.results(), want)
        kinds += [(want[0] == 0).sum(), (want[0] == 1).sum(), (want[0] == 2).sum()]
    assert (kinds > 0).all(), kinds


def test_step_rows_long_lists_and_many_candidates(T, oracle):
    """Costs that make rows drop at very many budgets (more than the list in LDS
    holds, so the threads scatter from their own stretches), and a model with
    more candidates than are staged at a time."""
    rng = np.random.default_rng(8)
    n, S = 6, 3
    # many cores and replicas with a fine tick: cost steps nearly every tick
    coef = np.stack([rng.integers(lo, hi + 1, size=(n, S)) for lo, hi in
                     ((200_000, 900_000), (1000, 5000), (0, 3), (64, 64), (200, 2000))],
                    axis=-1).astype(np.int32)
    w = wl.Workload("steps-long", wl.JOINT, n, S, 64, [1, 2, 3, 4, 6, 8, 12, 16, 24, 32], 150, 20,
                    300_000, False, coef, rng.integers(50, 4000, n).astype(np.int32),
                    rng.integers(200_000, 300_001, n).astype(np.int32))
    for prune in (2, 3):
        print(f"[case] step rows long lists prune={prune} K={w.n_cand}", flush=True)
        b = T.DeviceBatch(w, prune=prune)
        b.solve()
        want = oracle.solve(w, threads=6)
        same(b.results(), want)
        assert (want[0] == 0).any()


def test_step_rows_other_entry_points(T, oracle):
    w = wl.workload(2, 60)
    rng = np.random.default_rng(12)
    w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 6, w.n_inst),
                       1 << 20).astype(np.int32)
    want = oracle.vertical_fallback(w, threads=8)
    print("[case] step rows fallback", flush=True)
    b = T.DeviceBatch(w, prune=2)
    b.solve_vertical_fallback()
    got = b.fallback_results()
    keys = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h", "cfg_h")
    same([got[k] for k in keys], [want[k] for k in keys], keys)
    j = wl.workload(1, 120)
    pred = np.clip(j.lam.astype(np.int64) + rng.integers(-50, 80, j.n_inst), 1, 1 << 20).astype(
        np.int32)
    print("[case] step rows stability", flush=True)
    bj = T.DeviceBatch(j, prune=3)
    st = bj.check_stability(pred)
    same((st.cpu().numpy(),) + bj.results(), oracle.stability(j, pred),
         ("stable",) + NAMES)


@pytest.mark.parametrize("idx,k", [(1, 4096), (3, 300)])
def test_step_rows_full_size(T, oracle, idx, k):
    """Full batch in the launch configuration the benchmark times; the checker
    covers a sample of instances."""
    w = wl.workload(idx)
    print(f"[case] step rows full workload {idx} N={w.n_inst}", flush=True)
    b = T.DeviceBatch(w, prune=2)
    b.solve()
    got = b.results()
    rng = np.random.default_rng(idx)
    pick = np.sort(rng.choice(w.n_inst, size=min(k, w.n_inst), replace=False))
    want = oracle.solve(w.take(pick), threads=16)
    same([g[pick] for g in got], want)
