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


def _drops_per_row(w, lt, cost, i):
    """Budgets at which each row f[s][.] of instance i drops, s = S-1 .. 0, from the
    checker's candidate tables by the recurrence as defined (test helper)."""
    T, inf = int(w.slo_us[i] // w.tick_us), 1 << 30
    f, out = np.zeros(T + 1, np.int64), []
    for s in range(w.n_stage - 1, -1, -1):
        g = np.full(T + 1, inf, np.int64)
        for k in np.nonzero(lt[i, s] >= 0)[0]:
            l, c = int(lt[i, s, k]), int(cost[i, s, k])
            if l <= T:
                np.minimum(g[l:], f[:T + 1 - l] + c, out=g[l:])
        f = np.minimum(g, inf)
        out.append(int((np.diff(np.concatenate([[inf], f])) < 0).sum()))
    return out


def test_step_rows_long_lists_and_many_candidates(T, oracle):
    """Costs that make rows drop at very many budgets (more than the 1024 the list
    in LDS holds, so the threads scatter from their own stretches), and models with
    more candidates than are staged at a time."""
    rng = np.random.default_rng(8)
    n, S, c_max, r_max, tick, slo_max = 6, 7, 64, 72, 20, 327_000
    # many cores and replicas with a fine tick: the total steps down nearly every tick
    coef = np.stack([rng.integers(lo, hi + 1, size=(n, S)) for lo, hi in
                     ((200_000, 900_000), (1000, 5000), (0, 3), (c_max, c_max), (200, 2000))],
                    axis=-1).astype(np.int32)
    w = wl.Workload("steps-long", wl.JOINT, n, S, c_max, [1, 2, 3, 4, 6, 8, 12, 16, 24, 32],
                    r_max, tick, slo_max, False, coef, rng.integers(50, 4000, n).astype(np.int32),
                    rng.integers(slo_max * 3 // 4, slo_max + 1, n).astype(np.int32))
    lt, cost, _ = oracle.candidates(w)
    assert ((lt >= 0).sum(axis=2) > 512).any()            # more entries than one staging round
    drops = np.array([_drops_per_row(w, lt, cost, i) for i in range(n)])   # [n][S], s = S-1 .. 0
    # a list that outgrows its area before a model that scatters (row s >= 2), and
    # one before the model of which only the answer is formed (row s = 1)
    assert (drops[:, :S - 2] > 1024).any() and (drops[:, S - 2] > 1024).any(), drops
    assert (drops[:, 0] <= 1024).all()                     # (the first rows keep their lists)
    want = oracle.solve(w, threads=6)
    assert (want[0] == 0).any()
    for prune in (2, 3):
        print(f"[case] step rows long lists prune={prune} K={w.n_cand}", flush=True)
        b = T.DeviceBatch(w, prune=prune)
        b.solve()
        same(b.results(), want)


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


@pytest.mark.parametrize("prune", [2, 3])
@pytest.mark.parametrize("idx", [1, 3])
def test_step_rows_full_size(T, full_checker, idx, prune):
    """Full batches in the launch configuration the benchmark times: every instance
    against the checker."""
    w, want = full_checker(idx)
    print(f"[case] step rows full workload {idx} N={w.n_inst} prune={prune}", flush=True)
    b = T.DeviceBatch(w, prune=prune)
    b.solve()
    same(b.results(), want)
