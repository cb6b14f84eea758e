"""GPU parity with dominated candidates pruned before the recurrence: the
answers must be the same as the CPU checker's (which prunes nothing), bit for
bit, and the candidates that survive must be exactly the cost/latency
staircase of each row."""

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
    for n, g, x in zip(names, got, want):
        bad = np.nonzero((g != x).reshape(len(x), -1).any(axis=1))[0]
        assert bad.size == 0, f"{n} differs at {bad[:8]}: got {g[bad[:2]]}, want {x[bad[:2]]}"


def staircase(lt, cost):
    """Survivors of one row by the definition: feasible, and no other candidate
    is (<=, <=) on (lt, cost) with one strict or with a smaller index."""
    keep = np.zeros(lt.shape, bool)
    feas = np.nonzero(lt >= 0)[0]
    for k in feas:
        o = feas[feas != k]
        le = (lt[o] <= lt[k]) & (cost[o] <= cost[k])
        strict = (lt[o] < lt[k]) | (cost[o] < cost[k]) | (o < k)
        keep[k] = not (le & strict).any()
    return keep


@pytest.mark.parametrize("idx,n", [(0, 64), (1, 150), (2, 80), (3, 60), (4, 120)])
def test_pruned_solve_and_survivors(T, oracle, idx, n):
    w = wl.workload(idx, n)
    if idx == 4:
        rng = np.random.default_rng(4)
        w = w.with_r_fixed(rng.integers(1, 6, size=(w.n_inst, w.n_stage)))
    print(f"[case] pruned workload {idx} N={n}", flush=True)
    b = T.DeviceBatch(w, prune=1)
    lt_g, cost_g = b.candidates()
    lt_o, cost_o, _ = oracle.candidates(w)
    kept = lt_g >= 0
    # survivors keep their values; everything else reads as infeasible
    assert (lt_g[kept] == lt_o[kept]).all() and (cost_g[kept] == cost_o[kept]).all()
    assert (cost_g[~kept] == -1).all()
    # Exactly the staircase, wherever the cost table (two words per table slot of the
    # row) holds one bin per cost up to the fastest candidate's; a row whose fastest
    # candidate costs more gets coarser bins and may keep a few candidates more.
    cap = 2 * ((w.n_cand + 7) // 8 * 8)
    exact = 0
    for i in range(0, w.n_inst, 7):
        for s in range(w.n_stage):
            must = staircase(lt_o[i, s], cost_o[i, s])
            feas = lt_o[i, s] >= 0
            if not feas.any():
                assert not kept[i, s].any()
                continue
            fastest = np.lexsort((cost_o[i, s][feas], lt_o[i, s][feas]))[0]
            if cost_o[i, s][feas][fastest] + 2 <= cap:
                assert (kept[i, s] == must).all(), (i, s)
                exact += 1
            else:
                assert (kept[i, s] | ~must).all() and not (kept[i, s] & ~feas).any(), (i, s)
    assert exact > 0
    assert kept.sum() < 0.25 * (lt_o >= 0).sum()
    b.solve()
    same(b.results(), oracle.solve(w, threads=8))


def test_pruned_tiny_random(T, oracle):
    rng = np.random.default_rng(123)
    for rep in range(40):
        w = wl.tiny_random(rng, rep % 2, n_inst=int(rng.integers(1, 70)))
        if w.slo_max_us // w.tick_us > 32767:
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        if rep % 4 == 3:
            w = w.with_model(1, rng.integers(0, 1500, size=w.coef.shape[:-1]))
        print(f"[case] pruned tiny rep {rep} K={w.n_cand} S={w.n_stage}", flush=True)
        b = T.DeviceBatch(w, prune=1)
        b.solve()
        same(b.results(), oracle.solve(w))


@pytest.mark.parametrize("S", [12, 70])
def test_pruned_many_models(T, oracle, S):
    """Pipelines whose pruned rows do not fit the staging buffer of stage 2 together
    (sixteen candidates per model, so the buffer holds sixteen entries: the models
    go through it in several batches), and one with more models than a wavefront
    has lanes (served by the kernel for unpruned rows)."""
    rng = np.random.default_rng(31 + S)
    n, c_max, r_max = 48, 4, 60
    bs = [1, 2, 4, 8]
    coef = np.stack([rng.integers(lo, hi + 1, size=(n, S)) for lo, hi in
                     ((200, 6000), (50, 1500), (0, 20), (1, 4), (1, 300))],
                    axis=-1).astype(np.int32)
    lam = rng.integers(200, 4000, n).astype(np.int32)
    slo = rng.integers(20_000, 2_000_000, n).astype(np.int32)
    w = wl.Workload(f"many-{S}", wl.JOINT, n, S, c_max, bs, r_max, 250, 2_000_000, False, coef,
                    lam, slo)
    print(f"[case] pruned, {S} models", flush=True)
    b = T.DeviceBatch(w, prune=1)
    assert T.check_problem(b.p) == T.OK
    lt_g, _ = b.candidates()
    survivors = (lt_g >= 0).sum(axis=-1)                    # [n, S]
    padded = ((survivors + 3) // 4 * 4).sum(axis=-1)        # entries of an instance, rows on groups of four
    assert (padded > 2 * 16).all(), "every instance needs more than two batches"
    want = oracle.solve(w, threads=8)
    b.solve()
    same(b.results(), want)
    assert (want[0] == 0).sum() > 30


def test_pruned_with_binned_costs(T, oracle):
    """r_max * c_max beyond the cost table: costs are binned, fewer candidates
    are dropped, the answers stay the same and no survivor is dominated by a
    candidate of a cheaper bin."""
    rng = np.random.default_rng(6)
    n, S, c_max, r_max = 96, 3, 8, 1200
    bs = [1, 2, 4, 8]
    coef = np.stack([rng.integers(lo, hi + 1, size=(n, S)) for lo, hi in
                     ((20_000, 200_000), (5_000, 50_000), (0, 50), (2, 8), (100, 1000))],
                    axis=-1).astype(np.int32)
    lam = rng.integers(2_000, 40_000, n).astype(np.int32)
    slo = rng.integers(100_000, 2_000_000, n).astype(np.int32)
    w = wl.Workload("binned", wl.JOINT, n, S, c_max, bs, r_max, 250, 2_000_000, False, coef,
                    lam, slo)
    print("[case] pruned binned costs", flush=True)
    b = T.DeviceBatch(w, prune=1)
    assert T.check_problem(b.p) == T.OK
    lt_g, cost_g = b.candidates()
    lt_o, cost_o, _ = oracle.candidates(w)
    kept = lt_g >= 0
    assert (lt_g[kept] == lt_o[kept]).all() and (cost_g[kept] == cost_o[kept]).all()
    assert (cost_o[lt_o >= 0].max() > 2560) and kept.sum() < (lt_o >= 0).sum()
    for i in range(0, n, 5):
        for s in range(S):
            must = staircase(lt_o[i, s], cost_o[i, s])
            assert (kept[i, s] | ~must).all()          # nothing needed was dropped
    want = oracle.solve(w, threads=8)
    b.solve()
    same(b.results(), want)
    assert (want[0] == 0).sum() > 20


def test_pruned_multi_pass_entry_points(T, oracle):
    w = wl.workload(2, 60)
    rng = np.random.default_rng(12)
    w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 6, w.n_inst),
                       1 << 20).astype(np.int32)
    want = oracle.vertical_fallback(w, threads=8)
    print("[case] pruned fallback", flush=True)
    b = T.DeviceBatch(w, prune=1)
    b.solve_vertical_fallback()
    got = b.fallback_results()
    keys = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h", "cfg_h")
    same([got[k] for k in keys], [want[k] for k in keys], keys)


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_pruned_full_size(T, full_checker, idx):
    """Full batches in the launch configuration the benchmark times: every instance
    against the checker (the dense GPU path is not consulted)."""
    w, want = full_checker(idx)
    print(f"[case] pruned full workload {idx} N={w.n_inst}", flush=True)
    b = T.DeviceBatch(w, prune=1)
    b.solve()
    same(b.results(), want)
