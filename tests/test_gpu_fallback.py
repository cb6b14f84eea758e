"""GPU parity for the horizontal-only solve (Algorithm 2) and for the vertical
solve with Algorithm 1's fallback, against the CPU checker, through the C ABI.
Integer work: every output must be equal."""

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

pytestmark = pytest.mark.gpu

FB_KEYS = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h", "cfg_h")


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_14843_amd import themis
    themis.lib()
    return themis


def same(got, want, names):
    for n, g, x in zip(names, got, want):
        bad = np.nonzero((g != x).reshape(len(x), -1).any(axis=1))[0]
        assert bad.size == 0, f"{n} differs at {bad[:8]}: got {g[bad[:2]]}, want {x[bad[:2]]}"


def as_joint(w):
    j = w.take(np.arange(w.n_inst))
    j.variant, j.r_fixed = wl.JOINT, None
    return j


# ------------------------------------------------------------ horizontal only
@pytest.mark.parametrize("idx,n", [(0, 64), (1, 150), (3, 40)])
def test_horizontal_given_cores(T, oracle, idx, n):
    w = as_joint(wl.workload(idx, n))
    rng = np.random.default_rng(idx)
    cores = rng.integers(1, w.c_max + 1, size=(w.n_inst, w.n_stage)).astype(np.int32)
    want = oracle.solve(w, threads=8, c_fixed=cores)
    print(f"[case] horizontal workload {idx} N={n}", flush=True)
    b = T.DeviceBatch(w)
    b.solve_horizontal(cores)
    got = b.results()
    same(got, want, FB_KEYS[:4])
    ok = want[0] == 0
    assert ok.any() and (got[3][ok][:, :, 0] == cores[ok]).all()


def test_horizontal_one_core_instances(T, oracle):
    """Algorithm 2 proper: no cores argument means one core per instance."""
    w = as_joint(wl.workload(1, 120))
    w.slo_us = (w.slo_us // 4).astype(np.int32)   # tight enough that one core sometimes fails
    want = oracle.solve(w, threads=8, c_fixed=np.ones((w.n_inst, w.n_stage), np.int32))
    print("[case] horizontal one core", flush=True)
    b = T.DeviceBatch(w)
    b.solve_horizontal(None)
    same(b.results(), want, FB_KEYS[:4])
    assert (want[0] == 0).any() and (want[0] == 1).any()


def test_horizontal_bad_cores_are_invalid(T, oracle):
    w = as_joint(wl.workload(0, 16))
    cores = np.ones((w.n_inst, w.n_stage), np.int32)
    cores[2, 0] = 0
    cores[5, -1] = w.c_max + 1
    print("[case] horizontal bad cores", flush=True)
    b = T.DeviceBatch(w)
    b.solve_horizontal(cores)
    st, cost, ticks, cfg = b.results()
    assert st[2] == T.INVALID and st[5] == T.INVALID and cost[2] == -1 and not cfg[5].any()
    good = np.ones(w.n_inst, bool)
    good[[2, 5]] = False
    want = oracle.solve(w.take(np.nonzero(good)[0]), c_fixed=cores[good])
    same([st[good], cost[good], ticks[good], cfg[good]], want, FB_KEYS[:4])


# ------------------------------------------------------------ fallback
def overloaded(idx, n, seed, factor):
    """A vertical workload whose rates are pushed up so that the running
    replicas often cannot keep the SLO."""
    w = wl.workload(idx, n)
    rng = np.random.default_rng(seed)
    if w.r_fixed is None:
        w = w.with_r_fixed(rng.integers(1, max(2, w.r_max // 4), size=(w.n_inst, w.n_stage)))
    w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, factor, w.n_inst),
                       1 << 20).astype(np.int32)
    return w


def run_fallback(T, w):
    print(f"[case] fallback {w.name} N={w.n_inst} S={w.n_stage} K={w.n_cand}", flush=True)
    b = T.DeviceBatch(w)
    b.solve_vertical_fallback()
    return b, b.fallback_results()


@pytest.mark.parametrize("idx,n,factor", [(2, 120, 6), (4, 150, 300), (0, 64, 5)])
def test_fallback_matches_checker(T, oracle, idx, n, factor):
    w = overloaded(idx, n, 7 + idx, factor)
    want = oracle.vertical_fallback(w, threads=8)
    _, got = run_fallback(T, w)
    same([got[k] for k in FB_KEYS], [want[k] for k in FB_KEYS], FB_KEYS)
    lv, lam = want["lambda_v"], w.lam
    # the case mix the test is meant to see
    assert (lv == lam).any() and ((lv > 0) & (lv < lam)).any()
    assert (want["status_h"][(lv > 0) & (lv < lam)] == 0).any()


def test_fallback_tiny_random(T, oracle):
    rng = np.random.default_rng(21)
    mix = np.zeros(3, int)
    for rep in range(25):
        w = wl.tiny_random(rng, wl.VERTICAL, n_inst=int(rng.integers(1, 60)))
        if w.slo_max_us // w.tick_us > 32767:
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 12, w.n_inst),
                           1 << 20).astype(np.int32)
        want = oracle.vertical_fallback(w)
        _, got = run_fallback(T, w)
        same([got[k] for k in FB_KEYS], [want[k] for k in FB_KEYS], FB_KEYS)
        lv = want["lambda_v"]
        mix += [(lv == w.lam).sum(), ((lv > 0) & (lv < w.lam)).sum(),
                ((lv == 0) & (want["status"] == 1)).sum()]
    assert (mix > 5).all(), mix


def test_fallback_edge_rates_and_invalid(T, oracle):
    """Rates 1, 2 and 3 (search intervals of width 0, 1 and 2), the largest
    rate, and invalid instances."""
    w = overloaded(2, 40, 3, 6)
    w.slo_us[:12] = w.slo_us[:12] // 40           # hopeless at any rate, mostly
    w.lam[0:3] = [1, 2, 3]
    w.lam[3] = 1 << 20
    w.lam[4] = 0                                   # invalid
    w.r_fixed[5, 0] = w.r_max + 1                  # invalid
    want = oracle.vertical_fallback(w)
    _, got = run_fallback(T, w)
    same([got[k] for k in FB_KEYS], [want[k] for k in FB_KEYS], FB_KEYS)
    assert got["status"][4] == T.INVALID and got["status_h"][5] == T.INVALID


def test_fallback_shortest_searches(T, oracle):
    """One slow model (0.6 s per batch, one replica): rate 1 fits, rates 2 and 3
    do not, so the searches start from intervals of width 1 and 2 and must
    settle on rate 1 with the remainder handed to new instances."""
    n = 3
    coef = np.tile(np.array([600_000, 0, 0, 1, 1], np.int32), (n, 1, 1))
    w = wl.Workload("edge", wl.VERTICAL, n, 1, 2, [1, 2], 4, 1000, 1_000_000, False, coef,
                    np.array([1, 2, 3], np.int32), np.full(n, 700_000, np.int32),
                    r_fixed=np.ones((n, 1), np.int32))
    want = oracle.vertical_fallback(w)
    assert want["lambda_v"].tolist() == [1, 1, 1] and want["cost_h"].tolist() == [0, 1, 2]
    _, got = run_fallback(T, w)
    same([got[k] for k in FB_KEYS], [want[k] for k in FB_KEYS], FB_KEYS)


def test_fallback_twice_on_one_workspace(T, oracle):
    """Search state left by one call must not leak into the next."""
    w1 = overloaded(2, 60, 1, 8)
    w2 = overloaded(2, 60, 2, 3)
    b, got1 = run_fallback(T, w1)
    import torch
    b.lam.copy_(torch.from_numpy(w2.lam))
    b.r_fixed.copy_(torch.from_numpy(w2.r_fixed))
    b.slo_us.copy_(torch.from_numpy(w2.slo_us))
    b.coef.copy_(torch.from_numpy(w2.coef))
    b.solve_vertical_fallback()
    got2 = b.fallback_results()
    for got, w in ((got1, w1), (got2, w2)):
        want = oracle.vertical_fallback(w, threads=8)
        same([got[k] for k in FB_KEYS], [want[k] for k in FB_KEYS], FB_KEYS)


# ------------------------------------------------------------ stability test
@pytest.mark.parametrize("idx,n,given", [(1, 200, False), (0, 64, True), (3, 50, False)])
def test_stability_matches_checker(T, oracle, idx, n, given):
    w = as_joint(wl.workload(idx, n))
    rng = np.random.default_rng(30 + idx)
    w.slo_us = (w.slo_us // 3).astype(np.int32)
    pred = np.clip(w.lam.astype(np.int64) + rng.integers(-20, 40, w.n_inst), 1, 1 << 20)
    pred = pred.astype(np.int32)
    pred[1] = 0                                   # invalid prediction: not stable
    cores = rng.integers(1, 3, size=(w.n_inst, w.n_stage)).astype(np.int32) if given else None
    want = oracle.stability(w, pred, cores)
    print(f"[case] stability workload {idx} N={n} given={given}", flush=True)
    b = T.DeviceBatch(w)
    stable = b.check_stability(pred, cores)
    got = (stable.cpu().numpy(),) + b.results()
    same(got, want, ("stable",) + FB_KEYS[:4])
    assert want[0].any() and not want[0].all() and want[0][1] == 0
