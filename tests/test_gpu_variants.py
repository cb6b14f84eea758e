"""GPU parity under the paper's printed model forms (queue of Eq. 4 / Eq. 3,
Eq. 1's delta*b term) and with the dense batch range 1..16 of Section 4.4,
against the CPU checker, through the C ABI.  Bit-exact."""

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


def variant_of(w, queue_model, form, seed):
    rng = np.random.default_rng(seed)
    d = rng.integers(0, 1500, size=w.coef.shape[:-1]) if form else None
    return w.with_model(queue_model, d)


@pytest.mark.parametrize("queue_model,form", [(1, 0), (2, 0), (0, 1), (1, 1), (2, 1)])
@pytest.mark.parametrize("idx,n", [(1, 120), (2, 60), (4, 100)])
def test_tables_and_solve(T, oracle, idx, n, queue_model, form):
    w = variant_of(wl.workload(idx, n), queue_model, form, 50 + idx)
    print(f"[case] variant workload {idx} queue={queue_model} form={form}", flush=True)
    lt_o, cost_o, _ = oracle.candidates(w)
    b = T.DeviceBatch(w)
    lt_g, cost_g = b.candidates()
    assert (lt_g == lt_o).all() and (cost_g == cost_o).all()
    want = oracle.solve(w, threads=8)
    b.solve()
    same(b.results(), want)
    assert (want[0] == 0).any()


def test_options_change_the_answer(T, oracle):
    """Guards against an option that is accepted but ignored: the shared queue
    and the sixth coefficient must each move some results on the GPU."""
    base = wl.workload(1, 200)
    b0 = T.DeviceBatch(base)
    b0.solve()
    r0 = b0.results()
    for qm, form in ((1, 0), (0, 1)):
        w = variant_of(base, qm, form, 5)
        b = T.DeviceBatch(w)
        b.solve()
        r = b.results()
        assert (r[1] != r0[1]).any() or (r[2] != r0[2]).any(), (qm, form)


def test_tiny_random_variants(T, oracle):
    rng = np.random.default_rng(77)
    for rep in range(30):
        w = wl.tiny_random(rng, rep % 2, n_inst=int(rng.integers(1, 50)))
        if w.slo_max_us // w.tick_us > 32767:
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        w = variant_of(w, rep % 3, (rep // 3) % 2, rep)
        print(f"[case] tiny variant rep {rep} queue={w.queue_model} form={w.profile_form}",
              flush=True)
        want = oracle.solve(w)
        b = T.DeviceBatch(w)
        b.solve()
        same(b.results(), want)


def test_invalid_sixth_coefficient(T, oracle):
    w = wl.workload(0, 12)
    d = np.zeros(w.coef.shape[:-1], np.int32)
    d[3, 1] = -5
    d[7, 0] = (1 << 20) + 1
    d[8, 2] = 1 << 20                       # largest accepted value
    w = w.with_model(1, d)
    want = oracle.solve(w)
    print("[case] invalid sixth coefficient", flush=True)
    b = T.DeviceBatch(w)
    b.solve()
    got = b.results()
    same(got, want)
    assert got[0][3] == T.INVALID and got[0][7] == T.INVALID and got[0][8] != T.INVALID


def test_dense_batch_range(T, oracle):
    """Section 4.4 searches every batch size 1..16, not only powers of two."""
    w = wl.workload(1, 150)
    w.batch_sizes = list(range(1, 17))
    w.c_max = 16
    for qm in (0, 1):
        wv = w.with_model(qm)
        print(f"[case] dense batches queue={qm} K={wv.n_cand}", flush=True)
        lt_o, cost_o, _ = oracle.candidates(wv)
        b = T.DeviceBatch(wv)
        lt_g, cost_g = b.candidates()
        assert (lt_g == lt_o).all() and (cost_g == cost_o).all()
        want = oracle.solve(wv, threads=8)
        b.solve()
        same(b.results(), want)
        assert (want[0] == 0).any()


def test_fallback_and_stability_under_paper_forms(T, oracle):
    """The multi-pass entry points use the same candidate evaluation."""
    w = wl.workload(2, 60)
    rng = np.random.default_rng(12)
    w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 6, w.n_inst),
                       1 << 20).astype(np.int32)
    w = variant_of(w, 1, 1, 13)
    want = oracle.vertical_fallback(w, threads=8)
    print("[case] fallback under Eq. 4 / Eq. 1", flush=True)
    b = T.DeviceBatch(w)
    b.solve_vertical_fallback()
    got = b.fallback_results()
    keys = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h", "cfg_h")
    same([got[k] for k in keys], [want[k] for k in keys], keys)
    assert ((want["lambda_v"] > 0) & (want["lambda_v"] < w.lam)).any()

    j = variant_of(wl.workload(1, 100), 1, 1, 14)
    j.slo_us = (j.slo_us // 3).astype(np.int32)
    pred = np.clip(j.lam.astype(np.int64) + rng.integers(-20, 40, j.n_inst), 1, 1 << 20)
    wants = oracle.stability(j, pred.astype(np.int32))
    print("[case] stability under Eq. 4 / Eq. 1", flush=True)
    bj = T.DeviceBatch(j)
    stable = bj.check_stability(pred.astype(np.int32))
    same((stable.cpu().numpy(),) + bj.results(), wants, ("stable",) + NAMES)
