"""GPU parity for the solve that handles every distinct instance once: its
outputs must equal the CPU checker's on the whole batch, duplicates and invalid
instances included, and equal those of the plain solve.  Integer work: every
output must be equal."""

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


@pytest.fixture(scope="module")
def oracle():
    from oracle import oracle as o
    return o


def same(got, want):
    for n, g, x in zip(NAMES, got, want):
        bad = np.nonzero((g != x).reshape(len(x), -1).any(axis=1))[0]
        assert bad.size == 0, f"{n} differs at {bad[:8]}: got {g[bad[:2]]}, want {x[bad[:2]]}"


def with_repeats(w, rng, n_out):
    """n_out instances drawn with replacement from w: most tuples recur."""
    return w.take(rng.integers(0, w.n_inst, n_out))


@pytest.mark.parametrize("idx,pool,n", [(1, 40, 500), (3, 25, 300), (0, 64, 64)])
def test_joint_with_recurring_instances(T, oracle, idx, pool, n):
    rng = np.random.default_rng(100 + idx)
    w = with_repeats(wl.workload(idx, pool), rng, n)
    b = T.DeviceBatch(w)
    b.solve_distinct()
    got = b.results()
    same(got, oracle.solve(w))
    b.solve()
    same(b.results(), got)


def test_vertical_with_recurring_replicas(T, oracle):
    rng = np.random.default_rng(7)
    w = with_repeats(wl.workload(2, 30), rng, 400)
    # the same rate and objective under other replica counts is another tuple
    w.r_fixed[::3] = np.maximum(1, w.r_fixed[::3] - 1)
    b = T.DeviceBatch(w)
    b.solve_distinct()
    same(b.results(), oracle.solve(w))


def test_trace_sweep_shares_everything_but_the_rate(T, oracle):
    # the per-second trace workload: shared coefficients, one objective, few rates;
    # the second pass carries the replicas of the previous second forward
    w = wl.workload(4, 3000)
    assert w.coef_shared and np.unique(w.lam).size < w.n_inst // 4
    b = T.DeviceBatch(w)
    b.solve_distinct()
    want_j = oracle.solve(w, threads=8)
    same(b.results(), want_j)
    wv = w.with_r_fixed(wl.replicas_carried_forward(want_j[0], want_j[3]))
    b = T.DeviceBatch(wv)
    b.solve_distinct()
    got_v = b.results()
    same(got_v, oracle.solve(wv, threads=8))
    assert (got_v[0] == 0).any()


def test_invalid_instances_and_their_copies(T, oracle):
    rng = np.random.default_rng(9)
    w = with_repeats(wl.workload(1, 20), rng, 200)
    w.lam[5] = 0                      # out of range
    w.lam[6] = 0                      # the same invalid tuple again
    w.slo_us[7] = w.slo_max_us + 1    # out of range
    w.coef[8, 0, 3] = 0               # a core cap below one; coefficients are per instance here
    w.coef[9] = w.coef[8]
    w.lam[9], w.slo_us[9] = w.lam[8], w.slo_us[8]
    assert not w.coef_shared
    b = T.DeviceBatch(w)
    b.solve_distinct()
    got = b.results()
    same(got, oracle.solve(w))
    assert (got[0][[5, 6, 7, 8, 9]] == 2).all()


def test_all_distinct_and_single_instance(T, oracle):
    rng = np.random.default_rng(3)
    for n in (1, 97):
        w = wl.tiny_random(rng, wl.JOINT, n_inst=n, max_stage=4)
        if w.slo_max_us // w.tick_us > 32767:
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        b = T.DeviceBatch(w)
        b.solve_distinct()
        same(b.results(), oracle.solve(w))


def test_tiny_random_with_repeats_and_options(T, oracle):
    rng = np.random.default_rng(2024)
    for rep in range(30):
        variant = int(rng.integers(0, 2))
        base = wl.tiny_random(rng, variant, n_inst=int(rng.integers(1, 12)),
                              max_stage=int(rng.integers(1, 5)))
        if base.slo_max_us // base.tick_us > 32767:     # finest ticks: stay on the accepted grid
            base.slo_max_us = 30_000 * base.tick_us
            base.slo_us = (base.slo_us % (base.slo_max_us + 1)).astype(np.int32)
        w = with_repeats(base, rng, int(rng.integers(1, 80)))
        w = w.with_model(queue_model=int(rng.integers(0, 3)))
        b = T.DeviceBatch(w, prune=int(rng.integers(0, 4)))
        b.solve_distinct()
        same(b.results(), oracle.solve(w))


def test_twice_on_one_workspace_and_on_a_stream(T, oracle):
    import torch
    rng = np.random.default_rng(11)
    w = with_repeats(wl.workload(1, 30), rng, 300)
    b = T.DeviceBatch(w)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()   # the inputs were copied on the default stream
    b.solve_distinct(stream=st)
    st.synchronize()
    want = oracle.solve(w)
    same(b.results(), want)
    b.status.fill_(77)
    b.solve_distinct()
    same(b.results(), want)


def test_argument_checks(T):
    import torch
    w = wl.workload(0, 8)
    b = T.DeviceBatch(w)
    small = torch.empty(T.workspace_bytes(b.p), dtype=torch.uint8, device="cuda:0")
    assert T.memo_workspace_bytes(b.p) > T.workspace_bytes(b.p)
    b.status.fill_(77)
    with pytest.raises(T.ThemisError) as e:
        T.themis_solve_distinct(b.p, b.coef, b.lam, b.slo_us, None, b.status, b.cost, b.ticks,
                                b.cfg, small)
    assert e.value.rc == T.ERR_WORKSPACE
    ws = torch.empty(T.memo_workspace_bytes(b.p), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(T.ThemisError) as e:
        T.themis_solve_distinct(b.p, b.coef, None, b.slo_us, None, b.status, b.cost, b.ticks,
                                b.cfg, ws)
    assert e.value.rc == T.ERR_NULL
    torch.cuda.synchronize()
    assert (b.status.cpu().numpy() == 77).all()   # nothing was launched
