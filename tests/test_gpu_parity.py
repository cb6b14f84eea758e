"""GPU parity: the HIP library against the CPU checker, element by element,
through the C ABI.  Everything here is integer work, so the bar is bit-exact
equality of status, cost, ticks and configuration."""

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_14843_amd import themis
    themis.lib()           # raises if the HIP library has not been built
    return themis


def gpu_solve(T, w, prune=0):
    print(f"[case] {w.name} N={w.n_inst} S={w.n_stage} K={w.n_cand} variant={w.variant} "
          f"tick={w.tick_us} slo_max={w.slo_max_us} prune={prune}", flush=True)
    b = T.DeviceBatch(w, prune=prune)
    b.solve()
    return b.results()


def assert_same(got, want, idx=None):
    names = ("status", "cost", "ticks", "cfg")
    for n, g, x in zip(names, got, want):
        if idx is not None:
            g = g[idx]
        bad = np.nonzero((g != x).reshape(len(x), -1).any(axis=1))[0]
        assert bad.size == 0, f"{n} differs at instances {bad[:8]}: got {g[bad[:2]]}, want {x[bad[:2]]}"


# ------------------------------------------------------------ stage 1 tables
@pytest.mark.parametrize("idx,n", [(0, 64), (1, 96), (2, 48), (3, 40), (4, 200)])
def test_candidate_tables(T, oracle, idx, n):
    w = wl.workload(idx, n)
    if idx == 4:  # second pass of the trace sweep: some fixed replicas
        rng = np.random.default_rng(4)
        w = w.with_r_fixed(rng.integers(1, 6, size=(w.n_inst, w.n_stage)))
    lt_o, cost_o, r_o = oracle.candidates(w)
    print(f"[case] tables workload {idx}", flush=True)
    lt_g, cost_g = T.DeviceBatch(w).candidates()
    assert (lt_g == lt_o).all()
    assert (cost_g == cost_o).all()
    feas = lt_o >= 0
    assert 0.02 < feas.mean() < 1.0
    c_of_k = np.arange(w.n_cand) // len(w.batch_sizes) + 1
    assert ((cost_g // c_of_k)[feas] == r_o[feas]).all()


# ------------------------------------------------------------ whole solve
@pytest.mark.parametrize("idx,n", [(0, 64), (1, 200), (2, 100), (3, 70), (4, 150)])
def test_solve_matches_oracle_small(T, oracle, idx, n):
    """Each workload at a size the checker finishes in seconds; N is not a
    multiple of anything the kernels tile by."""
    w = wl.workload(idx, n)
    want = oracle.solve(w, threads=8)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert (want[0] == 0).any()


def test_tiny_random_batches(T, oracle):
    """Many small search spaces: odd K, one batch size, one stage, tick 1 ..."""
    rng = np.random.default_rng(99)
    seen = set()
    for rep in range(40):
        variant = rep % 2
        w = wl.tiny_random(rng, variant, n_inst=int(rng.integers(1, 70)))
        if w.slo_max_us // w.tick_us > 32767:     # finest ticks: stay on the accepted grid
            w.slo_max_us = 30_000 * w.tick_us
            w.slo_us = (w.slo_us % (w.slo_max_us + 1)).astype(np.int32)
        want = oracle.solve(w)
        got = gpu_solve(T, w)
        assert_same(got, want)
        seen |= set(want[0].tolist())
    assert seen >= {0, 1}


def test_tight_slos_mix_feasible_and_infeasible(T, oracle):
    w = wl.workload(1, 300)
    w.slo_us = (w.slo_us // 25).astype(np.int32)
    want = oracle.solve(w, threads=8)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert set(want[0].tolist()) == {0, 1}


@pytest.mark.parametrize("cells", [1, 2, 3, 4, 6, 127, 128, 129, 1023, 1024, 1025, 2048, 2049,
                                   4097, 8193, 16385, 32768])
def test_row_lengths_around_tile_edges(T, oracle, cells):
    """Budgets T+1 just below, at and above the kernels' chunk and row sizes,
    up to the largest grid the interface accepts."""
    base = wl.workload(0, 6)
    # tick chosen so that the budget binds: three stages need roughly 30-150 ms
    tick = max(1, 100_000 // cells)
    slo_max = (cells - 1) * tick + tick - 1          # floor(slo_max/tick) = cells - 1
    slo = np.array([slo_max, slo_max - (tick - 1), max(0, slo_max - 2 * tick), slo_max // 2,
                    slo_max // 3, 0], np.int32)
    w = wl.Workload(f"edge{cells}", wl.JOINT, 6, base.n_stage, base.c_max, base.batch_sizes,
                    base.r_max, tick, slo_max, False, base.coef, base.lam, slo)
    want = oracle.solve(w)
    for prune in (0, 1):  # the kernel for unpruned rows, the one for pruned rows
        assert_same(gpu_solve(T, w, prune), want)


def test_invalid_and_degenerate_instances(T, oracle):
    w = wl.workload(0, 16)
    w.lam[1] = 0
    w.slo_us[2] = -5
    w.coef[3, 1, 4] = 0
    w.coef[4, 0, 3] = 0
    w.coef[5, 2, 0] = -1
    w.slo_us[6] = w.slo_max_us + 1
    w.lam[7] = (1 << 20) + 1
    w.slo_us[8] = 0                 # T = 0: nothing fits
    w.slo_us[9] = 999               # below one tick
    w.lam[10] = 1 << 20             # largest accepted arrival rate
    want = oracle.solve(w)
    for prune in (0, 1):
        assert_same(gpu_solve(T, w, prune), want)
    assert want[0][:11].tolist() == [0, 2, 2, 2, 2, 2, 2, 2, 1, 1, 1]


def test_vertical_invalid_replicas(T, oracle):
    w = wl.workload(2, 12)
    w.r_fixed[3, 2] = 0
    w.r_fixed[5, 7] = w.r_max + 1
    want = oracle.solve(w)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert want[0][3] == 2 and want[0][5] == 2


def test_large_coefficients_and_batches(T, oracle):
    """Values at the documented upper limits: 64-bit intermediates on both sides."""
    rng = np.random.default_rng(3)
    n, S = 40, 2
    coef = np.stack([rng.integers(0, (1 << 20) + 1, size=(n, S)),
                     rng.integers(0, (1 << 20) + 1, size=(n, S)),
                     rng.integers(0, (1 << 20) + 1, size=(n, S)),
                     rng.integers(1, 2000, size=(n, S)),
                     rng.integers(1, (1 << 20) + 1, size=(n, S))], axis=-1).astype(np.int32)
    coef[::3, :, :3] //= 4096
    lam = rng.integers(1, (1 << 20) + 1, size=n).astype(np.int32)
    lam[::2] = rng.integers(1, 50, size=lam[::2].size)
    slo = rng.integers(0, 2_000_000_000, size=n).astype(np.int32)
    w = wl.Workload("big", wl.JOINT, n, S, 1024, [1, 3, 1024], 15, 70_000, 2_000_000_000,
                    False, coef, lam, slo)
    want = oracle.solve(w, threads=8)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert (want[0] == 0).any()


def test_rows_longer_than_the_staging_buffer(T, oracle):
    """More than 512 feasible candidates per model: the min-plus stage walks
    such rows in parts."""
    rng = np.random.default_rng(8)
    n, S = 24, 3
    coef = np.stack([rng.integers(500, 3000, size=(n, S)), rng.integers(50, 400, size=(n, S)),
                     rng.integers(0, 3, size=(n, S)), rng.integers(20, 60, size=(n, S)),
                     rng.integers(1, 200, size=(n, S))], axis=-1).astype(np.int32)
    lam = rng.integers(5000, 40000, size=n).astype(np.int32)
    slo = rng.integers(1_500, 9_000, size=n).astype(np.int32)
    w = wl.Workload("longrows", wl.JOINT, n, S, 100, [1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32],
                    100, 10, 9_000, False, coef, lam, slo)
    lt, _, _ = oracle.candidates(w)
    assert ((lt >= 0).sum(axis=2) > 512).any()
    want = oracle.solve(w, threads=8)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert (want[0] == 0).any()


@pytest.mark.parametrize("prune", [0, 1])
def test_largest_candidate_count(T, oracle, prune):
    """K = 8192 candidates per model (512 cores x 16 batch sizes), the most the
    interface takes: one row no longer fits the staging buffer of stage 2 and
    stage 1 is down to two rows per workgroup."""
    rng = np.random.default_rng(31)
    n, S, c_max, r_max = 7, 1, 512, 60
    bs = [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256]
    coef = np.stack([rng.integers(lo, hi + 1, size=(n, S)) for lo, hi in
                     ((200_000, 900_000), (5_000, 50_000), (0, 50), (1, 700), (100, 1000))],
                    axis=-1).astype(np.int32)
    lam = rng.integers(50, 3000, n).astype(np.int32)
    slo = rng.integers(100_000, 2_000_000, n).astype(np.int32)
    w = wl.Workload("kmax", wl.JOINT, n, S, c_max, bs, r_max, 1000, 2_000_000, False, coef,
                    lam, slo)
    assert w.n_cand == 8192
    print(f"[case] largest K prune={prune}", flush=True)
    b = T.DeviceBatch(w, prune=prune)
    assert T.check_problem(b.p) == T.OK
    if not prune:
        lt_g, cost_g = b.candidates()
        lt_o, cost_o, _ = oracle.candidates(w)
        assert (lt_g == lt_o).all() and (cost_g == cost_o).all()
        assert (lt_o >= 0).sum(axis=2).max() > 512      # more feasible entries than the buffer
    want = oracle.solve(w, threads=7)
    b.solve()
    assert_same(b.results(), want)
    assert (want[0] == 0).sum() >= 4


def test_shared_coefficients(T, oracle):
    w = wl.workload(4, 333)
    want = oracle.solve(w, threads=8)
    got = gpu_solve(T, w)
    assert_same(got, want)


# ------------------------------------------------------------ full sizes
def _sample(n, k, seed):
    return np.sort(np.random.default_rng(seed).choice(n, size=k, replace=False))


def test_full_workload1_every_instance(T, full_checker):
    w, want = full_checker(1)
    got = gpu_solve(T, w)
    assert_same(got, want)


@pytest.mark.parametrize("idx", [2, 3])
def test_full_size_every_instance(T, full_checker, idx):
    """Workloads 2 and 3 at full size, in the launch configuration the benchmark
    times: every instance against the checker."""
    w, want = full_checker(idx)
    got = gpu_solve(T, w)
    assert_same(got, want)
    assert (want[0] == 0).mean() > 0.5


@pytest.mark.parametrize("idx,k", [(2, 160), (3, 128)])
def test_full_size_sampled(T, oracle, idx, k):
    """A quick pre-check of the same two batches: a seeded sample of instances
    against the checker, and properties that hold for every instance."""
    w = wl.workload(idx)
    got = gpu_solve(T, w)
    pick = _sample(w.n_inst, k, idx)
    # always include the extremes of the budget range
    pick = np.unique(np.concatenate([pick, [int(np.argmax(w.slo_us)), int(np.argmin(w.slo_us))]]))
    want = oracle.solve(w.take(pick), threads=8)
    assert_same(got, want, idx=pick)
    st = got[0]
    assert set(np.unique(st).tolist()) <= {0, 1}
    # properties that hold for every instance, at any size
    solved = st == 0
    T_i = w.slo_us // w.tick_us
    assert (got[2][solved] <= T_i[solved]).all() and (got[2][solved] >= w.n_stage).all()
    assert (got[1][solved] >= w.n_stage).all()
    assert (got[3][solved][:, :, 0] >= 1).all() and (got[3][solved][:, :, 0] <= w.c_max).all()
    assert np.isin(got[3][solved][:, :, 1], w.batch_sizes).all()
    assert (got[3][solved][:, :, 2] >= 1).all() and (got[3][solved][:, :, 2] <= w.r_max).all()
    assert (got[1][solved] == (got[3][solved][:, :, 0] * got[3][solved][:, :, 2]).sum(axis=1)).all()
    assert (got[1][~solved] == -1).all() and (got[3][~solved] == 0).all()


@pytest.mark.parametrize("prune", [0, 1])
def test_full_trace_sweep_both_passes(T, oracle, prune):
    """Workload 4 end to end: joint solve of every second, replicas carried
    forward on the host, vertical-only solve of every second.  The checker
    only needs one solve per distinct arrival rate (coefficients and SLO are
    shared), which covers every instance exactly.  (With pruning this is the
    case of many short rows, which stage 2 pulls in chunks.)"""
    w = wl.workload(4)
    got_j = gpu_solve(T, w, prune)
    lam_u, first, inv = np.unique(w.lam, return_index=True, return_inverse=True)
    want_u = oracle.solve(w.take(first), threads=8)
    want_j = tuple(a[inv] for a in want_u)
    assert_same(got_j, want_j)
    # second pass: inputs come from the checker's joint results, not the GPU's
    r_fixed = wl.replicas_carried_forward(want_j[0], want_j[3])
    wv = w.with_r_fixed(r_fixed)
    got_v = gpu_solve(T, wv, prune)
    key = np.concatenate([w.lam[:, None], r_fixed], axis=1)
    _, first_v, inv_v = np.unique(key, axis=0, return_index=True, return_inverse=True)
    want_vu = oracle.solve(wv.take(first_v), threads=8)
    want_v = tuple(a[inv_v.reshape(-1)] for a in want_vu)
    assert_same(got_v, want_v)
    assert (want_v[0] == 0).any()


# ------------------------------------------------------------ call protocol
def test_stage_calls_equal_whole_solve(T):
    w = wl.workload(1, 130)
    b = T.DeviceBatch(w)
    b.solve()
    whole = b.results()
    b2 = T.DeviceBatch(w)
    T.themis_stage_candidates(b2.p, b2.coef, b2.lam, b2.slo_us, None, b2.workspace)
    T.themis_stage_minplus(b2.p, b2.workspace)
    T.themis_stage_backtrack(b2.p, b2.status, b2.cost, b2.ticks, b2.cfg, b2.workspace)
    assert_same(b2.results(), whole)


def test_repeated_calls_reuse_workspace(T, oracle):
    """Same buffers, different inputs, back to back: no state may leak."""
    import torch
    w = wl.workload(1, 64)
    b = T.DeviceBatch(w)
    b.workspace.fill_(0xAB)
    b.solve()
    first = b.results()
    w2 = wl.workload(1, 128).take(np.arange(64, 128))
    b.coef.copy_(torch.from_numpy(w2.coef))
    b.lam.copy_(torch.from_numpy(w2.lam))
    b.slo_us.copy_(torch.from_numpy(w2.slo_us))
    b.solve()
    second = b.results()
    assert_same(first, oracle.solve(w))
    assert_same(second, oracle.solve(w2))


def test_non_default_stream(T, oracle):
    import torch
    w = wl.workload(0)
    b = T.DeviceBatch(w)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        b.solve(stream=s)
    s.synchronize()
    assert_same(b.results(), oracle.solve(w))


def test_two_solves_in_flight_on_two_streams(T, oracle):
    """Two batches of different shape, each with its own workspace, solved
    concurrently on two streams several times over: nothing in the library is
    shared between calls except read-only tables."""
    import torch
    wa, wb = wl.workload(1, 600), wl.workload(2, 300)
    want_a, want_b = oracle.solve(wa, threads=8), oracle.solve(wb, threads=8)
    print("[case] two streams", wa.name, wb.name, flush=True)
    ba, bb = T.DeviceBatch(wa), T.DeviceBatch(wb, prune=1)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(4):
        ba.solve(stream=sa)
        bb.solve(stream=sb)
    torch.cuda.synchronize()
    assert_same(ba.results(), want_a)
    assert_same(bb.results(), want_b)


def test_argument_errors_launch_nothing(T):
    import ctypes
    w = wl.workload(0, 8)
    b = T.DeviceBatch(w)
    b.status.fill_(77)
    small = b.workspace[:256]
    with pytest.raises(T.ThemisError) as e:
        T.themis_solve_joint(b.p, b.coef, b.lam, b.slo_us, b.status, b.cost, b.ticks, b.cfg, small)
    assert e.value.rc == T.ERR_WORKSPACE
    misaligned = b.workspace[1:]
    with pytest.raises(T.ThemisError) as e:
        T.themis_solve_joint(b.p, b.coef, b.lam, b.slo_us, b.status, b.cost, b.ticks, b.cfg,
                             misaligned)
    assert e.value.rc == T.ERR_WORKSPACE
    rc = T.lib().themis_solve_joint(ctypes.byref(b.p), None, None, None, None, None, None, None,
                                    None, 0, None)
    assert rc == T.ERR_NULL
    rc = T.lib().themis_solve_vertical(ctypes.byref(b.p), b.coef.data_ptr(), b.lam.data_ptr(),
                                       b.slo_us.data_ptr(), None, b.status.data_ptr(),
                                       b.cost.data_ptr(), b.ticks.data_ptr(), b.cfg.data_ptr(),
                                       b.workspace.data_ptr(), b.workspace.numel(), None)
    assert rc == T.ERR_NULL
    import torch
    torch.cuda.synchronize()
    assert (b.status.cpu().numpy() == 77).all()


def test_relaxation_count(T, oracle):
    import torch
    w = wl.workload(1, 50)
    b = T.DeviceBatch(w)
    T.themis_stage_candidates(b.p, b.coef, b.lam, b.slo_us, None, b.workspace)
    cnt = torch.zeros(3, dtype=torch.int64, device="cuda:0")
    T.themis_count_relaxations(b.p, b.workspace, cnt)
    torch.cuda.synchronize()
    lt, _, _ = oracle.candidates(w)
    Ti = (w.slo_us // w.tick_us).astype(np.int64)
    per_model = np.where(lt >= 0, Ti[:, None, None] + 1 - lt, 0).sum(axis=2)     # [N][S]
    # The last model of the pipeline (a running minimum over its candidates) and
    # the first (only the answer is computed) take no relaxations when they have
    # candidates enough: n * positions >= 24 * wavefronts; this workload's rows (up
    # to 4000 ticks) need four wavefronts, and a batch this small is served by
    # workgroups of twice that.
    n = (lt >= 0).sum(axis=2)
    short = n * (Ti[:, None] // 512 + 1) >= 24 * 8
    skipped = np.zeros_like(short)
    skipped[:, -1] = short[:, -1]
    skipped[:, 0] = short[:, 0]
    want = int(per_model[~skipped].sum())
    assert skipped.any() and not skipped[:, [0, -1]].all()
    assert int(cnt[0].item()) == want
    assert int(cnt[1].item()) == int(n.sum())  # the table holds the feasible candidates
    # cells formed: every row but the first model's where only the answer is computed
    answer_only = np.zeros_like(short)
    answer_only[:, 0] = short[:, 0]
    assert int(cnt[2].item()) == int(((Ti + 1)[:, None] * ~answer_only).sum())
