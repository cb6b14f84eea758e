"""The solve entry points only enqueue kernels (no allocation, no
synchronisation, no memset), so a caller may capture them in a HIP graph.
Replays are checked against the eager result, with eager work of the same
library between the replays."""

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_14843_amd import themis
    themis.lib()
    return themis


@pytest.mark.parametrize("prune", [0, 1])
def test_captured_solve_replays(T, oracle, prune):
    import torch
    w = wl.workload(1, 300)
    want = oracle.solve(w, threads=8)
    print(f"[case] graph capture prune={prune}", flush=True)
    b = T.DeviceBatch(w, prune=prune)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        b.solve(stream=s)                      # warm-up outside the capture
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        b.solve(stream=torch.cuda.current_stream())
    other = T.DeviceBatch(wl.workload(0))
    for rep in range(3):
        for t in (b.status, b.cost, b.ticks, b.cfg):
            t.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, got, exp in zip(("status", "cost", "ticks", "cfg"), b.results(), want):
            assert np.array_equal(got, exp), f"replay {rep}: {name} differs"
        other.solve()                          # eager work between the replays
        other.results()


def test_captured_fallback_replays(T, oracle):
    import torch
    w = wl.workload(2, 40)
    w.lam = (w.lam * 4).astype(np.int32)
    want = oracle.vertical_fallback(w, threads=8)
    print("[case] graph capture fallback", flush=True)
    b = T.DeviceBatch(w)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        b.solve_vertical_fallback(stream=s)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        b.solve_vertical_fallback(stream=torch.cuda.current_stream())
    for rep in range(2):
        b.lambda_v.fill_(-7)
        b.status.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = b.fallback_results()
        for k in want:
            assert np.array_equal(got[k], want[k]), f"replay {rep}: {k} differs"


def test_captured_distinct_solve_replays(T, oracle):
    import torch
    rng = np.random.default_rng(5)
    base = wl.workload(1, 40)
    w = base.take(rng.integers(0, base.n_inst, 400))   # most inputs recur
    want = oracle.solve(w, threads=8)
    print("[case] graph capture distinct-instance solve", flush=True)
    b = T.DeviceBatch(w)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        b.solve_distinct(stream=s)             # warm-up (and workspace) outside the capture
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        b.solve_distinct(stream=torch.cuda.current_stream())
    other = T.DeviceBatch(wl.workload(0))
    for rep in range(3):
        for t in (b.status, b.cost, b.ticks, b.cfg):
            t.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, got, exp in zip(("status", "cost", "ticks", "cfg"), b.results(), want):
            assert np.array_equal(got, exp), f"replay {rep}: {name} differs"
        other.solve()                          # eager work between the replays
        other.results()
