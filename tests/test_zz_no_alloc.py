"""The entry point that allocates nothing (themis_solve_joint_static): its
outputs must equal themis_solve_joint's, element by element, on two calls in a
row, the second on a smaller batch (the built-in workspace keeps the first
call's contents), and a problem beyond the built-in workspace must be refused
before anything is launched.  Through the C ABI."""

import ctypes

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


def _both(T, w):
    """Results of the workspace-taking solve and of the static one for batch w."""
    import torch
    print(f"[case] static workspace: {w.name} N={w.n_inst}", flush=True)
    b = T.DeviceBatch(w)
    assert T.workspace_bytes(b.p) <= T.STATIC_SCRATCH_BYTES
    b.solve()
    ref = b.results()
    outs = T.alloc_outputs(b.p)
    for t in outs:
        t.fill_(-77)
    vp = ctypes.c_void_p
    rc = T.lib().themis_solve_joint_static(
        ctypes.byref(b.p), vp(b.coef.data_ptr()), vp(b.lam.data_ptr()), vp(b.slo_us.data_ptr()),
        vp(outs[0].data_ptr()), vp(outs[1].data_ptr()), vp(outs[2].data_ptr()),
        vp(outs[3].data_ptr()), vp(torch.cuda.current_stream().cuda_stream))
    assert rc == T.OK
    torch.cuda.synchronize()
    return ref, tuple(t.cpu().numpy() for t in outs)


def test_static_workspace_equals_caller_workspace(T):
    # first a batch with long rows and many models, then a smaller one of another shape
    for w in (wl.workload(1, 700), wl.workload(0, 37)):
        ref, got = _both(T, w)
        for name, r, g in zip(NAMES, ref, got):
            assert np.array_equal(r, g), f"{name} differs on {w.name}"
        assert (ref[0] == 0).any()


def test_static_workspace_refuses_what_does_not_fit(T):
    import torch
    w = wl.workload(1)                       # 4096 pipelines: far beyond the built-in workspace
    p = T.problem_of(w)
    assert T.workspace_bytes(p) > T.STATIC_SCRATCH_BYTES
    dummy = torch.full((4096 * 5 * 5,), 77, dtype=torch.int32, device="cuda:0")
    with pytest.raises(T.ThemisError) as e:
        T.themis_solve_joint_static(p, dummy, dummy, dummy, dummy, dummy, dummy, dummy)
    assert e.value.rc == T.ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert (dummy.cpu().numpy() == 77).all()
