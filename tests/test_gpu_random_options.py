"""GPU parity on random search spaces of realistic size with every option drawn
at random: joint or vertical, queue model, sixth coefficient, pruning, and the
entry point (plain solve, horizontal solve, stability test, fallback solve).
Bit-exact against the CPU checker, through the C ABI."""

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

pytestmark = pytest.mark.gpu

FB = ("status", "cost", "ticks", "cfg", "lambda_v", "status_h", "cost_h", "ticks_h", "cfg_h")


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2407_14843_amd import themis
    themis.lib()
    return themis


def as_joint(w):
    j = w.take(np.arange(w.n_inst))
    j.variant, j.r_fixed = wl.JOINT, None
    return j


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_options(T, oracle, seed):
    rng = np.random.default_rng(seed)
    seen = set()
    refused = 0
    for rep in range(80):
        variant = int(rng.integers(0, 2))
        w = wl.medium_random(rng, variant)
        qm, form, prune = (int(rng.integers(0, 3)), int(rng.integers(0, 2)),
                           int(rng.integers(0, 4)))
        w = w.with_model(qm, rng.integers(0, 3000, size=w.coef.shape[:-1]) if form else None)
        if rng.random() < 0.3:      # overload: exercises the search of the fallback
            w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 20, w.n_inst),
                               1 << 20).astype(np.int32)
        mode = int(rng.integers(0, 4 if variant == wl.VERTICAL else 3))
        print(f"[case] seed {seed} rep {rep} variant {variant} queue {qm} form {form} "
              f"prune {prune} mode {mode} N {w.n_inst} S {w.n_stage} K {w.n_cand}", flush=True)
        if w.n_stage * w.r_max * w.c_max > 32767:
            # totals beyond sixteen bits: the library must refuse, and launch nothing
            import torch
            p = T.problem_of(w, prune)
            assert T.check_problem(p) == T.ERR_RANGE and T.workspace_bytes(p) == 0
            dummy = torch.full((4096,), 77, dtype=torch.int32, device="cuda:0")
            ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
            with pytest.raises(T.ThemisError) as e:
                T.themis_solve_joint(p, dummy, dummy, dummy, dummy, dummy, dummy, dummy, ws)
            assert e.value.rc == T.ERR_RANGE
            torch.cuda.synchronize()
            assert (dummy.cpu().numpy() == 77).all()
            refused += 1
            continue
        seen.add((mode, prune))
        if mode == 0:
            b = T.DeviceBatch(w, prune=prune)
            b.solve()
            got, want = b.results(), oracle.solve(w)
        elif mode == 1:
            j = as_joint(w)
            cores = None
            if rng.random() < 0.5:
                cores = rng.integers(1, w.c_max + 1, size=(w.n_inst, w.n_stage)).astype(np.int32)
            b = T.DeviceBatch(j, prune=prune)
            b.solve_horizontal(cores)
            got = b.results()
            want = oracle.solve(j, c_fixed=np.ones((w.n_inst, w.n_stage), np.int32)
                                if cores is None else cores)
        elif mode == 2:
            j = as_joint(w)
            pred = np.clip(j.lam.astype(np.int64) + rng.integers(-50, 80, j.n_inst), 1,
                           1 << 20).astype(np.int32)
            b = T.DeviceBatch(j, prune=prune)
            stable = b.check_stability(pred)
            got = (stable.cpu().numpy(),) + b.results()
            want = oracle.stability(j, pred)
        else:
            b = T.DeviceBatch(w, prune=prune)
            b.solve_vertical_fallback()
            r, o = b.fallback_results(), oracle.vertical_fallback(w)
            got, want = [r[k] for k in FB], [o[k] for k in FB]
        for x, (g, e) in enumerate(zip(got, want)):
            assert np.array_equal(g, e), f"output {x} differs in rep {rep}"
    assert len(seen) >= 12
    print(f"[case] seed {seed}: {refused} problems refused", flush=True)
