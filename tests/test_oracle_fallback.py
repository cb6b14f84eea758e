"""Pins for the checker's version of Algorithm 1's fallback (Section 4.4):
binary search on the arrival rate when the given replicas cannot meet the SLO,
then new instances for the remaining rate with the cores kept.

Nothing here compares the checker with itself or with the GPU path: expected
values are hand-traced (tests/golden/fallback_example.json) or come from the
exhaustive enumeration, which has no dynamic program and no search in it.
"""

import json
import os

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fallback_example.json")


def _one(coef_rows, lam, slo_us, c_max, batch_sizes, r_max, tick, r_fixed):
    coef = np.asarray(coef_rows, np.int32)[None, :, :]
    S = coef.shape[1]
    return wl.Workload("t", wl.VERTICAL, 1, S, c_max, list(batch_sizes), r_max, tick,
                       max(slo_us, 1), False, coef, np.array([lam], np.int32),
                       np.array([slo_us], np.int32),
                       r_fixed=np.asarray(r_fixed, np.int32).reshape(1, S))


def test_hand_traced_fallback(oracle):
    """Catches: midpoint taken as (right-left)//2, branches swapped (a feasible
    midpoint must raise the lower end), result taken at `right`, remainder
    solved with free cores or with the replicas still pinned, remainder rate
    not reduced by the absorbed rate."""
    g = json.load(open(GOLDEN))
    for cs in g["cases"]:
        w = _one([g["coef"]], cs["lambda"], g["slo_us"], g["c_max"], g["batch_sizes"],
                 g["r_max"], g["tick_us"], [g["r_fixed"]])
        out = oracle.vertical_fallback(w)
        for key in ("status", "lambda_v", "cost", "ticks", "status_h", "cost_h", "ticks_h"):
            assert int(out[key][0]) == cs[key], (cs["lambda"], key)
        assert out["cfg"][0].tolist() == cs["cfg"]
        assert out["cfg_h"][0].tolist() == cs["cfg_h"]
    nv = g["never"]
    w = _one([g["coef"]], nv["lambda"], nv["slo_us"], g["c_max"], g["batch_sizes"],
             g["r_max"], g["tick_us"], [g["r_fixed"]])
    out = oracle.vertical_fallback(w)
    assert (int(out["status"][0]), int(out["lambda_v"][0]), int(out["status_h"][0])) == \
        (nv["status"], nv["lambda_v"], nv["status_h"])
    assert int(out["cost"][0]) == -1 and not out["cfg"][0].any() and not out["cfg_h"][0].any()


def test_pinned_cores_match_enumeration(oracle):
    """The remainder solve (cores given, instance count and batch free) against
    the exhaustive walk with the same cores pinned.  Catches: pin applied to the
    wrong model, pinned candidate still competing with others, pin ignored."""
    rng = np.random.default_rng(11)
    n_solved = 0
    for _ in range(40):
        w = wl.tiny_random(rng, wl.JOINT, 12, 3)
        cfx = rng.integers(1, w.c_max + 1, size=(w.n_inst, w.n_stage)).astype(np.int32)
        st, cost, ticks, cfg = oracle.solve(w, c_fixed=cfx)
        for i in range(w.n_inst):
            rc, bc, bt, bcfg, _ = oracle.bruteforce(w, i, c_fixed=cfx[i])
            assert (int(st[i]), int(cost[i]), int(ticks[i])) == (rc, bc, bt)
            assert cfg[i].tolist() == bcfg.tolist()
            if rc == 0:
                assert cfg[i][:, 0].tolist() == cfx[i].tolist()
                n_solved += 1
    assert n_solved > 100


def _vertical_feasible(oracle, w, i, lam):
    wi = w.take(np.array([i]))
    wi.lam = np.array([lam], np.int32)
    return oracle.bruteforce(wi, 0)


def test_fallback_invariants_by_enumeration(oracle):
    """What any correct run of the search must leave behind, checked by
    enumeration: the returned vertical configuration is the optimum at
    lambda_v; lambda_v + 1 is not absorbable (the search ends with right =
    left + 1 and `right` only ever holds rates that failed) unless lambda_v is
    lambda itself; the new instances are the optimum for lambda - lambda_v
    with the vertical cores."""
    rng = np.random.default_rng(5)
    seen = {"outright": 0, "split": 0, "split_h_ok": 0, "none": 0}
    for _ in range(60):
        w = wl.tiny_random(rng, wl.VERTICAL, 10, 3)
        # push the rates up so that the given replicas are often not enough
        w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 12, w.n_inst),
                           1 << 20).astype(np.int32)
        out = oracle.vertical_fallback(w)
        for i in range(w.n_inst):
            lam, lv = int(w.lam[i]), int(out["lambda_v"][i])
            rc0, *_ = _vertical_feasible(oracle, w, i, lam)
            if rc0 == 0:
                assert lv == lam and out["status"][i] == 0 and out["status_h"][i] == 0
                assert out["cost_h"][i] == 0 and not out["cfg_h"][i].any()
                seen["outright"] += 1
                continue
            if lv == 0:
                assert out["status"][i] == 1 and out["status_h"][i] == 2
                assert _vertical_feasible(oracle, w, i, 1)[0] == 1
                seen["none"] += 1
                continue
            assert 1 <= lv < lam and out["status"][i] == 0
            rc, bc, bt, bcfg, _ = _vertical_feasible(oracle, w, i, lv)
            assert (rc, bc, bt) == (0, int(out["cost"][i]), int(out["ticks"][i]))
            assert bcfg.tolist() == out["cfg"][i].tolist()
            assert _vertical_feasible(oracle, w, i, lv + 1)[0] == 1
            # the remainder: joint over (batch, instances) with the cores kept
            wi = w.take(np.array([i]))
            wi.lam = np.array([lam - lv], np.int32)
            wi.r_fixed = None
            wi.variant = wl.JOINT
            rc, bc, bt, bcfg, _ = oracle.bruteforce(wi, 0, c_fixed=out["cfg"][i][:, 0])
            assert (rc, bc, bt) == (int(out["status_h"][i]), int(out["cost_h"][i]),
                                    int(out["ticks_h"][i]))
            assert bcfg.tolist() == out["cfg_h"][i].tolist()
            seen["split"] += 1
            seen["split_h_ok"] += rc == 0
    assert min(seen.values()) > 10, seen


def test_fallback_invalid_inputs(oracle):
    """Invalid instances are flagged in both halves and leave nothing behind."""
    rng = np.random.default_rng(3)
    w = wl.tiny_random(rng, wl.VERTICAL, 6, 2)
    w.lam[1] = 0
    w.r_fixed[3, 0] = w.r_max + 1
    out = oracle.vertical_fallback(w)
    for i in (1, 3):
        assert out["status"][i] == 2 and out["status_h"][i] == 2 and out["lambda_v"][i] == 0
        assert not out["cfg"][i].any() and not out["cfg_h"][i].any()


# ---------------------------------------------------------------- stability test
def _joint(coef_rows, lam, slo_us, c_max, batch_sizes, r_max, tick):
    coef = np.asarray(coef_rows, np.int32)[None, :, :]
    return wl.Workload("t", wl.JOINT, 1, coef.shape[1], c_max, list(batch_sizes), r_max, tick,
                       max(slo_us, 1), False, coef, np.array([lam], np.int32),
                       np.array([slo_us], np.int32))


def test_hand_derived_stability(oracle):
    """Catches: comparing instance counts only (batch ignored), calling two
    failed solves 'the same', solving with free cores instead of one core."""
    g = json.load(open(GOLDEN))
    for cs in g["stability"]["cases"]:
        w = _joint([g["coef"]], cs["now"], cs["slo_us"], g["c_max"], g["batch_sizes"],
                   g["r_max"], g["tick_us"])
        stable, st, cost, ticks, cfg = oracle.stability(w, np.array([cs["pred"]], np.int32))
        assert int(stable[0]) == cs["stable"], cs
        assert cfg[0].tolist() == cs["cfg_now"]


def test_stability_by_enumeration(oracle):
    """stable <=> the exhaustive optimum with the cores pinned exists at both
    rates and is the same triple for every model."""
    rng = np.random.default_rng(8)
    n_stable = n_unstable = 0
    for rep in range(40):
        w = wl.tiny_random(rng, wl.JOINT, 12, 3)
        # predicted rate close to the current one, so that both outcomes occur
        pred = np.clip(w.lam.astype(np.int64) + rng.integers(-30, 60, w.n_inst), 1, 1 << 20)
        cores = None if rep % 2 else rng.integers(1, w.c_max + 1,
                                                  size=(w.n_inst, w.n_stage)).astype(np.int32)
        stable, st, cost, ticks, cfg = oracle.stability(w, pred.astype(np.int32), cores)
        for i in range(w.n_inst):
            cx = np.ones(w.n_stage, np.int32) if cores is None else cores[i]
            a = oracle.bruteforce(w, i, c_fixed=cx)
            wp = w.take(np.array([i]))
            wp.lam = np.array([pred[i]], np.int32)
            b = oracle.bruteforce(wp, 0, c_fixed=cx)
            want = int(a[0] == 0 and b[0] == 0 and a[3].tolist() == b[3].tolist())
            assert int(stable[i]) == want
            assert (int(st[i]), int(cost[i]), int(ticks[i])) == a[:3]
            assert cfg[i].tolist() == a[3].tolist()
            n_stable += want
            n_unstable += 1 - want
    assert n_stable > 30 and n_unstable > 30, (n_stable, n_unstable)


def test_given_cores_out_of_range_are_invalid(oracle):
    rng = np.random.default_rng(2)
    w = wl.tiny_random(rng, wl.JOINT, 5, 2)
    cores = np.ones((w.n_inst, w.n_stage), np.int32)
    cores[1, 0] = 0
    cores[3, -1] = w.c_max + 1
    st = oracle.solve(w, c_fixed=cores)[0]
    assert st[1] == 2 and st[3] == 2 and (st[[0, 2, 4]] != 2).all()


def test_replicas_given_latency_never_grows_with_cores(oracle):
    """With the replicas given, more cores never slow a candidate down and never
    make a feasible one infeasible (Eq. 1 divides by the cores; none of the
    queue terms of Eqs. 3-4 grows).  Hence the replicas can absorb a rate
    exactly when the fastest candidates of all models fit the budget together,
    which is what a search on the rate may test instead of solving the whole
    recurrence.  Checked on the checker's own candidate tables and statuses,
    under every queue model and both profile forms."""
    rng = np.random.default_rng(77)
    seen = np.zeros(2, int)
    for rep in range(60):
        w = wl.medium_random(rng, wl.VERTICAL)
        if rep % 2:
            w.lam = np.minimum(w.lam.astype(np.int64) * rng.integers(1, 8, w.n_inst),
                               1 << 20).astype(np.int32)
        d = rng.integers(0, 2000, size=w.coef.shape[:-1]) if rep % 3 == 0 else None
        w = w.with_model(rep % 3, d)
        lt, _, _ = oracle.candidates(w)
        status = oracle.solve(w)[0]
        nb = len(w.batch_sizes)
        lt = lt.reshape(w.n_inst, w.n_stage, w.c_max, nb).astype(np.int64)
        big = np.int64(1) << 40
        filled = np.where(lt < 0, big, lt)
        # along the cores axis: non-increasing, and infeasible only below feasible
        assert (np.diff(filled, axis=2) <= 0).all()
        fastest = filled[:, :, -1, :].min(axis=2)          # at the largest core count
        assert (fastest == filled.min(axis=(2, 3))).all()
        T = w.slo_us.astype(np.int64) // w.tick_us
        fits = (fastest < big).all(axis=1) & (np.where(fastest < big, fastest, 0).sum(axis=1) <= T)
        valid = status != 2
        assert ((status == 0) == fits)[valid].all()
        seen += [(status == 0).sum(), (status == 1).sum()]
    assert (seen > 50).all(), seen
