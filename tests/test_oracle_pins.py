"""Pins for the CPU checker: things the paper and the mathematics fix.

None of these compares the checker with itself or with the GPU path.  Each
test names the mistake it is meant to catch.
"""

import itertools
import json
import os

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def _mk(variant, coef_rows, lam, slo_us, c_max, batch_sizes, r_max, tick, r_fixed=None):
    coef = np.asarray(coef_rows, np.int32)[None, :, :]
    S = coef.shape[1]
    rf = None if r_fixed is None else np.asarray(r_fixed, np.int32).reshape(1, S)
    return wl.Workload("t", variant, 1, S, c_max, list(batch_sizes), r_max, tick,
                       max(slo_us, 1), False, coef, np.array([lam], np.int32),
                       np.array([slo_us], np.int32), r_fixed=rf)


# ---------------------------------------------------------------- worked examples
@pytest.mark.parametrize("case", ["joint_one_stage", "vertical_one_stage"])
def test_worked_examples(oracle, case):
    """Hand-derived candidate values and answers (tests/golden/worked_examples.json).

    Catches: wrong rounding direction, queue delay not scaled by the replica
    count, core cap p ignored, floor instead of ceil in the instance count,
    latency-before-cost tie order, lexicographic order reversed.
    """
    g = json.load(open(GOLDEN))[case]
    vert = "r_fixed" in g
    for sv in g["solves"]:
        S = sv["n_stage"]
        w = _mk(wl.VERTICAL if vert else wl.JOINT, [g["coef"]] * S, g["lambda"],
                sv["slo_us"], g["c_max"], g["batch_sizes"], g["r_max"], g["tick_us"],
                r_fixed=[g["r_fixed"]] * S if vert else None)
        st, cost, ticks, cfg = oracle.solve(w)
        assert (int(st[0]), int(cost[0]), int(ticks[0])) == (sv["status"], sv["cost"], sv["ticks"])
        assert cfg[0].tolist() == sv["cfg"]
        rc, bc, bt, bcfg, _ = oracle.bruteforce(w, 0)
        assert (rc, bc, bt, bcfg.tolist()) == (sv["status"], sv["cost"], sv["ticks"], sv["cfg"])
    # candidate table at an SLO loose enough that nothing is cut by the budget
    w = _mk(wl.VERTICAL if vert else wl.JOINT, [g["coef"]], g["lambda"], 10_000_000,
            g["c_max"], g["batch_sizes"], g["r_max"], g["tick_us"],
            r_fixed=[g["r_fixed"]] if vert else None)
    lt, cost, r = oracle.candidates(w)
    nb = len(g["batch_sizes"])
    for cd in g["candidates"]:
        k = (cd["c"] - 1) * nb + g["batch_sizes"].index(cd["b"])
        if cd.get("feasible", True):
            assert (lt[0, 0, k], cost[0, 0, k], r[0, 0, k]) == (cd["lt"], cd["cost"], cd["r"])
            assert cd["lt"] == -(-(cd["proc"] + cd["queue"]) // g["tick_us"])
        else:
            assert (lt[0, 0, k], cost[0, 0, k], r[0, 0, k]) == (-1, -1, -1)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("variant", [wl.JOINT, wl.VERTICAL])
def test_matches_exhaustive_enumeration(oracle, variant):
    """DP vs explicit enumeration of Eq. 6 on tiny random pipelines.

    The enumeration walks the replica count explicitly and tests both
    constraints on whole assignments, so it also checks that deriving the
    replica count per candidate loses nothing, and that "infeasible" is
    reported exactly when no assignment exists.
    """
    rng = np.random.default_rng(20240714 + variant)
    n_feas = n_infeas = n_multi = 0
    for _ in range(1500):
        w = wl.tiny_random(rng, variant)
        st, cost, ticks, cfg = oracle.solve(w)
        rc, bc, bt, bcfg, visited = oracle.bruteforce(w, 0)
        assert rc == st[0], (w, rc, st[0])
        assert (bc, bt) == (cost[0], ticks[0])
        assert bcfg.tolist() == cfg[0].tolist()
        n_feas += rc == 0
        n_infeas += rc == 1
        n_multi += (rc == 0 and w.n_stage >= 3)
    # the sample must exercise both outcomes and multi-stage pipelines
    assert n_feas > 300 and n_infeas > 300 and n_multi > 100


def test_python_enumeration_agrees(oracle):
    """A second, pure-Python enumeration (itertools) on very small cases.

    Guards the C enumerator itself: same definition, different language and
    loop structure (flat product + sort key).
    """
    rng = np.random.default_rng(77)
    for _ in range(150):
        w = wl.tiny_random(rng, wl.JOINT, max_stage=2)
        lam, slo, tick = int(w.lam[0]), int(w.slo_us[0]), w.tick_us
        T = slo // tick
        per_stage = []
        for s in range(w.n_stage):
            a, k, q, p, o = (int(x) for x in w.coef[0, s])
            opts = []
            for c, b, n in itertools.product(range(1, w.c_max + 1), w.batch_sizes,
                                             range(1, w.r_max + 1)):
                proc = -(-(a + k * b + q * b * b) // min(c, p)) + o
                if lam * proc > n * b * 10**6:
                    continue
                queue = -(-((b - 1) * 10**6 * n) // lam)
                opts.append((n * c, -(-(proc + queue) // tick), (c, b, n)))
            per_stage.append(opts)
        best = None
        for combo in itertools.product(*per_stage):
            ticks = sum(x[1] for x in combo)
            if ticks > T:
                continue
            key = (sum(x[0] for x in combo), ticks, tuple(x[2] for x in combo))
            if best is None or key < best:
                best = key
        rc, bc, bt, bcfg, _ = oracle.bruteforce(w, 0)
        if best is None:
            assert rc == 1
        else:
            assert (rc, bc, bt) == (0, best[0], best[1])
            assert [tuple(r) for r in bcfg.tolist()] == list(best[2])


# ---------------------------------------------------------------- closed forms
def test_loose_slo_is_separable(oracle):
    """With a budget no model can exhaust, the optimum is each model's cheapest
    candidate on its own (sum of per-stage minima).  Catches a DP that couples
    stages wrongly or drops a stage."""
    w = wl.workload(1, 48)
    w.slo_us[:] = w.slo_max_us = 2_000_000_000 // 4
    w.tick_us = 50_000
    lt, cost, _ = oracle.candidates(w)
    st, c, _, _ = oracle.solve(w)
    feas = lt >= 0
    assert feas.any(axis=2).all()
    big = np.where(feas, cost, np.iinfo(np.int32).max)
    T = w.slo_us // w.tick_us
    assert (np.where(feas, lt, 0).max(axis=2).sum(axis=1) <= T).all()
    assert (st == 0).all()
    assert (c == big.min(axis=2).sum(axis=1)).all()


def test_single_stage_is_plain_argmin(oracle):
    """One model: the answer is the candidate with the least (cost, lt, index)."""
    w = wl.workload(0)
    w1 = wl.Workload("s1", wl.JOINT, w.n_inst, 1, w.c_max, w.batch_sizes, w.r_max,
                     w.tick_us, w.slo_max_us, False,
                     np.ascontiguousarray(w.coef[:, :1]), w.lam, w.slo_us // 12)
    lt, cost, r = oracle.candidates(w1)
    st, c, tk, cfg = oracle.solve(w1)
    nb = len(w1.batch_sizes)
    seen = set()
    for i in range(w1.n_inst):
        ks = [k for k in range(w1.n_cand) if lt[i, 0, k] >= 0]
        if not ks:
            assert st[i] == 1
            seen.add(1)
            continue
        k = min(ks, key=lambda k: (cost[i, 0, k], lt[i, 0, k], k))
        assert (st[i], c[i], tk[i]) == (0, cost[i, 0, k], lt[i, 0, k])
        assert cfg[i, 0].tolist() == [k // nb + 1, w1.batch_sizes[k % nb], r[i, 0, k]]
        seen.add(0)
    assert seen == {0, 1}


def test_cost_matches_milp(oracle):
    """The solve is a multiple-choice knapsack (one candidate per model, weights
    lt, capacity T, minimise cost): scipy's MILP solver must find the same
    optimal cost.  A library routine the checker does not use."""
    from scipy.optimize import Bounds, LinearConstraint, milp

    w = wl.workload(1, 12)
    w.slo_us[:] = w.slo_us // 3      # tighten so the budget binds
    lt, cost, _ = oracle.candidates(w)
    st, c, _, _ = oracle.solve(w)
    S, K = w.n_stage, w.n_cand
    checked = 0
    for i in range(w.n_inst):
        feas = lt[i] >= 0
        if not feas.any(axis=1).all():
            assert st[i] == 1
            continue
        idx = [(s, k) for s in range(S) for k in range(K) if feas[s, k]]
        cvec = np.array([cost[i, s, k] for s, k in idx], float)
        pick = np.zeros((S, len(idx)))
        for j, (s, _) in enumerate(idx):
            pick[s, j] = 1
        wrow = np.array([[lt[i, s, k] for s, k in idx]], float)
        res = milp(cvec, integrality=np.ones(len(idx)), bounds=Bounds(0, 1),
                   constraints=[LinearConstraint(pick, 1, 1),
                                LinearConstraint(wrow, 0, int(w.slo_us[i] // w.tick_us))])
        if res.status == 2:      # infeasible
            assert st[i] == 1
        else:
            assert res.status == 0 and st[i] == 0
            assert round(res.fun) == c[i]
            checked += 1
    assert checked >= 6


# ---------------------------------------------------------------- invariants
def test_cost_monotone_in_slo(oracle):
    """More budget never costs more, and never turns feasible into infeasible."""
    base = wl.workload(1, 8)
    prev_cost = None
    for scale in (0.05, 0.1, 0.2, 0.35, 0.5, 0.75, 1.0):
        w = base.head(8)
        w.slo_us = (base.slo_us * scale).astype(np.int32)
        st, c, _, _ = oracle.solve(w)
        cur = np.where(st == 0, c, 10**9)
        if prev_cost is not None:
            assert (cur <= prev_cost).all()
        prev_cost = cur
    assert (prev_cost < 10**9).all()


def test_tick_refinement(oracle):
    """A finer grid (tick dividing the coarse tick) admits a superset of the
    coarse grid's configurations, so it is never more expensive."""
    rng = np.random.default_rng(5)
    base = wl.workload(0)
    base.slo_us = (base.slo_us // 3).astype(np.int32)
    costs = {}
    for tick in (4000, 2000, 1000, 500, 250):
        w = base.head(64)
        w.tick_us = tick
        st, c, _, _ = oracle.solve(w)
        costs[tick] = np.where(st == 0, c, 10**9)
    ticks = sorted(costs, reverse=True)
    for coarse, fine in zip(ticks, ticks[1:]):
        assert (costs[fine] <= costs[coarse]).all()
    assert (costs[4000] != costs[250]).any()


def test_joint_not_worse_than_vertical(oracle):
    """If the fixed-replica problem is feasible with replicas within r_max, the
    joint problem is feasible and at most as expensive."""
    w = wl.workload(2, 64)
    wj = wl.Workload("j", wl.JOINT, w.n_inst, w.n_stage, w.c_max, w.batch_sizes, 4,
                     w.tick_us, w.slo_max_us, False, w.coef, w.lam, w.slo_us)
    sv, cv, _, _ = oracle.solve(w)
    sj, cj, _, _ = oracle.solve(wj)
    feas = sv == 0
    assert feas.sum() > 10
    assert (sj[feas] == 0).all()
    assert (cj[feas] <= cv[feas]).all()


def test_stage_permutation_invariance(oracle):
    """Reordering the models changes neither feasibility, cost nor ticks."""
    w = wl.workload(1, 24)
    w.slo_us = (w.slo_us // 3).astype(np.int32)
    st, c, tk, _ = oracle.solve(w)
    perm = np.array([3, 0, 4, 2, 1])
    w2 = w.head(24)
    w2.coef = np.ascontiguousarray(w.coef[:, perm])
    st2, c2, tk2, _ = oracle.solve(w2)
    assert (st == st2).all() and (c == c2).all() and (tk == tk2).all()
    assert set(st.tolist()) == {0, 1} or (st == 0).all()


def test_batch_one_cost_monotone_in_lambda(oracle):
    """With batch size 1 only there is no queueing term, so a higher arrival
    rate can only need more replicas: cost is non-decreasing in lambda."""
    base = wl.workload(0)
    prev = None
    for lam in (5, 10, 20, 50, 100, 200, 400):
        w = wl.Workload("b1", wl.JOINT, base.n_inst, base.n_stage, base.c_max, [1],
                        base.r_max, base.tick_us, base.slo_max_us, False, base.coef,
                        np.full(base.n_inst, lam, np.int32), base.slo_us)
        st, c, _, _ = oracle.solve(w)
        cur = np.where(st == 0, c, 10**9)
        if prev is not None:
            assert (cur >= prev).all()
        prev = cur


# ---------------------------------------------------------------- forward sparse DP
def _prefix_states(w, i, lt, cost):
    """Eq. 6 by prefixes: after model s, the set of reachable exact latency sums of
    models 0..s, each with the least total cores that reaches it (a dictionary,
    grown model by model from the candidate tables; sums beyond the budget are
    dropped).  The answer is the least total over the final set and, among the
    sums attaining it, the least."""
    T = int(w.slo_us[i]) // w.tick_us
    states = {0: 0}
    for s in range(w.n_stage):
        options = [(int(l), int(c)) for l, c in zip(lt[i, s], cost[i, s]) if l >= 0]
        grown = {}
        for spent, total in states.items():
            for l, c in options:
                if spent + l <= T and total + c < grown.get(spent + l, 10**9):
                    grown[spent + l] = total + c
        states = grown
    if not states:
        return (1, -1, -1)
    least = min(states.values())
    return (0, least, min(t for t, c in states.items() if c == least))


def test_forward_sparse_dp_agrees(oracle):
    """The checker's suffix recurrence over dense rows against a forward recurrence
    over sparse sets of prefix sums: structurally unlike it (other direction,
    other state representation), same optimum and same least latency."""
    w = wl.workload(0)
    w.slo_us = (w.slo_us // 3).astype(np.int32)
    lt, cost, _ = oracle.candidates(w)
    st, c, tk, _ = oracle.solve(w)
    for i in range(w.n_inst):
        assert _prefix_states(w, i, lt, cost) == (st[i], c[i], tk[i])
    assert set(st.tolist()) == {0, 1}


# ---------------------------------------------------------------- interface rules
def test_invalid_inputs_flagged(oracle):
    w = wl.workload(0, 8)
    w.lam[1] = 0
    w.slo_us[2] = -5
    w.coef[3, 1, 4] = 0          # o < 1
    w.coef[4, 0, 3] = 0          # p < 1
    w.coef[5, 2, 0] = -1         # a < 0
    w.slo_us[6] = w.slo_max_us + 1
    st, c, tk, cfg = oracle.solve(w)
    assert st.tolist() == [0, 2, 2, 2, 2, 2, 2, 0]
    assert (c[1:7] == -1).all() and (tk[1:7] == -1).all() and (cfg[1:7] == 0).all()
    lt, cost, r = oracle.candidates(w)
    assert (lt[1:7] == -1).all()


def test_solution_is_consistent_with_tables(oracle):
    """Every reported configuration re-evaluates to the reported cost and ticks."""
    w = wl.workload(1, 32)
    lt, cost, r = oracle.candidates(w)
    st, c, tk, cfg = oracle.solve(w)
    nb = len(w.batch_sizes)
    for i in np.nonzero(st == 0)[0]:
        ks = [(cfg[i, s, 0] - 1) * nb + w.batch_sizes.index(int(cfg[i, s, 1]))
              for s in range(w.n_stage)]
        assert sum(cost[i, s, k] for s, k in enumerate(ks)) == c[i]
        assert sum(lt[i, s, k] for s, k in enumerate(ks)) == tk[i]
        assert all(r[i, s, k] == cfg[i, s, 2] for s, k in enumerate(ks))
        assert tk[i] <= w.slo_us[i] // w.tick_us
