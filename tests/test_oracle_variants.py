"""Pins for the checker's paper-form model options: the queue of Eq. 4 and of
Eq. 3, and Eq. 1's delta*b term.  Expected values are hand-derived
(tests/golden/worked_examples.json), exact rational arithmetic on Eq. 1 as
printed, or the exhaustive enumeration (which has its own arithmetic)."""

import json
import os
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def _mk(coef_rows, lam, slo_us, c_max, batch_sizes, r_max, tick, queue_model, form):
    coef = np.asarray(coef_rows, np.int32)[None, :, :]
    return wl.Workload("t", wl.JOINT, 1, coef.shape[1], c_max, list(batch_sizes), r_max, tick,
                       max(slo_us, 1), False, coef, np.array([lam], np.int32),
                       np.array([slo_us], np.int32), queue_model=queue_model,
                       profile_form=form)


@pytest.mark.parametrize("queue_model", [1, 2])
def test_paper_forms_worked_example(oracle, queue_model):
    """Catches: delta*b divided by the cores or dropped, queue still scaled by
    the instance count, Eq. 3's busy term with the wrong sign."""
    g = json.load(open(GOLDEN))["paper_forms_one_stage"]
    for sv in g["solves"]:
        w = _mk([g["coef"]] * sv["n_stage"], g["lambda"], sv["slo_us"], g["c_max"],
                g["batch_sizes"], g["r_max"], g["tick_us"], queue_model, 1)
        st, cost, ticks, cfg = oracle.solve(w)
        assert (int(st[0]), int(cost[0]), int(ticks[0]), cfg[0].tolist()) == \
            (sv["status"], sv["cost"], sv["ticks"], sv["cfg"])
        rc, bc, bt, bcfg, _ = oracle.bruteforce(w, 0)
        assert (rc, bc, bt, bcfg.tolist()) == (sv["status"], sv["cost"], sv["ticks"], sv["cfg"])
    w = _mk([g["coef"]], g["lambda"], 10_000_000, g["c_max"], g["batch_sizes"], g["r_max"],
            g["tick_us"], queue_model, 1)
    lt, cost, r = oracle.candidates(w)
    nb = len(g["batch_sizes"])
    for cd in g["candidates"]:
        k = (cd["c"] - 1) * nb + g["batch_sizes"].index(cd["b"])
        if cd.get("feasible", True):
            assert (lt[0, 0, k], cost[0, 0, k], r[0, 0, k]) == (cd["lt"], cd["cost"], cd["r"])
            assert cd["lt"] == -(-(cd["proc"] + cd["queue"]) // g["tick_us"])
        else:
            assert lt[0, 0, k] == -1
    # the default queue on the same coefficients gives the other, larger waits
    w.queue_model = 0
    lt0 = oracle.candidates(w)[0]
    assert (lt0[0, 0, 1], lt0[0, 0, 3]) == (g["default_queue_lt"]["c1b2"], g["default_queue_lt"]["c2b2"])


def test_eq1_as_printed(oracle):
    """With no core cap in reach, no quadratic term, a 1 us grid and batch 1
    (no queueing), the tick count of a candidate is Eq. 1 itself rounded up:
    ceil((gamma*b + epsilon)/c) + delta*b + eta, in exact rationals."""
    rng = np.random.default_rng(1)
    for _ in range(50):
        eps, gam, dlt, eta = (int(rng.integers(lo, hi)) for lo, hi in
                              ((0, 30000), (0, 6000), (0, 3000), (1, 2000)))
        c_max = int(rng.integers(1, 9))
        bs = sorted(set(int(x) for x in rng.integers(1, 17, 4)))
        lam = int(rng.integers(1, 3000))
        w = _mk([[eps, gam, 0, c_max, eta, dlt]], lam, 50_000_000, c_max, bs, 32767, 1, 1, 1)
        lt, cost, r = oracle.candidates(w)
        for c in range(1, c_max + 1):
            for j, b in enumerate(bs):
                proc = ceil(Fraction(gam * b + eps, c)) + dlt * b + eta
                n = max(1, ceil(Fraction(lam * proc, b * 10**6)))
                want = proc + ceil(Fraction((b - 1) * 10**6, lam))
                k = (c - 1) * len(bs) + j
                assert (lt[0, 0, k], r[0, 0, k], cost[0, 0, k]) == (want, n, n * c)


@pytest.mark.parametrize("variant", [wl.JOINT, wl.VERTICAL])
@pytest.mark.parametrize("queue_model,form", [(1, 0), (2, 1), (0, 1)])
def test_variants_match_enumeration(oracle, variant, queue_model, form):
    rng = np.random.default_rng(100 + 10 * queue_model + form)
    solved = 0
    for _ in range(25):
        w = wl.tiny_random(rng, variant, 10, 3)
        d = rng.integers(0, 2500, size=w.coef.shape[:-1]) if form else None
        w = w.with_model(queue_model, d)
        st, cost, ticks, cfg = oracle.solve(w)
        for i in range(w.n_inst):
            rc, bc, bt, bcfg, _ = oracle.bruteforce(w, i)
            assert (int(st[i]), int(cost[i]), int(ticks[i]), cfg[i].tolist()) == \
                (rc, bc, bt, bcfg.tolist())
            solved += rc == 0
    assert solved > 60


def test_eq3_equals_eq4_under_the_throughput_constraint(oracle):
    """Section 4.2's argument for dropping Eq. 3's second term: once
    n*h >= lambda it is negative.  The two options must therefore agree on
    every candidate table and every solve."""
    rng = np.random.default_rng(9)
    for rep in range(30):
        w = wl.tiny_random(rng, rep % 2, 12, 3)
        d = rng.integers(0, 2500, size=w.coef.shape[:-1])
        a, b = w.with_model(1, d), w.with_model(2, d)
        for x, y in zip(oracle.candidates(a), oracle.candidates(b)):
            assert (x == y).all()
        for x, y in zip(oracle.solve(a), oracle.solve(b)):
            assert (x == y).all()


def test_shared_queue_never_costs_more(oracle):
    """Eq. 4's wait is at most the per-replica wait, so every candidate stays
    feasible with no more ticks, and the optimum cannot get worse; a zero
    sixth coefficient changes nothing."""
    rng = np.random.default_rng(10)
    better = 0
    for rep in range(30):
        w = wl.tiny_random(rng, rep % 2, 12, 3)
        s0, c0, _, _ = oracle.solve(w)
        s1, c1, _, _ = oracle.solve(w.with_model(1))
        assert ((s0 == 0) <= (s1 == 0)).all()
        both = (s0 == 0) & (s1 == 0)
        assert (c1[both] <= c0[both]).all()
        better += int((c1[both] < c0[both]).sum() + ((s0 == 1) & (s1 == 0)).sum())
        z = w.with_model(0, np.zeros(w.coef.shape[:-1], np.int32))
        for x, y in zip(oracle.solve(w), oracle.solve(z)):
            assert (x == y).all()
    assert better > 5


def test_sixth_coefficient_out_of_range_is_invalid(oracle):
    rng = np.random.default_rng(4)
    w = wl.tiny_random(rng, wl.JOINT, 4, 2)
    d = np.zeros(w.coef.shape[:-1], np.int32)
    d[1, 0] = -1
    d[2, 1] = (1 << 20) + 1
    st = oracle.solve(w.with_model(0, d))[0]
    assert st[1] == 2 and st[2] == 2 and st[0] != 2 and st[3] != 2
