"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer.

oracle/*.c is compiled with -fsanitize=address,undefined into a small host
program (tests/host/oracle_sanitized.c) that replays a file of cases: the
hand-worked examples of tests/golden/ with their expected answers, tiny random
pipelines that it compares with the exhaustive enumeration, and instances at the
limits of the accepted input ranges (the largest intermediates).  Any memory
error or undefined arithmetic in the checker ends the program with a report.
"""
import json
import os
import shutil
import subprocess

import numpy as np
import pytest

from paper_2407_14843_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden", "worked_examples.json")


def _case(w, enumerate_all, expected=None):
    out = [w.variant, w.queue_model, w.profile_form, w.n_stage, w.c_max, len(w.batch_sizes)]
    out += list(w.batch_sizes)
    out += [w.r_max, w.tick_us, w.slo_max_us, w.n_inst, int(enumerate_all), int(expected is not None)]
    parts = [np.asarray(out, np.int32), w.coef.reshape(-1), w.lam, w.slo_us]
    if w.variant == wl.VERTICAL:
        parts.append(w.r_fixed.reshape(-1))
    if expected is not None:
        parts += [np.asarray(e, np.int32).reshape(-1) for e in expected]
    return np.concatenate([np.asarray(p, np.int32).reshape(-1) for p in parts])


def _golden_cases():
    g_all = json.load(open(GOLDEN))
    cases = []
    for name in ("joint_one_stage", "vertical_one_stage", "paper_forms_one_stage"):
        g = g_all[name]
        vert = "r_fixed" in g
        for sv in g["solves"]:
            S = sv["n_stage"]
            coef = np.asarray([g["coef"]] * S, np.int32)[None]
            w = wl.Workload("g", wl.VERTICAL if vert else wl.JOINT, 1, S, g["c_max"],
                            list(g["batch_sizes"]), g["r_max"], g["tick_us"], max(sv["slo_us"], 1),
                            False, coef, np.array([g["lambda"]], np.int32),
                            np.array([sv["slo_us"]], np.int32),
                            r_fixed=np.full((1, S), g["r_fixed"], np.int32) if vert else None,
                            queue_model=1 if name.startswith("paper") else 0,
                            profile_form=1 if name.startswith("paper") else 0)
            cases.append(_case(w, True, ([sv["status"]], [sv["cost"]], [sv["ticks"]], sv["cfg"])))
    return cases


def test_checker_under_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not found")
    exe = tmp_path / "oracle_sanitized"
    build = subprocess.run(
        [gcc, "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-fno-omit-frame-pointer", "-Wall", "-Wextra",
         os.path.join(ROOT, "tests", "host", "oracle_sanitized.c"),
         os.path.join(ROOT, "oracle", "themis_oracle.c"),
         os.path.join(ROOT, "oracle", "themis_bruteforce.c"), "-o", str(exe)],
        capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr[-3000:]

    cases = _golden_cases()
    n_golden = len(cases)
    rng = np.random.default_rng(77)
    for rep in range(60):
        w = wl.tiny_random(rng, rep % 2, n_inst=int(rng.integers(1, 5)), max_stage=3)
        if rep % 5 == 4:                                   # the paper's printed forms
            w = w.with_model(int(rng.integers(1, 3)), rng.integers(0, 1500, size=w.coef.shape[:-1]))
        if rep % 11 == 0:
            w.lam[0] = 0                                   # an invalid instance
        cases.append(_case(w, True))
    # realistic search spaces (no enumeration) and the limits of the input ranges
    cases.append(_case(wl.workload(1, 3), False))
    cases.append(_case(wl.workload(2, 2), False))
    top = 1 << 20
    coef = np.array([[[top, top, top, 1, top], [0, 0, 0, 7, 1]]], np.int32)
    big = wl.Workload("limits", wl.JOINT, 1, 2, 4, [1, 1024], 15, 70_000, 2_000_000_000, False,
                      coef, np.array([top], np.int32), np.array([2_000_000_000], np.int32))
    cases.append(_case(big, False))
    path = tmp_path / "cases.bin"
    np.concatenate([np.asarray([len(cases)], np.int32)] + cases).tofile(path)

    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe), str(path)], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert f"sanitized ok: {len(cases)} cases" in run.stdout
    assert n_golden >= 10
