#!/usr/bin/env python3
"""Benchmark of the batched autoscaling solve on one MI355X.

A step is one pass of the whole solve (candidate tables -> min-plus DP ->
selection and reconstruction) over one batch of synthetic instances whose
inputs are already resident in HBM.  The steps are timed twice: as single calls
of the solve entry point (`value`, `ms_per_step`), and stage by stage with HIP
events between the stages (`kernel_ms`, the roofline figures,
`ms_per_step_stage_by_stage`).  The headline workload is the largest of the
five (workload 3: 65536 pipelines of 8 models); the other four, the exact
work-reducing forms and the further entry points are timed in the same run and
reported beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 0..4] [--no-others]
"""

from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X figures used as roofline denominators.
HBM_PEAK_GBS = 8000.0
N_CU, CLOCK_GHZ = 256, 2.4
LDS_BYTES_PER_CLK_CU = 128          # ds_read path per compute unit
LDS_PEAK_GBS = N_CU * LDS_BYTES_PER_CLK_CU * CLOCK_GHZ          # 78643 GB/s
VALU_PEAK_GOPS = N_CU * 64 * CLOCK_GHZ                          # 39322 G lane-ops/s
# HBM bytes per stage-2 pass from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, see
# profiles/*_hbm_bytes.txt): workload -> (bytes, the `bytes_per_launch` of the run
# the counters were taken on, fingerprint of the kernel sources at that time).
# `roofline.traffic` is null unless both still match this run.
K2_HBM_TRAFFIC = {
    "w1-joint-4096x5": (116046179, 5247396664, "dc14bc4491f9ff0e"),
    "w3-joint-65536x8": (11099767522, 1422380424686, "dc14bc4491f9ff0e"),
}
# the same for stage 1 (input check + candidate kernel): workload -> (bytes, fingerprint)
K1_HBM_TRAFFIC = {
    "w1-joint-4096x5": (20024054, "dc14bc4491f9ff0e"),
    "w3-joint-65536x8": (1056689776, "dc14bc4491f9ff0e"),
}
KERNEL_SOURCES = ("k1_candidates.hip", "candidate_eval.h", "k2_minplus.hip", "instance_queue.h",
                  "themis_internal.h")


def kernel_fingerprint():
    """sha256 (first 16 hex digits) over the sources of stages 1 and 2."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2407_14843_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def hbm_traffic(workload, bytes_per_launch):
    rec = K2_HBM_TRAFFIC.get(workload)
    if rec is None or rec[1] != bytes_per_launch or rec[2] != kernel_fingerprint():
        return None
    return rec[0]


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def run_workload(themis, wl, idx, steps, warmup, n_inst=None, prune=0, copy_leg=False):
    """Time `steps` solves of workload idx; returns a dict of measurements."""
    import numpy as np
    import torch

    w = wl.workload(idx, n_inst)
    passes = [w]
    if idx == 4:
        passes = [w, None]          # second pass is built from the first one's output
    out = {"workload": w.name, "n_inst": w.n_inst, "n_stage": w.n_stage, "n_cand": w.n_cand}
    total_ms = 0.0
    staged_ms = 0.0
    copy_ms = 0.0
    k_ms = [0.0, 0.0, 0.0]
    cells = 0
    formed = 0
    relax = 0
    entries = 0
    solved = 0
    for pi, wp in enumerate(passes):
        if wp is None:
            # trace sweep, vertical pass: replicas carried forward from the
            # joint pass this same library just produced
            st, _, _, cfg = first_results
            wp = w.with_r_fixed(wl.replicas_carried_forward(st, cfg))
        b = themis.DeviceBatch(wp, "cuda:0", prune=prune)
        p = b.p
        stream = torch.cuda.current_stream()

        def step(ev=None):
            themis.themis_stage_candidates(p, b.coef, b.lam, b.slo_us, b.r_fixed, b.workspace, stream)
            if ev:
                ev[1].record(stream)
            themis.themis_stage_minplus(p, b.workspace, stream)
            if ev:
                ev[2].record(stream)
            themis.themis_stage_backtrack(p, b.status, b.cost, b.ticks, b.cfg, b.workspace, stream)

        for _ in range(warmup):
            b.solve(stream)
        torch.cuda.synchronize()
        # the timed steps: one call of the whole solve each, nothing in between
        t0 = time.perf_counter()
        for _ in range(steps):
            b.solve(stream)
        torch.cuda.synchronize()
        total_ms += (time.perf_counter() - t0) * 1e3
        # the same steps issued stage by stage with HIP events between the stages
        # (an event costs a few microseconds of GPU time, so this leg is a little slower)
        evs = [_events(4) for _ in range(steps)]
        t0 = time.perf_counter()
        for e in evs:
            e[0].record(stream)
            step(e)
            e[3].record(stream)
        torch.cuda.synchronize()
        staged_ms += (time.perf_counter() - t0) * 1e3
        for e in evs:
            for j in range(3):
                k_ms[j] += e[j].elapsed_time(e[j + 1])

        # the same steps with the results copied to pinned host memory after each
        # (the boundary hands over device buffers, so this leg is extra)
        host = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
                for t in (b.status, b.cost, b.ticks, b.cfg)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps if copy_leg else 0):
            b.solve(stream)
            for h, t in zip(host, (b.status, b.cost, b.ticks, b.cfg)):
                h.copy_(t, non_blocking=True)
        torch.cuda.synchronize()
        copy_ms += (time.perf_counter() - t0) * 1e3

        res = b.results()
        if pi == 0:
            first_results = res
        solved += int((res[0] == 0).sum())
        cnt = torch.zeros(3, dtype=torch.int64, device="cuda:0")
        themis.themis_count_relaxations(p, b.workspace, cnt)
        torch.cuda.synchronize()
        relax += int(cnt[0].item())
        entries += int(cnt[1].item())
        formed += int(cnt[2].item())
        Ti = (wp.slo_us.astype(np.int64) // wp.tick_us)
        cells += int(((Ti + 1) * wp.n_stage).sum())
        del b
        torch.cuda.empty_cache()

    n_solves = w.n_inst * len(passes)
    ms_per_step = total_ms / steps
    k_ms = [x / steps for x in k_ms]
    out.update({
        "solves_per_step": n_solves,
        "ms_per_step": ms_per_step,
        "ms_per_step_with_result_copy": copy_ms / steps if copy_leg else None,
        "ms_per_step_stage_by_stage": staged_ms / steps,
        "solves_per_s": n_solves / (ms_per_step * 1e-3),
        "dp_cells_per_s": cells / (ms_per_step * 1e-3),
        "dp_cells_formed_per_s": formed / (ms_per_step * 1e-3),
        "relaxations_per_s": relax / (ms_per_step * 1e-3),
        "dp_cells": cells,
        "dp_cells_formed": formed,
        "relaxations_executed": relax,
        "relaxations_nominal": cells * w.n_cand,
        "feasible_fraction": solved / n_solves,
        "kernel_ms": {"candidates": k_ms[0], "minplus": k_ms[1], "backtrack": k_ms[2]},
    })
    # stage 1: 8 bytes written per candidate that reaches the table (the feasible
    # ones, less the pruned), + 20 bytes of coefficients read per model
    k1_bytes = entries * 8 + w.n_inst * w.n_stage * 20 * len(passes)
    out["candidates_bytes"] = k1_bytes
    out["table_entries"] = entries
    out["candidates_evaluated"] = w.n_inst * w.n_stage * w.n_cand * len(passes)
    out["candidates_GBs"] = k1_bytes / (k_ms[0] * 1e-3) / 1e9 if k_ms[0] > 0 else None
    # stage 2, LDS bytes: 16-bit cells, so 2 bytes read per relaxation and 2 bytes
    # written per cell into each of the two row copies
    out["minplus_lds_bytes"] = relax * 2 + formed * 4
    return out


def _time_calls(fn, steps, warmup):
    """Wall time per call of fn() (enqueue only), bracketed by synchronisation."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def two_streams(themis, wl, idx, steps, warmup):
    """The same steps issued alternately on two streams, each with its own batch
    object and workspace (what a caller with several batches in flight does):
    the thinning end of one solve overlaps the start of the next."""
    import torch
    w = wl.workload(idx)
    bs = [themis.DeviceBatch(w, "cuda:0") for _ in range(2)]
    ss = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    for k in range(2 * warmup):
        bs[k % 2].solve(ss[k % 2])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        bs[k % 2].solve(ss[k % 2])
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return {"ms_per_step": ms, "solves_per_s": w.n_inst / (ms * 1e-3)}


def small_batches(themis, wl):
    """Latency of a whole solve on small batches (what a controller that decides for
    a few pipelines at a time sees), issued call by call and as replays of a HIP
    graph captured from the same call, which removes the gaps between the
    solve's launches: microseconds per solve, synchronised after every solve."""
    import torch
    out = {}
    for idx, n in ((0, None), (1, 64), (1, 512)):
        for prune in (0, 1):
            w = wl.workload(idx, n)
            b = themis.DeviceBatch(w, "cuda:0", prune=prune)
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                for _ in range(3):
                    b.solve(stream=s)
            s.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                b.solve(stream=torch.cuda.current_stream())
            reps = 200

            def timed(fn):
                fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    fn()
                    torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e6 / reps

            with torch.cuda.stream(s):
                eager = timed(lambda: b.solve(stream=s))
            replay = timed(g.replay)
            out[f"{w.name}[{w.n_inst}]" + ("-pruned" if prune else "")] = {
                "us_per_solve": eager, "us_per_graph_replay": replay}
    return out


def next_rows(themis, wl, steps, warmup):
    """Timings of the entry points beyond the two plain solves, each on a seeded
    workload of the shapes above: horizontal-only solve and stability test
    (Algorithm 2, Section 5.1.3) and the paper's printed model forms on workload 1;
    the vertical solve with Algorithm 1's fallback on workload 2 with its arrival
    rates multiplied by U{1..5}, so that the running replicas often do not suffice;
    the trace sweep (workload 4, both passes) with every distinct instance solved once."""
    import numpy as np
    out = {}
    w1 = wl.workload(1)
    rng = np.random.default_rng(wl.BASE_SEED + 101)

    b = themis.DeviceBatch(w1)
    ms = _time_calls(lambda: b.solve_horizontal(None), steps, warmup)
    st = b.results()[0]
    out["horizontal_one_core"] = {"workload": w1.name, "ms_per_call": ms,
                                  "solves_per_s": w1.n_inst / (ms * 1e-3),
                                  "feasible_fraction": float((st == 0).mean())}

    pred = np.clip(w1.lam.astype(np.int64) + rng.integers(-20, 40, w1.n_inst), 1, 1 << 20)
    ms = _time_calls(lambda: b.check_stability(pred.astype(np.int32)), steps, warmup)
    import torch
    torch.cuda.synchronize()
    out["stability_test"] = {"workload": w1.name, "ms_per_call": ms,
                             "instances_per_s": w1.n_inst / (ms * 1e-3),
                             "stable_fraction": float(b.stable.float().mean().item()),
                             "passes": 2}
    del b

    d = rng.integers(0, 1500, size=w1.coef.shape[:-1])
    wv = w1.with_model(1, d)
    bv = themis.DeviceBatch(wv)
    ms = _time_calls(lambda: bv.solve(), steps, warmup)
    out["paper_forms_eq4_eq1"] = {"workload": w1.name, "ms_per_call": ms,
                                  "solves_per_s": w1.n_inst / (ms * 1e-3),
                                  "feasible_fraction": float((bv.results()[0] == 0).mean())}
    del bv

    w2 = wl.workload(2)
    w2.lam = np.minimum(w2.lam.astype(np.int64) * rng.integers(1, 6, w2.n_inst),
                        1 << 20).astype(np.int32)
    for prune in (0, 1):
        bf = themis.DeviceBatch(w2, prune=prune)
        ms = _time_calls(lambda: bf.solve_vertical_fallback(), max(2, steps // 4), 1)
        r = bf.fallback_results()
        lv = r["lambda_v"]
        out["vertical_fallback" + ("_pruned" if prune else "")] = {
            "workload": w2.name + ", rates x U{1..5}", "ms_per_call": ms,
            "instances_per_s": w2.n_inst / (ms * 1e-3),
            "passes_of_the_three_stages": 3,
            "absorbed_outright": float((lv == w2.lam).mean()),
            "split_between_old_and_new_instances": float(((lv > 0) & (lv < w2.lam)).mean()),
            "remainder_served": float((r["status_h"][(lv > 0) & (lv < w2.lam)] == 0).mean())}
        del bf
    torch.cuda.empty_cache()

    # the trace sweep with every distinct instance solved once (few distinct rates:
    # coefficients and objective are shared); NOT the measured hot path, which
    # solves every instance
    w4 = wl.workload(4)
    n_steps = max(2, steps // 4)
    bj = themis.DeviceBatch(w4)
    ms_j = _time_calls(lambda: bj.solve_distinct(), n_steps, 1)
    st, _, _, cfg = bj.results()
    r_fixed = wl.replicas_carried_forward(st, cfg)
    bv = themis.DeviceBatch(w4.with_r_fixed(r_fixed))
    ms_v = _time_calls(lambda: bv.solve_distinct(), n_steps, 1)
    key = np.concatenate([w4.lam[:, None], r_fixed], axis=1)
    out["trace_sweep_distinct_instances_only"] = {
        "workload": w4.name, "ms_per_call": ms_j + ms_v,
        "instances_per_s": 2 * w4.n_inst / ((ms_j + ms_v) * 1e-3),
        "joint_pass_ms": ms_j, "vertical_pass_ms": ms_v,
        "distinct_joint": int(np.unique(w4.lam).size),
        "distinct_vertical": int(np.unique(key, axis=0).shape[0]),
        "feasible_fraction": float((bv.results()[0] == 0).mean())}
    del bj, bv
    torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, idx, sample):
    """The CPU checker, as it stands, timed on this machine's host cores on a seeded
    sample of the workload's instances (the rate extrapolates linearly: instances
    are independent)."""
    import numpy as np
    from oracle import oracle
    oracle.build(force=False)
    full = wl.workload(idx)
    n = min(sample, full.n_inst)
    pick = np.sort(np.random.default_rng(wl.BASE_SEED + 900 + idx).choice(
        full.n_inst, size=n, replace=False))
    w = full.take(pick)
    threads = min(os.cpu_count() or 1, 16)
    oracle.solve(w.head(min(8, w.n_inst)))       # load + touch
    t0 = time.perf_counter()
    oracle.solve(w, threads=threads)
    dt = time.perf_counter() - t0
    one = w.head(max(1, n // 32))
    t0 = time.perf_counter()
    oracle.solve(one, threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": w.n_inst / dt, "unit": "solves/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of the {full.n_inst} instances of {full.name}, drawn without "
                      f"replacement (seed {wl.BASE_SEED + 900 + idx}), instance range sharded "
                      f"over {threads} threads, one run, {dt:.2f} s wall",
            "single_thread_value": one.n_inst / dt1,
            "single_thread_sample": f"first {one.n_inst} instances of that sample, {dt1:.2f} s"}


def _probe_lib():
    """The probe library (LDS read and vector-issue micro-kernels), built beside
    the solve library but not part of it."""
    path = os.path.join(ROOT, "paper_2407_14843_amd", "libthemis_probe.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2407_14843_amd.build`")
    L = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    L.probe_lds_read.restype = ctypes.c_int
    L.probe_lds_read.argtypes = [ctypes.c_int] * 4 + [vp, vp]
    L.probe_valu.restype = ctypes.c_int
    L.probe_valu.argtypes = [ctypes.c_int] * 3 + [vp, vp]
    return L


def lds_probe():
    """Measure LDS read bandwidth for each read width / alignment and the issue rate
    of the vector instructions the kernels are made of; prints one JSON line."""
    import torch
    P = _probe_lib()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream()
    sp, st = ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(stream.cuda_stream)

    def lds(width, mis, iters, blocks):
        rc = P.probe_lds_read(width, mis, iters, blocks, sp, st)
        assert rc == 0, f"probe_lds_read({width}, {mis}) returned {rc}"

    def valu_op(op, iters, blocks):
        rc = P.probe_valu(op, iters, blocks, sp, st)
        assert rc == 0, f"probe_valu({op}) returned {rc}"

    blocks, iters = N_CU * 2 * 4, 2000
    res = {}
    for width, mis in ((4, 0), (4, 2), (8, 0), (8, 4), (8, 2), (8, -1), (8, -2), (16, 0), (16, 8),
                       (16, 4), (16, 2)):
        lds(width, mis, 50, blocks)
        torch.cuda.synchronize()
        e0, e1 = _events(2)
        e0.record(stream)
        lds(width, mis, iters, blocks)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        gbs = blocks * 1024 * iters * 4 * width / (ms * 1e-3) / 1e9
        name = {-1: "read2_b32 adjacent, 4-byte aligned", -2: "read2st64_b32"}.get(
            mis, f"b{width * 8}+{mis}")
        res[name] = {"ms": ms, "GB/s": gbs,
                                       "bytes_per_clk_per_cu": gbs / N_CU / CLOCK_GHZ}
    valu = {}
    names = ["v_pk_add_u16", "v_pk_min_u16", "v_add_u32", "v_min_u32",
             "v_pk_add_u16/v_pk_min_u16 alternating", "v_pk_add_u16 (sgpr operand)",
             "v_fma_f64", "v_mul_f64", "v_add_f64", "v_floor_f64", "v_rcp_f64", "v_cvt_f64_u32",
             "v_cvt_u32_f64", "v_mul_lo_u32", "v_cmp_ge_f64", "v_cndmask_b32", "v_mul_u32_u24",
             "v_cndmask_b32_e64 (sgpr-pair mask)", "v_max_f64", "v_add_f64 clamp",
             "v_cmp_ge_f64_e64 (sgpr-pair result)", "v_mad_u32_u16",
             "v_pk_add_u16 op_sel (one half to both lanes)", "v_lshl_add_u32",
             "v_add_u32_sdwa (16-bit operand)"]
    vblocks, viters = N_CU * 8 * 4, 4000
    for op, name in enumerate(names):
        valu_op(op, 10, vblocks)
        torch.cuda.synchronize()
        e0, e1 = _events(2)
        e0.record(stream)
        valu_op(op, viters, vblocks)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        gops = vblocks * 256 * viters * 16 / (ms * 1e-3) / 1e9
        valu[name] = {"ms": ms, "G lane-instr/s": gops,
                      "lanes_per_clk_per_cu": gops / N_CU / CLOCK_GHZ}
    print(json.dumps({"lds_read_probe": res, "valu_probe": valu, "blocks": blocks,
                      "threads": 1024, "iters": iters, "assumed_clock_ghz": CLOCK_GHZ}),
          flush=True)


def _fractions(m):
    """Roofline fractions of stages 1 and 2 from one run_workload() record."""
    k2s = m["kernel_ms"]["minplus"] * 1e-3
    return {
        "minplus_lds_frac": m["minplus_lds_bytes"] / k2s / 1e9 / LDS_PEAK_GBS,
        "minplus_valu_frac": m["relaxations_executed"] / k2s / 1e9 / VALU_PEAK_GOPS,
        "candidates_hbm_frac": (None if m["candidates_GBs"] is None
                                else m["candidates_GBs"] / HBM_PEAK_GBS),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3,
                    help="the headline workload (default 3, the largest: 65536 x 8)")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the other numbered workloads and the further entry points")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline leg")
    ap.add_argument("--cpu-sample", type=int, default=2048,
                    help="instances of the headline workload the CPU baseline solves")
    ap.add_argument("--prune", action="store_true",
                    help="time the solve with dominated candidates pruned as the main figure "
                         "(same answers, fewer relaxations); the default times the dense solve")
    ap.add_argument("--no-result-copy", action="store_true",
                    help="skip the extra leg that repeats the steps with the results copied to "
                         "the host (keeps a profiler's kernel counts to the timed steps)")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="skip the leg that issues the steps on two streams")
    ap.add_argument("--no-pruned", action="store_true",
                    help="skip the extra legs that time the work-reducing forms beside the "
                         "dense one")
    ap.add_argument("--copy-calib", action="store_true",
                    help="only run one 1 GiB device-to-device copy kernel (reference point for "
                         "HBM byte counters)")
    ap.add_argument("--lds-probe", action="store_true",
                    help="only measure LDS read bandwidth (roofline denominator)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this solve runs on one GPU; instances are independent, so N GPUs "
              "would each take a contiguous shard. Only --gpus 1 is measured.", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    from paper_2407_14843_amd import themis, workloads as wl
    themis.lib()
    if a.lds_probe:
        lds_probe()
        return
    if a.copy_calib:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calib_bytes_read": src.numel() * 4,
                          "copy_calib_bytes_written": dst.numel() * 4}), flush=True)
        return

    m = run_workload(themis, wl, a.workload, a.steps, a.warmup, prune=int(a.prune),
                     copy_leg=not a.no_result_copy)
    k2_ms = m["kernel_ms"]["minplus"]
    k2_gbs = m["minplus_lds_bytes"] / (k2_ms * 1e-3) / 1e9
    line = {
        "metric": "joint-scaling DP solves/sec",
        "value": m["solves_per_s"],
        "unit": "solves/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": m["ms_per_step"],
        "ms_per_step_with_result_copy": m["ms_per_step_with_result_copy"],
        "ms_per_step_stage_by_stage": m["ms_per_step_stage_by_stage"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": m["workload"], "n_inst": m["n_inst"], "n_stage": m["n_stage"],
                   "candidates_per_stage": m["n_cand"], "prune": bool(a.prune)},
        # nominal cells: every (model, budget) pair of every instance, S * (T + 1)
        "dp_cells_per_s": m["dp_cells_per_s"],
        # cells whose value the kernels form (the model handled last only yields the answer)
        "dp_cells_formed_per_s": m["dp_cells_formed_per_s"],
        "relaxations_per_s": m["relaxations_per_s"],
        "feasible_fraction": m["feasible_fraction"],
        "kernel_ms": m["kernel_ms"],
        "roofline": {
            "kernel": ("k2_minplus_pruned" if a.prune else "k2_minplus_wide") +
                      " (all class launches of a step)", "bound": "lds",
            "achieved": k2_gbs, "peak": LDS_PEAK_GBS, "unit": "GB/s",
            "frac": k2_gbs / LDS_PEAK_GBS,
            "traffic": hbm_traffic(m["workload"], m["minplus_lds_bytes"]),
            "bytes_per_launch": m["minplus_lds_bytes"],
            "valu_frac": (m["relaxations_executed"] / (k2_ms * 1e-3) / 1e9) / VALU_PEAK_GOPS,
        },
        "roofline_candidates": {
            "kernel": "k1_candidates (+ input check)", "bound": "hbm",
            "achieved": m["candidates_GBs"],
            "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": None if m["candidates_GBs"] is None else m["candidates_GBs"] / HBM_PEAK_GBS,
            "traffic": (K1_HBM_TRAFFIC[m["workload"]][0]
                        if m["workload"] in K1_HBM_TRAFFIC and not a.prune
                        and K1_HBM_TRAFFIC[m["workload"]][1] == kernel_fingerprint() else None),
            "bytes_per_launch": m["candidates_bytes"],
        },
    }
    errors = {}

    def extra(name, fn):
        # a failure in a side leg must not cost the headline line
        try:
            line[name] = fn()
        except Exception as e:  # noqa: BLE001
            errors[name] = f"{type(e).__name__}: {e}"
            torch.cuda.empty_cache()

    if a.workload != 4 and not a.no_two_streams:
        extra("two_streams", lambda: two_streams(themis, wl, a.workload, a.steps, a.warmup))
    # the same solve with dominated candidates dropped before the recurrence: same
    # answers, a fraction of the relaxations; reported beside the dense figures
    if not a.prune and not a.no_pruned:
        def pruned_leg():
            pr = run_workload(themis, wl, a.workload, a.steps, a.warmup, prune=1)
            out = {k: pr[k] for k in ("solves_per_s", "dp_cells_per_s", "ms_per_step",
                                      "kernel_ms", "relaxations_executed")}
            out["relaxations_dense"] = m["relaxations_executed"]
            out.update(_fractions(pr))
            return out
        extra("pruned", pruned_leg)
        # and with the rows of the recurrence kept as step functions (candidates x
        # breakpoints instead of candidates x budgets), alone and with the pruning
        for name, mode in (("step_rows", 2), ("pruned_step_rows", 3)):
            def step_leg(mode=mode):
                sr = run_workload(themis, wl, a.workload, a.steps, a.warmup, prune=mode)
                return {k: sr[k] for k in ("solves_per_s", "ms_per_step", "kernel_ms")}
            extra(name, step_leg)
    if not a.no_others:
        def others_leg():
            others = {}
            n_steps = max(3, a.steps // 2)
            for idx in range(5):
                if idx == a.workload:
                    continue
                o = run_workload(themis, wl, idx, n_steps, 2, prune=int(a.prune))
                rec = {k: o[k] for k in (
                    "solves_per_s", "dp_cells_per_s", "dp_cells_formed_per_s",
                    "relaxations_per_s", "ms_per_step", "feasible_fraction", "kernel_ms",
                    "candidates_GBs")}
                rec.update(_fractions(o))
                if not a.prune and not a.no_pruned:
                    op = run_workload(themis, wl, idx, n_steps, 2, prune=1)
                    rec["pruned"] = {k: op[k] for k in (
                        "solves_per_s", "ms_per_step", "kernel_ms", "relaxations_executed")}
                    rec["pruned"].update(_fractions(op))
                others[o["workload"]] = rec
            return others
        extra("other_workloads", others_leg)
        extra("next_rows", lambda: next_rows(themis, wl, max(3, a.steps // 2), 2))
        extra("small_batches", lambda: small_batches(themis, wl))
    if not a.no_cpu:
        extra("cpu_baseline", lambda: cpu_baseline(wl, a.workload, a.cpu_sample))
    if errors:
        line["errors"] = errors
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
