#!/usr/bin/env python3
"""Benchmark of the batched activation-checkpoint DP on one MI355X.

One "step" = one pass of the whole hot path (threshold precompute, feasibility frontier and the
full table fill of every chain of the batch) with the chain descriptors already resident in HBM.
Prints ONE JSON line:

  value / ms_per_step   K solves enqueued back to back between two synchronisations (the
                        pipelined mean: the host's launch work hides behind the previous solve)
  latency_ms            every solve timed on its own with HIP events on the launch stream, after
                        3 warm-ups: median, min, max of >= 10 solves
  roofline              of the kernel that takes most of a solve.  `achieved` = bytes that the
                        kernel's waves really ask the memory system for (counted on the device:
                        work skipped by the feasibility tests is not billed) / its launch time
                        from HIP events; `traffic` = HBM bytes per launch from the committed
                        rocprofv3 counter summary; `method_floor` = what the method itself needs
                        (5 bytes per cell stored once, 2 vector operations per candidate)
  measured_roofs        copy bandwidth, Infinity-Cache read bandwidth, the block-product kernel's
                        access pattern without arithmetic, register-only candidate rates
  other_workloads       the L = 96, B = 64 workload with the same figures
  cpu_baseline          the CPU oracle on a bounded sample of the same workload

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu] [--all] [--roofs | --no-roofs]
                  [--no-others] [--latency-solves N] [--calib-copy MIB]
                  [--groups G] [--row-launches 0|1] [--list-split 0|1|2|4] [--stagger 1] [--frontier 0|1|2]
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Roofs.  HBM3E of one MI355X: 8 TB/s.  Vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz =
# 39.3e12 lane-operations per second; float64 add/min issue at that rate (78.6 TFLOP/s fp64
# vector peak counts an FMA as two), and so do 32-bit integer operations.
PEAK_HBM = 8.0e12
PEAK_VALU_OPS = 256 * 64 * 2.4e9
# What the method itself needs, whatever the kernel design: every cell is stored once (4-byte cost
# + 1-byte candidate number), and every candidate takes one add and one min / compare.
FLOOR_BYTES_PER_CELL = 5.0
FLOOR_OPS_PER_EVAL = 2


def counts(L, M, B):
    cells = B * (L * (L + 1) // 2) * (M + 1)
    evals = B * (M + 1) * (L * (L + 1) * (L + 2) // 6)
    return cells, evals


def gemm_evals(L, M, B, T=8):
    """Nominal candidates of the block-product kernel per step: for every tile of block diagonal
    D >= 2 the splits between its row block and its column block."""
    nblk = (L + T - 1) // T
    evals = 0
    for D in range(2, nblk):
        for I in range(nblk - D):
            evals += T * min(T, L - (I + D) * T) * ((D - 1) * T + 1)
    return evals * (M + 1) * B


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this
    workload (profiles/<kernel>_<workload>_pmc.txt, line 'traffic_bytes_per_launch: N'), or None."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def upload(batch, dev):
    import numpy as np
    import torch

    def up(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    return dict(uf=up(batch.uf), ub=up(batch.ub), wa=up(batch.wa), wabar=up(batch.wabar),
                wdelta=up(batch.wdelta), of=up(batch.of), ob=up(batch.ob))


def first_chains(batch, n):
    """The first n chains of a workload as a batch of their own (the planner's small-batch case)."""
    import dataclasses
    cut = lambda a: None if a is None else a[:n]
    return dataclasses.replace(batch, name=f"{batch.name}_first{n}", B=n, uf=cut(batch.uf), ub=cut(batch.ub),
                               wa=cut(batch.wa), wabar=cut(batch.wabar), wdelta=cut(batch.wdelta), of=cut(batch.of),
                               ob=cut(batch.ob))


def run_config(amd, idx, steps, warmup, dev, profile=True, solves=10, sched=None, chains=None):
    import torch
    from workloads import make_config
    batch = make_config(idx)
    if chains:
        batch = first_chains(batch, chains)
    L, M, B = batch.L, batch.M, batch.B
    t = upload(batch, dev)
    rows, pitch = amd.ckpt_table_rows(L), amd.ckpt_row_pitch(M)
    cost = torch.empty((B, rows, pitch), dtype=torch.int32, device=dev)
    arg = torch.empty((B, rows, pitch), dtype=torch.uint8, device=dev)
    ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device=dev)
    opt = dict(wdelta=t["wdelta"], of=t["of"], ob=t["ob"])
    amd.ckpt_init()

    def step():
        if sched:
            amd.ckpt_solve_batched_opts(t["uf"], t["ub"], t["wa"], t["wabar"], L, M, B, cost, arg, ws, **opt, **sched)
        else:
            amd.ckpt_solve_batched(t["uf"], t["ub"], t["wa"], t["wabar"], L, M, B, cost, arg, ws, **opt)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    flags = amd.ckpt_check_inputs(ws, L, M, B)
    assert not flags.any(), flags
    # every solve on its own: events on the launch stream (the solve forks from and joins into it)
    lat = []
    for k in range(3 + solves if solves > 0 else 0):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        step()
        e1.record()
        e1.synchronize()
        if k >= 3:
            lat.append(e0.elapsed_time(e1))
    kinds = None
    if profile:
        acc = {}
        reps = max(1, min(steps, 5))
        for r in range(reps):
            res = amd.ckpt_solve_profiled(t["uf"], t["ub"], t["wa"], t["wabar"], L, M, B, cost, arg, ws,
                                          count_bytes=(r == 0), **opt)
            for name, v in res.items():
                a = acc.setdefault(name, [0.0, 0, 0.0, 0.0])
                a[0] += v[0]; a[1] += v[1]
                if len(v) == 4:
                    a[2], a[3] = v[2], v[3]
        kinds = {k: dict(ms_per_step=v[0] / reps, launches_per_step=v[1] // reps, bytes_loaded_per_step=v[2],
                         bytes_stored_per_step=v[3]) for k, v in acc.items()}
    cells, evals = counts(L, M, B)
    return dict(batch=batch, ms=wall / steps * 1e3, cells=cells, evals=evals, kinds=kinds,
                latency={"median": statistics.median(lat), "min": min(lat), "max": max(lat), "solves": len(lat)}
                if lat else None)


def roofline_of(r):
    """Roofline object of the kernel that takes most of a solve (block product or rows)."""
    batch, kinds = r["batch"], r["kinds"]
    dom = max(("gemm_kernel", "tile_rows_kernel"), key=lambda k: kinds[k]["ms_per_step"])
    k = kinds[dom]
    launches = max(1, k["launches_per_step"])
    per_launch_s = k["ms_per_step"] * 1e-3 / launches
    moved = (k["bytes_loaded_per_step"] + k["bytes_stored_per_step"]) / launches
    g_evals = gemm_evals(batch.L, batch.M, batch.B)
    if dom == "gemm_kernel":
        dom_evals, ops_per_eval = g_evals, 2
        alu_unit = "Tlane-op/s (float64 add + min per candidate, nominal candidate count)"
    else:
        dom_evals, ops_per_eval = r["evals"] - g_evals, 4
        alu_unit = "Tlane-op/s (32-bit add, compare, two selects per candidate, nominal candidate count)"
    step_s = r["ms"] * 1e-3
    floor_bytes = FLOOR_BYTES_PER_CELL * r["cells"]
    floor_ops = FLOOR_OPS_PER_EVAL * r["evals"]
    solve_bytes = sum(kinds[n]["bytes_loaded_per_step"] + kinds[n]["bytes_stored_per_step"]
                      for n in ("gemm_kernel", "tile_rows_kernel"))
    return {"bound": "hbm", "kernel": dom, "achieved": moved / per_launch_s / 1e9, "peak": PEAK_HBM / 1e9,
            "unit": "GB/s", "frac": moved / per_launch_s / PEAK_HBM,
            "traffic": measured_traffic(batch.name, dom),
            "requested_bytes_per_launch": moved, "avg_launch_ms": per_launch_s * 1e3, "launches_per_step": launches,
            "counted": "bytes the kernel's waves ask for (256 per wave and load, 320 per wave and stored cell), "
                       "counted on the device; work skipped by the feasibility tests is not billed",
            "alu": {"achieved": ops_per_eval * dom_evals / launches / per_launch_s / 1e12, "peak": PEAK_VALU_OPS / 1e12,
                    "unit": alu_unit, "frac": ops_per_eval * dom_evals / launches / per_launch_s / PEAK_VALU_OPS},
            "whole_solve": {"requested_bytes": solve_bytes, "GB/s": solve_bytes / step_s / 1e9,
                            "frac_of_hbm_peak": solve_bytes / step_s / PEAK_HBM},
            "method_floor": {"compulsory_bytes": floor_bytes, "hbm_ms": floor_bytes / PEAK_HBM * 1e3,
                             "alu_ops": floor_ops, "alu_ms": floor_ops / PEAK_VALU_OPS * 1e3,
                             "solve_over_hbm_floor": step_s / (floor_bytes / PEAK_HBM),
                             "solve_over_alu_floor": step_s / (floor_ops / PEAK_VALU_OPS),
                             "note": "5 bytes per cell stored once; one add and one min or compare per candidate"}}


def summary_of(r):
    s = r["ms"] * 1e-3
    return {"ms_per_step": r["ms"], "evals_per_s": r["evals"] / s, "cells_per_s": r["cells"] / s,
            "latency_ms": r["latency"], "L": r["batch"].L, "M": r["batch"].M, "B": r["batch"].B}


def measure_roofs(dev, quick=True):
    """Roofs measured on this machine with the microbenchmarks of libckpt_roofs.so."""
    import torch
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2302_02599_amd", "libckpt_roofs.so"))
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.ckpt_roof_copy.argtypes = [vp, vp, sz, i, vp, vp]
    lib.ckpt_roof_read.argtypes = [vp, sz, i, vp, vp, vp]
    lib.ckpt_roof_read_rows.argtypes = [vp, i, i, i, i, vp, vp, vp, vp]
    lib.ckpt_roof_alu.argtypes = [i, i, i, vp, vp, vp, vp, vp]
    st = vp(torch.cuda.current_stream().cuda_stream)
    ms, dbl = ctypes.c_float(), ctypes.c_double()
    sink = torch.zeros(16, dtype=torch.int32, device=dev)
    out = {}
    nbytes = 1 << 30
    a = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    assert lib.ckpt_roof_copy(b.data_ptr(), a.data_ptr(), nbytes, 4, st, ctypes.byref(ms)) == 0
    out["copy_1GiB"] = {"GB/s_read_plus_write": 2 * 4 * nbytes / ms.value / 1e6}
    assert lib.ckpt_roof_read(a.data_ptr(), nbytes, 4, sink.data_ptr(), st, ctypes.byref(ms)) == 0
    out["read_1GiB"] = {"GB/s": 4 * nbytes / ms.value / 1e6}
    for mib in ((64, 192) if quick else (16, 64, 128, 192, 256, 512)):
        n = mib << 20
        reps = max(2, (4 << 30) // n)
        assert lib.ckpt_roof_read(a.data_ptr(), n, reps, sink.data_ptr(), st, ctypes.byref(ms)) == 0
        out[f"read_{mib}MiB_repeated"] = {"GB/s": reps * n / ms.value / 1e6, "passes": reps}
    del b
    # the block product's access pattern: 4160-column rows, 90 steps, 170 tiles (about 6.5 GB of rows)
    pitch, nq, tiles = 4160, 90, 170
    tab = torch.zeros((tiles * 16 * nq + 2) * pitch, dtype=torch.int32, device=dev)
    for shift in (0, 37):
        assert lib.ckpt_roof_read_rows(tab.data_ptr(), pitch, nq, tiles, shift, sink.data_ptr(), st, ctypes.byref(ms),
                                       ctypes.byref(dbl)) == 0
        out[f"read_16_rows_per_step_shift_{shift}"] = {"GB/s": dbl.value / ms.value / 1e6, "bytes": dbl.value}
    del tab, a
    seed = torch.arange(4096, dtype=torch.int32, device=dev) * 2654435
    blocks, iters = 256 * 4 * 4, 2000
    res = torch.empty(blocks * 64, dtype=torch.int32, device=dev)
    for kind, name in ((0, "f64_add_min"), (1, "u32_add_compare_two_selects"), (2, "u32_add_min")):
        assert lib.ckpt_roof_alu(kind, blocks, iters, seed.data_ptr(), res.data_ptr(), st, ctypes.byref(ms),
                                 ctypes.byref(dbl)) == 0
        out[f"register_only_{name}"] = {"Tevals/s": dbl.value / ms.value / 1e9}
    return out


def time_planner_steps(amd, idx, dev, reps=20):
    """Microseconds per call of the planner-side steps on workload idx (tables already filled)."""
    import torch
    from workloads import make_config
    batch = make_config(idx)
    L, M, B = batch.L, batch.M, batch.B
    sol = amd.solve(batch, device=str(dev))
    wa, wabar = torch.from_numpy(batch.wa).to(dev), torch.from_numpy(batch.wabar).to(dev)
    budgets = torch.full((B,), M, dtype=torch.int32, device=dev)
    out = torch.zeros(2, dtype=torch.int32, device=dev)
    cap = L * (L + 1) // 2 + L
    ops = torch.zeros((B, cap, 2), dtype=torch.uint8, device=dev)
    n_ops = torch.zeros(B, dtype=torch.int32, device=dev)
    ws = torch.empty(amd.ckpt_schedule_workspace_bytes(L, B), dtype=torch.uint8, device=dev)
    by_wa, by_wabar = wa.to(torch.int64) * 1000, wabar.to(torch.int64) * 1000
    budget_bytes = torch.full((B,), 1000 * M, dtype=torch.int64, device=dev)
    o_wa, o_wabar = torch.empty_like(wa), torch.empty_like(wabar)
    uf, ub = torch.from_numpy(batch.uf).to(dev), torch.from_numpy(batch.ub).to(dev)
    extra = {k: None if getattr(batch, k) is None else torch.from_numpy(getattr(batch, k)).to(dev)
             for k in ("wdelta", "of", "ob")}
    sim_time = torch.zeros(B, dtype=torch.int64, device=dev)
    sim_peak = torch.zeros(B, dtype=torch.int64, device=dev)
    sim_status = torch.zeros(B, dtype=torch.int32, device=dev)
    blocks = torch.zeros((B, L), dtype=torch.int32, device=dev)
    n_blocks = torch.zeros(B, dtype=torch.int32, device=dev)
    steps = {
        "ckpt_select_plan": lambda: amd.ckpt_select_plan(sol.cost, L, M, B, budgets, out),
        "ckpt_schedule_batched": lambda: amd.ckpt_schedule_batched(sol.arg, wa, wabar, L, M, B, budgets, ops, cap,
                                                                   n_ops, ws),
        "ckpt_block_indices_batched": lambda: amd.ckpt_block_indices_batched(ops, cap, n_ops, L, B, blocks, n_blocks),
        "ckpt_simulate_batched": lambda: amd.ckpt_simulate_batched(uf, ub, wa, wabar, L, B, ops, cap, n_ops, sim_time,
                                                                   sim_peak, sim_status, **extra),
        "ckpt_discretize": lambda: amd.ckpt_discretize(by_wa, by_wabar, budget_bytes, L, M, B, o_wa, o_wabar),
    }
    res = {}
    for name, fn in steps.items():
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / reps * 1e6
    assert (o_wa == wa).all() and int(out[0]) >= 0 and int(n_ops.min()) > 0 and int(n_blocks.min()) >= 0
    root = amd.ckpt_row_index(L, 1, L)
    assert (sim_status == 0).all() and (sim_time == sol.cost[:, root, M]).all() and int(sim_peak.max()) <= M
    return {"workload": batch.name, "us_per_call": res}


def time_d2h(amd, idx, dev):
    """Copy of the finished tables to pinned host memory; reported beside the solve, never part of it."""
    import torch
    from workloads import make_config
    sol = amd.solve(make_config(idx), device=str(dev))
    host = [torch.empty(t.shape, dtype=t.dtype, pin_memory=True) for t in (sol.cost, sol.arg)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for h, t in zip(host, (sol.cost, sol.arg)):
        h.copy_(t, non_blocking=True)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    nbytes = sum(h.numel() * h.element_size() for h in host)
    return {"ms": el * 1e3, "bytes": nbytes, "GB/s": nbytes / el / 1e9}


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(idx, budget_s=20.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload:
    whole chains of the batch, one after the other, until about budget_s seconds are spent;
    then one more chain on a single thread."""
    from oracle import oracle
    from workloads import make_config
    batch = make_config(idx)
    threads = oracle.max_threads()
    cells_chain, evals_chain = counts(batch.L, batch.M, 1)
    done, t0 = 0, time.perf_counter()
    while done < batch.B:
        oracle.solve_chain(batch.L, batch.M, *batch.chain(done), nthreads=threads)
        done += 1
        el = time.perf_counter() - t0
        if el + el / done > budget_s:
            break
    el = time.perf_counter() - t0
    t1 = time.perf_counter()
    oracle.solve_chain(batch.L, batch.M, *batch.chain(0), nthreads=1)
    el1 = time.perf_counter() - t1
    return {"value": evals_chain * done / el, "unit": "evals/s", "cores": threads, "kind": "oracle",
            "cells_per_s": cells_chain * done / el,
            "single_thread": {"value": evals_chain / el1, "unit": "evals/s", "sample": f"chain 0, {el1:.1f} s"},
            "cpu": cpu_model(), "host_cpus": os.cpu_count(),
            "sample": f"chains 0..{done - 1} of {batch.B} of {batch.name}, full tables, {el:.1f} s, "
                      f"OpenMP over the rows of one segment length"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload index 0..4 (default 4: L=192, M=4096, B=8)")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="first copy MIB mebibytes device to device (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--all", action="store_true", help="also time the other workloads, the planner-side steps, the "
                                                       "single-chain case and the copy of the tables to the host")
    ap.add_argument("--roofs", action="store_true", help="full sweep of the roof microbenchmarks")
    ap.add_argument("--no-roofs", action="store_true", help="skip the roof microbenchmarks")
    ap.add_argument("--no-others", action="store_true", help="skip the second workload (short counter runs)")
    ap.add_argument("--latency-solves", type=int, default=10, help="solves timed on their own (0: none)")
    ap.add_argument("--groups", type=int, default=0, help="experiment: chain groups (0 automatic, 1 one stream)")
    ap.add_argument("--row-launches", type=int, default=0, help="experiment: 1 = one launch per tile row")
    ap.add_argument("--list-split", type=int, default=0, help="experiment: waves per work list, 0 automatic")
    ap.add_argument("--stagger", type=int, default=0, help="experiment: phase-shift half of the chain groups")
    ap.add_argument("--frontier", type=int, default=0, help="experiment: 1 always run the exact frontier, 2 never")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build solves on one GPU; chains would be split across GPUs with no "
              "exchange, and no multi-GPU path exists here. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2302_02599_amd as amd
    amd.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if a.calib_copy:
        # a plain device copy of known size, first in the trace: scale for the rocprofv3 byte counters
        src = torch.empty(a.calib_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    sched = None
    if a.groups or a.row_launches or a.list_split or a.stagger or a.frontier:
        sched = dict(groups=a.groups, row_launches=a.row_launches, list_split=a.list_split, stagger=a.stagger,
                     frontier=a.frontier)

    r = run_config(amd, a.config, a.steps, a.warmup, dev, sched=sched, solves=a.latency_solves)
    batch = r["batch"]
    out = {
        "metric": "min-plus candidate evaluations per second (whole batch, tables resident in HBM)",
        "value": r["evals"] / (r["ms"] * 1e-3), "unit": "evals/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": r["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32",
        "arith": "float64 keys cost + candidate/256 (exact: integers below 2^34 scaled by 2^-8) in gemm_kernel, "
                 "uint32 everywhere else; tables int32 cost + uint8 candidate",
        "data": "synthetic",
        "config": {"workload": batch.name, "L": batch.L, "M": batch.M, "B": batch.B, "cells": r["cells"],
                   "evals": r["evals"], "counts": "nominal: infeasible cells and candidates skipped by the "
                                                  "feasibility tests count", "schedule": sched or "automatic"},
        "cells_per_s": r["cells"] / (r["ms"] * 1e-3),
        "latency_ms": r["latency"],
        "kernels": r["kinds"],
        "roofline": roofline_of(r),
    }
    others = {}
    if a.config != 3 and not a.no_others:
        o = run_config(amd, 3, 10, 3, dev, sched=sched)
        others[o["batch"].name] = dict(summary_of(o), roofline=roofline_of(o), kernels=o["kinds"])
    if a.all:
        for idx in range(3):
            if idx != a.config:
                o = run_config(amd, idx, 20, 3, dev, profile=False, sched=sched)
                others[o["batch"].name] = summary_of(o)
        o = run_config(amd, a.config, 20, 3, dev, profile=False, sched=sched, chains=1)
        others[o["batch"].name] = summary_of(o)
        out["planner_steps"] = time_planner_steps(amd, a.config, dev)
        out["tables_d2h"] = time_d2h(amd, a.config, dev)
    out["other_workloads"] = others
    if not a.no_roofs:
        out["measured_roofs"] = measure_roofs(dev, quick=not a.roofs)
    out["cpu_baseline"] = None if a.no_cpu else cpu_baseline(a.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
