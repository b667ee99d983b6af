#!/usr/bin/env python3
"""Benchmark of the batched activation-checkpoint DP on one MI355X.

One "step" = one pass of the whole hot path (threshold precompute + full table fill of
every chain of the batch) with the chain descriptors already resident in HBM.  Prints
ONE JSON line: min-plus candidate evaluations per second on the named workload, DP
cells per second, the roofline of the dominant kernel (durations from HIP events
recorded by the library on the launch stream) and the CPU oracle timed on a bounded
sample of the same workload.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu] [--all] [--calib-copy MIB]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Roofs.  HBM3E of one MI355X: 8 TB/s.  Vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz =
# 39.3e12 lane-operations per second; float64 add/min issue at that rate (78.6 TFLOP/s fp64
# vector peak counts an FMA as two), and so do 32-bit integer operations.
PEAK_HBM = 8.0e12
PEAK_VALU_OPS = 256 * 64 * 2.4e9
# Algorithmic work of gemm_kernel per candidate of the middle splits: 16 operand rows of 4 B feed
# an 8x8 tile of cells, i.e. 1 byte of table reads per candidate; one float64 add and one float64
# min per candidate.  Every cell of the tile costs 5 bytes stored (cost + candidate number: the
# partial result for rows 0..6, the finished cell for row 7), and row 7, which the kernel finishes
# itself, one 4-byte operand load per split in the column block and per C_all.
GEMM_BYTES_PER_EVAL = 1.0
GEMM_BYTES_PER_CELL = 5.0
GEMM_OPS_PER_EVAL = 2


def counts(L, M, B):
    cells = B * (L * (L + 1) // 2) * (M + 1)
    evals = B * (M + 1) * (L * (L + 1) * (L + 2) // 6)
    return cells, evals


def row_loads(L, T, D, I, r):
    """(operand loads, stored cells) of one lane finishing row r of tile (I, I + D): 9 loads per
    split in the row block (left + 8 right; clamped columns are loaded too), one per split in the
    column block, one C_all operand per cell with j > i."""
    J, i = I + D, I * T + r
    cols = [j for j in range(J * T, min(L, J * T + T)) if j >= i]
    near_i = 0 if D == 0 else ((T - r) if D == 1 else (T - 1 - r))
    loads = near_i * (1 + T)
    loads += sum(1 for j in cols for q in range(max(i + 1, J * T + 1), j + 1))
    loads += sum(1 for j in cols if j > i)
    return loads, len(cols)


def gemm_work(L, M, B, T=8):
    """(middle candidates, cells, row-7 operand loads) of gemm_kernel per step: for every tile of
    block diagonal D >= 2 the splits strictly between its row block and its column block, plus
    the first stage of the column block; and the loads with which it finishes row 7.  Nominal
    counts: candidates that the feasibility test drops still count, as infeasible cells do in
    the headline metric."""
    nblk = (L + T - 1) // T
    evals = cells = loads7 = 0
    for D in range(2, nblk):
        for I in range(nblk - D):
            cols = min(T, L - (I + D) * T)
            cells += T * cols
            evals += T * cols * ((D - 1) * T + 1)
            loads7 += row_loads(L, T, D, I, T - 1)[0]
    return evals * (M + 1) * B, cells * (M + 1) * B, loads7 * (M + 1) * B


def gemm_bytes(L, M, B, T=8):
    evals, cells, loads7 = gemm_work(L, M, B, T)
    return GEMM_BYTES_PER_EVAL * evals + GEMM_BYTES_PER_CELL * cells + 4 * loads7


def row_bytes(L, M, B, T=8):
    """Algorithmic bytes of all row_kernel launches of a step (nominal: waves that the frontier
    test skips still count): 4 bytes per operand load, 5 bytes per cell of gemm partial (D >= 2)
    and 5 bytes stored per cell.  Row 7 of the tiles of D >= 2 belongs to gemm_kernel."""
    nblk = (L + T - 1) // T
    total = 0
    for D in range(nblk):
        for I in range(nblk - D):
            for r in range(T):
                if I * T + r >= L or (D >= 2 and r == T - 1):
                    continue
                loads, stored = row_loads(L, T, D, I, r)
                total += 4 * loads + (5 * T if D >= 2 else 0) + 5 * stored
    return total * (M + 1) * B


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


def run_config(amd, idx, steps, warmup, dev, profile=True):
    import torch
    from workloads import make_config
    batch = make_config(idx)
    L, M, B = batch.L, batch.M, batch.B
    t = upload(batch, dev)
    rows, pitch = amd.ckpt_table_rows(L), amd.ckpt_row_pitch(M)
    cost = torch.empty((B, rows, pitch), dtype=torch.int32, device=dev)
    arg = torch.empty((B, rows, pitch), dtype=torch.uint8, device=dev)
    ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device=dev)
    opt = dict(wdelta=t["wdelta"], of=t["of"], ob=t["ob"])

    def step():
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
    kinds = None
    if profile:
        acc = {}
        for _ in range(max(1, min(steps, 5))):
            for name, (ms, n) in amd.ckpt_solve_profiled(t["uf"], t["ub"], t["wa"], t["wabar"], L, M, B, cost,
                                                         arg, ws, **opt).items():
                a = acc.setdefault(name, [0.0, 0, 0])
                a[0] += ms; a[1] += n; a[2] += 1
        kinds = {k: dict(ms_per_step=v[0] / v[2], launches_per_step=v[1] // v[2]) for k, v in acc.items()}
    cells, evals = counts(L, M, B)
    return dict(batch=batch, ms=wall / steps * 1e3, cells=cells, evals=evals, kinds=kinds)


def time_planner_steps(amd, idx, dev, reps=20):
    """Microseconds per call of the planner-side steps on workload idx (tables already filled)."""
    import numpy as np
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
    steps = {
        "ckpt_select_plan": lambda: amd.ckpt_select_plan(sol.cost, L, M, B, budgets, out),
        "ckpt_schedule_batched": lambda: amd.ckpt_schedule_batched(sol.arg, wa, wabar, L, M, B, budgets, ops, cap,
                                                                   n_ops, ws),
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
    assert (o_wa == wa).all() and int(out[0]) >= 0 and int(n_ops.min()) > 0
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
    ap.add_argument("--all", action="store_true", help="also time the other four workloads (few steps each)")
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

    r = run_config(amd, a.config, a.steps, a.warmup, dev)
    batch = r["batch"]
    evals_per_s = r["evals"] / (r["ms"] * 1e-3)
    kinds = r["kinds"]
    dom = max(("gemm_kernel", "row_kernel"), key=lambda k: kinds[k]["ms_per_step"])
    gemm_evals, _, gemm_loads7 = gemm_work(batch.L, batch.M, batch.B)
    dom_ms = kinds[dom]["ms_per_step"]
    launches = max(1, kinds[dom]["launches_per_step"])
    per_launch_s = dom_ms * 1e-3 / launches
    if dom == "gemm_kernel":
        alg_bytes = gemm_bytes(batch.L, batch.M, batch.B) / launches
        dom_evals, ops_per_eval = gemm_evals, GEMM_OPS_PER_EVAL   # the middle splits; row 7 adds < 1 %
        alu_unit = "Tlane-op/s (float64 add + min per candidate)"
    else:
        alg_bytes = row_bytes(batch.L, batch.M, batch.B) / launches
        dom_evals, ops_per_eval = r["evals"] - gemm_evals - gemm_loads7, 4   # add, compare, two selects each
        alu_unit = "Tlane-op/s (32-bit add, compare, two selects per candidate)"
    alg_ops = ops_per_eval * dom_evals / launches
    roofline = {"bound": "hbm", "kernel": dom, "achieved": alg_bytes / per_launch_s / 1e9, "peak": PEAK_HBM / 1e9,
                "unit": "GB/s", "frac": alg_bytes / per_launch_s / PEAK_HBM,
                "traffic": measured_traffic(batch.name, dom),
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": per_launch_s * 1e3,
                "launches_per_step": launches, "evals_in_kernel_per_step": dom_evals,
                "alu": {"achieved": alg_ops / per_launch_s / 1e12, "peak": PEAK_VALU_OPS / 1e12,
                        "unit": alu_unit, "frac": alg_ops / per_launch_s / PEAK_VALU_OPS}}
    out = {
        "metric": "min-plus candidate evaluations per second (whole batch, tables resident in HBM)",
        "value": evals_per_s, "unit": "evals/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": r["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": batch.name, "L": batch.L, "M": batch.M, "B": batch.B, "cells": r["cells"],
                   "evals": r["evals"]},
        "cells_per_s": r["cells"] / (r["ms"] * 1e-3),
        "kernels": kinds,
        "roofline": roofline,
    }
    if a.all:
        others = {}
        for idx in range(5):
            if idx == a.config:
                continue
            o = run_config(amd, idx, 5, 2, dev, profile=False)
            others[o["batch"].name] = {"ms_per_step": o["ms"], "evals_per_s": o["evals"] / (o["ms"] * 1e-3),
                                       "cells_per_s": o["cells"] / (o["ms"] * 1e-3)}
        out["other_workloads"] = others
        out["planner_steps"] = time_planner_steps(amd, a.config, dev)
        out["tables_d2h"] = time_d2h(amd, a.config, dev)
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(a.config)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
