#!/usr/bin/env python3
"""Benchmark of the DMMV single-move descent on one MI355X.

One "step" is one full pass of the hot path over one workload: dmmv_solve from the
configured starting point for the configured number of iterations (residual once, then per
iteration: score every move, arg-min, apply).  The descent stalls at a local optimum long
before the configured iteration count, so the timed solves run in fixed-work mode
(keep_going): every iteration still scores all n*(|D|-1) moves of the current state and
reduces them; iterations after the stall have no move left to apply.  Inputs are resident in
HBM before the timed region starts.

Prints ONE JSON line.  `value` = candidate moves evaluated per second over the whole timed
region.  `roofline` describes the dominant kernel (the evaluation kernel that streams all of
A), timed with HIP events on the library's stream.  `cpu_baseline` is the CPU oracle timed on
a bounded sample of the same workload on this host.  Further objects of the same line:
`other_workloads` (the same measurements for the other four workloads), `descent` (sparse and
batched: the real descent with and without exact pruning), `alns` (wall time of the ALNS outer
loop; batched also `alns_full_evaluation`, dense `alns_value_search`), `swap` (one search of the
swap move), `residual` (batched: the sequential-order and the matrix-core residual).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
ALU_PEAK_TFLOPS = {"f32": 157.3, "f64": 78.6}
FLOPS_PER_PAIR = 3          # multiply + add of the fma, and the max; |.| is an operand modifier
# HBM bytes per launch of the evaluation kernel, from rocprofv3 FETCH_SIZE + WRITE_SIZE runs
# calibrated against a plain copy (summaries under profiles/hbm_traffic_*.md)
MEASURED_TRAFFIC_BYTES = {
    "tomography_256x256_180x363_csr_f32": 100.2e6,
}


def algorithmic_bytes_per_eval(inst) -> float:
    """Bytes one evaluation launch must move: the matrix once (value + 4-byte index per stored
    entry and the column pointers for a sparse one), r, and the current index of every variable."""
    w = inst.dtype.itemsize
    if inst.kind == "csr":
        return inst.nnz * (w + 4) + (inst.n + 1) * 8 + inst.m * w + inst.n * 4
    if inst.kind == "batched":
        return inst.m * inst.n * w + inst.R * inst.m * w + inst.R * inst.n * 4
    return inst.m * inst.n * w + inst.m * w + inst.n * 4


def pairs_per_eval(inst) -> float:
    """(row, move) pairs of one evaluation, non-null moves only."""
    rows = inst.nnz / inst.n if inst.kind == "csr" else inst.m
    return float(inst.R) * inst.n * (inst.nd - 1) * rows


def roofline_for(inst, eval_ms: float) -> dict:
    dt = "f64" if inst.dtype == np.float64 else "f32"
    if inst.kind == "csr":
        b = algorithmic_bytes_per_eval(inst)
        ach = b / (eval_ms * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": "k_eval_stream", "achieved": ach, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": MEASURED_TRAFFIC_BYTES.get(inst.name),
                "algorithmic_bytes_per_launch": b, "avg_launch_ms": eval_ms}
    flops = pairs_per_eval(inst) * FLOPS_PER_PAIR
    ach = flops / (eval_ms * 1e-3) / 1e12
    peak = ALU_PEAK_TFLOPS[dt]
    return {"bound": "alu", "kernel": "k_eval_batched" if inst.kind == "batched" else "k_eval_dense",
            "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
            "flops_per_launch": flops, "avg_launch_ms": eval_ms,
            "hbm_GBs_algorithmic": algorithmic_bytes_per_eval(inst) / (eval_ms * 1e-3) / 1e9}


def cpu_baseline(inst, budget_s: float) -> dict:
    """The oracle as it stands, on a bounded sample of the workload."""
    from oracle import oracle as orc

    cores = len(os.sched_getaffinity(0))
    if inst.kind == "batched":
        # a few instances, a few iterations, all host threads (instances are independent)
        threads = orc.num_threads()
        rows = min(inst.R, max(threads, 16))
        est_pair_rate = 4.0e8                       # pairs/s/thread, only to size the sample
        per_row_iter = inst.m * inst.n * inst.nd
        iters = int(max(1, min(inst.iters, budget_s * est_pair_rate * threads / (rows * per_row_iter))))
        sel = np.linspace(0, inst.R - 1, rows).astype(np.int64)
        t0 = time.perf_counter()
        res = orc.solve_batched(inst.A, inst.b[sel], inst.D, inst.scale[sel], inst.x0[sel], iters)
        dt = time.perf_counter() - t0
        evals = int(np.minimum(res.iters_done + 1, iters).sum())
        moves = evals * inst.n * (inst.nd - 1)
        return {"value": moves / dt, "unit": "moves/s", "cores": threads, "kind": "oracle",
                "sample": f"{rows} of {inst.R} instances x up to {iters} iterations "
                          f"({evals} evaluations), {dt:.1f} s", "host_cores_visible": cores}
    per_iter = inst.nnz * inst.nd
    # the oracle scores about 1e9 pairs/s on one core; only used to size the sample
    iters = int(max(1, min(inst.iters, budget_s * 1.0e9 / max(per_iter, 1))))
    t0 = time.perf_counter()
    if inst.kind == "csr":
        res = orc.solve_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b,
                            inst.D, inst.x0, iters)
    else:
        res = orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, iters)
    dt = time.perf_counter() - t0
    evals = min(res.iters_done + 1, iters)
    moves = evals * inst.n * (inst.nd - 1)
    return {"value": moves / dt, "unit": "moves/s", "cores": 1, "kind": "oracle",
            "sample": f"{evals} evaluations from the configured start (of {inst.iters}), {dt:.1f} s",
            "host_cores_visible": cores}


def run_config(idx: int, steps: int, warmup: int, iters_override, device: str, do_cpu: bool,
               cpu_budget: float) -> dict:
    import torch
    from paper_2508_13437_amd import dmmv
    from workloads import make_config

    t_gen = time.perf_counter()
    inst = make_config(idx)
    t_gen = time.perf_counter() - t_gen
    iters = int(iters_override) if iters_override else inst.iters
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    out = {}
    # how far does the real descent get (normal mode, stops at the local optimum)?
    with dmmv.from_instance(inst, device) as h:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = dmmv.dmmv_solve(h, x0, iters)
        torch.cuda.synchronize()
        normal_s = time.perf_counter() - t0
        improving = res.iters_done.cpu().numpy().astype(np.int64)
        t_final = res.max_violation.cpu().numpy().astype(np.float64)
    # timed: fixed-work mode
    with dmmv.from_instance(inst, device, keep_going=True, poll_every=0) as h:
        for _ in range(warmup):
            dmmv.dmmv_solve(h, x0, iters)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            dmmv.dmmv_solve(h, x0, iters)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        reps = max(3, min(200, int(0.5 / max(dt / (steps * iters), 1e-6))))
        eval_ms = dmmv.dmmv_time_eval(h, reps) / reps
    moves = float(steps) * iters * inst.moves_per_iter()
    out.update({
        "workload": inst.name, "kind": inst.kind, "m": inst.m, "n": inst.n, "nd": inst.nd,
        "R": inst.R, "nnz": inst.nnz, "iters_per_step": iters,
        "moves_per_sec": moves / dt, "iters_per_sec": steps * iters / dt,
        "instance_iters_per_sec": steps * iters * inst.R / dt,
        "ms_per_step": dt / steps * 1e3, "us_per_iter": dt / (steps * iters) * 1e6,
        "improving_moves_applied": int(improving.sum()),
        "descent_until_local_optimum_ms": normal_s * 1e3,
        "final_max_violation": float(t_final.max()),
        "dtype": "f64" if inst.dtype == np.float64 else "f32",
        "roofline": roofline_for(inst, eval_ms), "input_gen_s": round(t_gen, 2),
    })
    if inst.kind == "batched":
        out["residual"] = residual_timing(inst, device, x0)
        if inst.dtype == np.float32 and inst.nd <= 32:
            # the same evaluation with the multiply-adds on the matrix cores (options.batched_eval = 2)
            with dmmv.from_instance(inst, device, batched_eval=2) as h:
                dmmv.dmmv_set_x(h, x0)
                dmmv.dmmv_residual(h)
                out["eval_matrix_core_ms"] = dmmv.dmmv_time_eval(h, 3) / 3
                out["eval_vector_unit_ms"] = eval_ms
    if inst.kind == "csr":
        out["descent"] = descent_timing(inst, device, x0, iters)
    if inst.kind == "batched":
        out["descent"] = descent_timing_batched(inst, device, x0, iters, normal_s, improving, t_final)
        # the outer loop with the full evaluation in its local search, for comparison
        out["alns_full_evaluation"] = alns_timing(inst, device, x0, prune=False)
    out["alns"] = alns_timing(inst, device, x0)
    if inst.kind == "dense":
        # same loop, the local search finding each variable's best value by bisection over D
        out["alns_value_search"] = alns_timing(inst, device, x0, value_search=True)
    out["swap"] = swap_timing(inst, device, x0, iters)
    if do_cpu:
        out["cpu_baseline"] = cpu_baseline(inst, cpu_budget)
    return out


def descent_timing(inst, device: str, x0, iters: int) -> dict:
    """The real descent (stops at the local optimum) with the full evaluation and with
    options.prune, which scores only the columns that touch the row of largest |r| and applies the
    same moves: an EFFECTIVE rate, reported apart from the full-table moves/s."""
    import torch
    from paper_2508_13437_amd import dmmv

    res = {}
    for key, opt in (("full", {}), ("pruned", {"prune": True})):
        with dmmv.from_instance(inst, device, poll_every=64, **opt) as h:
            dmmv.dmmv_solve(h, x0, iters)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            out = dmmv.dmmv_solve(h, x0, iters)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
        moves = int(out.iters_done.cpu()[0])
        res[key] = {"ms": dt * 1e3, "moves_applied": moves, "final_max_violation": float(out.max_violation.cpu()[0])}
    res["note"] = ("wall time of dmmv_solve until the local optimum; the host polls every 64 iterations, "
                   "so up to 63 iterations past the last move are enqueued")
    return res


def descent_timing_batched(inst, device: str, x0, iters: int, full_s: float, full_moves, full_t) -> dict:
    """The real descent of every instance of a batch with options.prune (bounds on 16 screening
    rows, full scores best-first; one launch for all iterations) against the descent with the full
    evaluation measured above: the same moves, an EFFECTIVE rate reported apart from moves/s."""
    import torch
    from paper_2508_13437_amd import dmmv

    with dmmv.from_instance(inst, device, prune=True) as h:
        dmmv.dmmv_solve(h, x0, iters)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = dmmv.dmmv_solve(h, x0, iters)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    moves = out.iters_done.cpu().numpy().astype(np.int64)
    t = out.max_violation.cpu().numpy().astype(np.float64)
    return {"full": {"ms": full_s * 1e3, "moves_applied": int(full_moves.sum())},
            "pruned": {"ms": dt * 1e3, "moves_applied": int(moves.sum()),
                       "instance_iters_per_sec": float(moves.sum() + (moves < iters).sum()) / dt,
                       "effective_moves_per_sec": float(moves.sum() + (moves < iters).sum()) * inst.moves_per_iter()
                                                  / inst.R / dt},
            "same_moves_and_errors": bool(np.array_equal(moves, full_moves) and np.array_equal(t, full_t)),
            "instances_at_local_optimum": int((moves < iters).sum()),
            "note": "wall time of dmmv_solve (residual included) for all instances; pruned.instance_iters_per_sec "
                    "counts one iteration per applied move plus the one that finds no improving move; "
                    "effective_moves_per_sec prices each of them at the n (|D| - 1) candidates the full "
                    "evaluation would have scored (the pruned path scores a handful) - not comparable "
                    "with `value`"}


def swap_timing(inst, device: str, x0, iters: int) -> dict:
    """The swap move (Algorithm 2) at the starting point and at the local optimum of the descent:
    wall time of one search over all pairs (x_i > x_j) of every instance, nothing carried out."""
    import torch
    from paper_2508_13437_amd import dmmv

    res = {"pairs_per_instance": inst.n * (inst.n - 1) // 2}
    with dmmv.from_instance(inst, device) as h:
        for key, descend in (("at_x0", 0), ("at_local_optimum", iters)):
            dmmv.dmmv_solve(h, x0, descend)
            dmmv.dmmv_swap_move(h, apply=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            out = dmmv.dmmv_swap_move(h, apply=False)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            res[key] = {"ms": dt * 1e3, "instances_with_improving_swap": int((out.i >= 0).sum().cpu()),
                        "unordered_pairs_per_sec": res["pairs_per_instance"] * inst.R / dt}
    return res


def alns_timing(inst, device: str, x0, **hopt) -> dict:
    """The ALNS outer loop (destroy, repair, local search, accept) around the descent: wall time of
    one dmmv_alns call with the paper's destroy rate (0.5 % of n) and coefficient (alpha = 0.3)."""
    import torch
    from paper_2508_13437_amd import dmmv

    outer = {"csr": 20, "dense": 200, "batched": 4}[inst.kind]
    ls_moves = 8 if inst.kind != "batched" else 4
    hopt.setdefault("prune", inst.kind in ("csr", "batched"))
    with dmmv.from_instance(inst, device, alns=True, **hopt) as h:
        dmmv.dmmv_alns(h, x0, 2, ls_moves=ls_moves, seed=1)             # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = dmmv.dmmv_alns(h, x0, outer, ls_moves=ls_moves, seed=1)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tr = res.trace.cpu().numpy().reshape(-1, 4)
        tt = res.trace_t.cpu().numpy().reshape(-1, 2)
    return {"outer_iterations": outer, "ls_moves_cap": ls_moves, "destroy_count": max(1, -(-inst.n * 5 // 1000)),
            "ms_per_outer_iteration": dt / outer * 1e3, "outer_iterations_per_sec": outer / dt,
            "accepted": int(tr[:, 3].sum()), "local_search_moves": int(tr[:, 2].sum()),
            "worst_remove_used": int(tr[:, 0].sum()), "greedy_repair_used": int(tr[:, 1].sum()),
            "instances": int(inst.R), "max_t_best": float(res.t_best.cpu().max())}


def residual_timing(inst, device: str, x0) -> dict:
    """The one-off batched residual r = (X Q^T) diag(s) - B: the sequential-order VALU kernel
    (bitwise reproducible, what dmmv_solve uses by default) and the matrix-core kernel
    (options.residual_mfma), each timed over a few calls with events on the library's stream."""
    import torch
    from paper_2508_13437_amd import dmmv

    res = {"flops": 2.0 * inst.m * inst.n * inst.R}
    for key, opt in (("valu", {}), ("mfma", {"residual_mfma": True})):
        with dmmv.from_instance(inst, device, **opt) as h:
            dmmv.dmmv_set_x(h, x0)
            dmmv.dmmv_residual(h)
            reps = 3
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(h.stream)
            for _ in range(reps):
                dmmv.dmmv_residual(h)
            e1.record(h.stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / reps
        res[key + "_ms"] = ms
        res[key + "_TFLOPs"] = res["flops"] / (ms * 1e-3) / 1e12
    res["note"] = ("ms per dmmv_residual call (kernel + max|r| + the copy of r out); mfma: bf16 planes of X "
                   "(1 when X is bf16-valued, else 3) x bf16-exact codes, fp32 accumulate")
    return res


def traffic_probe(idx: int, device: str, reps: int) -> None:
    """For `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs: launches the evaluation
    kernel of workload idx `reps` times and one plain device-to-device copy of a known size
    (256 MiB read + 256 MiB written) whose counter reading calibrates the counters' unit."""
    import torch
    from paper_2508_13437_amd import dmmv
    from workloads import make_config

    inst = make_config(idx)
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=device).fill_(1)
    dst = torch.empty_like(src)
    with dmmv.from_instance(inst, device, keep_going=True, poll_every=0) as h:
        dmmv.dmmv_set_x(h, x0)
        dmmv.dmmv_residual(h)
        ms = dmmv.dmmv_time_eval(h, reps)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps({"probe": inst.name, "eval_launches": reps + 1, "eval_avg_ms": ms / reps,
                      "copy_bytes_read": int(src.numel()), "copy_bytes_written": int(src.numel()),
                      "algorithmic_bytes_per_launch": algorithmic_bytes_per_eval(inst)}))


def residual_probe(idx: int, device: str, reps: int) -> None:
    """For `rocprofv3 --pmc` runs on the matrix-core residual: `reps` calls of dmmv_residual
    with options.residual_mfma on batched workload idx, nothing else."""
    import torch
    from paper_2508_13437_amd import dmmv
    from workloads import make_config

    inst = make_config(idx)
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    with dmmv.from_instance(inst, device, residual_mfma=True) as h:
        dmmv.dmmv_set_x(h, x0)
        for _ in range(reps):
            dmmv.dmmv_residual(h)
        torch.cuda.synchronize()
    print(json.dumps({"probe": inst.name, "residual_calls": reps,
                      "useful_flops_per_call": 2.0 * inst.m * inst.n * inst.R}))


def descent_probe(idx: int, device: str, reps: int) -> None:
    """For `rocprofv3 --pmc` runs on the pruned batched descent: `reps` calls of dmmv_solve with
    options.prune on batched workload idx (one launch of k_descent_batched_pruned each)."""
    import torch
    from paper_2508_13437_amd import dmmv
    from workloads import make_config

    inst = make_config(idx)
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    with dmmv.from_instance(inst, device, prune=True) as h:
        for _ in range(reps):
            out = dmmv.dmmv_solve(h, x0, inst.iters)
        torch.cuda.synchronize()
        moves = out.iters_done.cpu().numpy().astype(np.int64)
    print(json.dumps({"probe": inst.name, "descents": reps, "moves_applied_per_descent": int(moves.sum()),
                      "instance_iterations_per_descent": int(moves.sum() + (moves < inst.iters).sum()),
                      "candidates_per_instance_iteration": int(inst.n * (inst.nd - 1))}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="headline workload (1..5)")
    ap.add_argument("--iters", type=int, default=None, help="override iterations per step")
    ap.add_argument("--others", type=str, default="1,2,4,5",
                    help="comma list of further configs reported under other_workloads in the same "
                         "line ('' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=15.0)
    ap.add_argument("--traffic-probe", type=int, default=0, metavar="REPS",
                    help="only launch the evaluation kernel REPS times plus a calibration copy "
                         "(for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--residual-probe", type=int, default=0, metavar="REPS",
                    help="only run the matrix-core batched residual REPS times (for rocprofv3 --pmc runs)")
    ap.add_argument("--descent-probe", type=int, default=0, metavar="REPS",
                    help="only run the pruned batched descent REPS times (for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    device = "cuda:0"
    if args.traffic_probe > 0:
        traffic_probe(args.config, device, args.traffic_probe)
        return
    if args.residual_probe > 0:
        residual_probe(args.config, device, args.residual_probe)
        return
    if args.descent_probe > 0:
        descent_probe(args.config, device, args.descent_probe)
        return
    default_steps = {1: 20, 2: 10, 3: 5, 4: 1, 5: 1}
    steps = args.steps if args.steps is not None else default_steps[args.config]
    head = run_config(args.config, steps, args.warmup, args.iters, device,
                      not args.no_cpu_baseline, args.cpu_budget)
    line = {
        "metric": "candidate_moves_evaluated_per_sec", "value": head["moves_per_sec"],
        "unit": "moves/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "m": head["m"], "n": head["n"], "nd": head["nd"],
                   "R": head["R"], "nnz": head["nnz"], "iters_per_step": head["iters_per_step"],
                   "mode": "fixed-work (keep_going): every iteration scores all moves"},
        "iters_per_sec": head["iters_per_sec"], "us_per_iter": head["us_per_iter"],
        "improving_moves_applied": head["improving_moves_applied"],
        "final_max_violation": head["final_max_violation"],
        "roofline": head["roofline"],
    }
    if "residual" in head:
        line["residual"] = head["residual"]
    for key in ("eval_matrix_core_ms", "eval_vector_unit_ms"):
        if key in head:
            line[key] = head[key]
    if "descent" in head:
        line["descent"] = head["descent"]
    if "alns" in head:
        line["alns"] = head["alns"]
    if "alns_value_search" in head:
        line["alns_value_search"] = head["alns_value_search"]
    if "alns_full_evaluation" in head:
        line["alns_full_evaluation"] = head["alns_full_evaluation"]
    if "swap" in head:
        line["swap"] = head["swap"]
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    others = [int(v) for v in args.others.split(",") if v.strip() and int(v) != args.config]
    if others:
        line["other_workloads"] = []
        for idx in others:
            o = run_config(idx, default_steps[idx], 1 if idx < 4 else 0, None, device, False, 0)
            line["other_workloads"].append(o)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
