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
PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(workload: str):
    """HBM-side bytes per launch of the evaluation kernel, as `--traffic-summary` wrote them from two
    rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) calibrated against a plain copy; None when
    no such summary has been made for this workload."""
    path = os.path.join(PROFILES, f"hbm_traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f)


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


def roofline_for(inst, eval_ms: float, iter_us=None, cold_ms=None) -> dict:
    dt = "f64" if inst.dtype == np.float64 else "f32"
    if inst.kind == "csr":
        b = algorithmic_bytes_per_eval(inst)
        ach = b / (eval_ms * 1e-3) / 1e9
        tr = measured_traffic(inst.name)
        out = {"bound": "hbm", "kernel": "k_eval_fused", "achieved": ach, "peak": HBM_PEAK_GBS,
               "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
               "traffic": None if tr is None else tr["bytes_per_launch"],
               "algorithmic_bytes_per_launch": b, "avg_launch_ms": eval_ms,
               "covers": "the whole evaluation step (one kernel: stream every row partition, add the rows "
                         "outside each column, reduce to the arg-min records), launches back to back"}
        if tr is not None:
            out["measured_GBs"] = tr["bytes_per_launch"] / (eval_ms * 1e-3) / 1e9
            out["frac_measured"] = out["measured_GBs"] / HBM_PEAK_GBS
            out["traffic_source"] = tr.get("source")
        if iter_us is not None:
            # the same bytes over a whole iteration of the loop (evaluation + select/apply)
            out["iteration_us"] = iter_us
            out["frac_iteration"] = b / (iter_us * 1e-6) / 1e9 / HBM_PEAK_GBS
        if cold_ms is not None:
            # every launch preceded by a flush of the 256 MB Infinity Cache and the L2s (a 1 GiB
            # device-to-device copy, or a 1 GiB read): nothing of the matrix is left on the chip, so
            # these are rates out of HBM itself; after the copy the reads also push written lines out
            out["cold_launch_ms"], out["cold_after_read_ms"] = cold_ms[0], cold_ms[1]
            out["device_copy_GBs_measured"] = cold_ms[2]
            out["cold_GBs"] = b / (cold_ms[0] * 1e-3) / 1e9
            out["frac_cold"] = out["cold_GBs"] / HBM_PEAK_GBS
            out["cold_after_read_GBs"] = b / (cold_ms[1] * 1e-3) / 1e9
            out["frac_cold_after_read"] = out["cold_after_read_GBs"] / HBM_PEAK_GBS
        return out
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
    def once():
        if inst.kind == "csr":
            return orc.solve_csr(inst.m, inst.n, inst.csr_rowptr, inst.csr_col, inst.csr_val, inst.b,
                                 inst.D, inst.x0, iters)
        return orc.solve_dense(inst.A, inst.b, inst.D, inst.x0, iters)

    # a descent that stalls after a move or two is over in milliseconds: repeat it until the clock
    # has something to measure (the same evaluations every time)
    t0 = time.perf_counter()
    runs = 0
    while True:
        res = once()
        runs += 1
        dt = time.perf_counter() - t0
        if dt >= min(0.5, budget_s) or runs >= 1000:
            break
    evals = min(res.iters_done + 1, iters)
    moves = runs * evals * inst.n * (inst.nd - 1)
    return {"value": moves / dt, "unit": "moves/s", "cores": 1, "kind": "oracle",
            "sample": f"{runs} run(s) of {evals} evaluations from the configured start (of {inst.iters} "
                      f"iterations), {dt:.1f} s",
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
        loop = "all iterations in one launch" if dmmv.dmmv_loop_in_use(h) == 2 else "launches per iteration"
        cold_ms = cold_eval_ms(h, device) if inst.kind == "csr" else None
    moves = float(steps) * iters * inst.moves_per_iter()
    out.update({
        "workload": inst.name, "kind": inst.kind, "m": inst.m, "n": inst.n, "nd": inst.nd,
        "R": inst.R, "nnz": inst.nnz, "iters_per_step": iters, "loop": loop,
        "moves_per_sec": moves / dt, "iters_per_sec": steps * iters / dt,
        "instance_iters_per_sec": steps * iters * inst.R / dt,
        "ms_per_step": dt / steps * 1e3, "us_per_iter": dt / (steps * iters) * 1e6,
        "improving_moves_applied": int(improving.sum()),
        "descent_until_local_optimum_ms": normal_s * 1e3,
        "final_max_violation": float(t_final.max()),
        "dtype": "f64" if inst.dtype == np.float64 else "f32",
        "roofline": roofline_for(inst, eval_ms, dt / (steps * iters) * 1e6, cold_ms), "input_gen_s": round(t_gen, 2),
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
        out["l2"] = l2_timing(inst, device, x0)
    if inst.kind == "dense":
        out["descent"] = descent_timing_dense(inst, device, iters)
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
        # and with the pruned local search, one launch per outer iteration (small instances only)
        out["alns_pruned_local_search"] = alns_timing(inst, device, x0, prune=True)
    out["swap"] = swap_timing(inst, device, x0, iters)
    if do_cpu:
        out["cpu_baseline"] = cpu_baseline(inst, cpu_budget)
    return out


def cold_eval_ms(h, device: str, reps: int = 8):
    """One evaluation launch timed right after the caches were flushed on the same stream, averaged over
    `reps` such launches.  Two flushes: a 1 GiB device-to-device copy (it leaves the Infinity Cache
    full of written lines, which the evaluation's reads then push out to HBM), and a read of 1 GiB
    (clean lines only).  Either is long enough for the launch to be enqueued behind it."""
    import torch
    from paper_2508_13437_amd import dmmv

    src = torch.empty(1 << 28, dtype=torch.int32, device=device).fill_(1)
    dst = torch.empty_like(src)
    after_copy = after_read = 0.0
    with torch.cuda.stream(h.stream):
        for _ in range(reps):
            dst.copy_(src)
            after_copy += dmmv.dmmv_time_eval(h, -1)
        for _ in range(reps):
            src.max()
            after_read += dmmv.dmmv_time_eval(h, -1)
    # what a plain device-to-device copy of 1 GiB reaches on this device (read + written bytes per second)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(h.stream):
        dst.copy_(src)
        e0.record(h.stream)
        for _ in range(4):
            dst.copy_(src)
        e1.record(h.stream)
    e1.synchronize()
    copy_gbs = 4 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    return after_copy / reps, after_read / reps, copy_gbs


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


def descent_timing_dense(inst, device: str, iters: int) -> dict:
    """A dense single instance, three ways to iterate, the same moves from each: a launch of the
    evaluation and one of selection + apply per iteration (options.dense_loop = 1); all iterations
    in one launch of a fixed grid of workgroups that exchange one arg-min record per iteration
    (dense_loop = 2, when the instance fits); options.prune, one workgroup and one launch (bounds on
    16 rows, full scores best-first; small instances).  Two figures each: the time per iteration in
    fixed-work mode (every iteration scores all moves, nothing improves at the configured start),
    and the wall time of the real descent from a seeded RANDOM starting point (the configured one is
    a local optimum already).  EFFECTIVE rates, apart from `value`."""
    import torch
    from paper_2508_13437_amd import dmmv

    x_cfg = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    x0 = torch.from_numpy(np.random.default_rng(7).choice(inst.D, size=inst.n)).to(device)
    res = {}
    for key, opt in (("launch_per_step", {"dense_loop": 1}), ("one_launch", {"dense_loop": 2}),
                     ("pruned_one_launch", {"prune": True})):
        try:
            h_fixed = dmmv.from_instance(inst, device, keep_going=True, poll_every=0, **opt)
        except dmmv.DmmvError as e:
            res[key] = {"skipped": str(e)}
            continue
        entry = {}
        if key != "pruned_one_launch":          # the pruned descent has no fixed-work mode: it stops by itself
            with h_fixed as h:
                fixed = []
                for n_it in (200, 2200):
                    dmmv.dmmv_solve(h, x_cfg, n_it)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    dmmv.dmmv_solve(h, x_cfg, n_it)
                    torch.cuda.synchronize()
                    fixed.append(time.perf_counter() - t0)
                entry["fixed_work_us_per_iter"] = (fixed[1] - fixed[0]) / 2000 * 1e6
                entry["fixed_work_iters_per_sec"] = 2000 / (fixed[1] - fixed[0])
        else:
            h_fixed.close()
        with dmmv.from_instance(inst, device, poll_every=64, **opt) as h:
            dmmv.dmmv_solve(h, x0, iters)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            out = dmmv.dmmv_solve(h, x0, iters)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
        moves = int(out.iters_done.cpu()[0])
        entry.update({"descent_ms": dt * 1e3, "moves_applied": moves, "us_per_move": dt * 1e6 / max(moves, 1),
                      "final_max_violation": float(out.max_violation.cpu()[0])})
        res[key] = entry
    ran = [v for v in res.values() if "moves_applied" in v]
    res["same_moves_and_error"] = all(v["moves_applied"] == ran[0]["moves_applied"] and
                                      v["final_max_violation"] == ran[0]["final_max_violation"] for v in ran)
    res["note"] = ("fixed_work: time of 2000 further iterations inside one dmmv_solve call (a 2200-iteration call "
                   "minus a 200-iteration call); descent: wall time of dmmv_solve from a random starting point until "
                   "the local optimum or the configured iteration count (launch_per_step: the host polls every 64 "
                   "iterations)")
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


def l2_timing(inst, device: str, x0) -> dict:
    """The l2 change of every candidate (options.l2_rule): G = X^T R_mat for the whole batch, on the
    matrix cores with one row of the contraction per instruction (fp32), timed with events on the
    library's stream; and one iteration of the descent with the l2 change as second criterion."""
    import torch
    from paper_2508_13437_amd import dmmv

    flops = 2.0 * inst.m * inst.n * inst.R
    with dmmv.from_instance(inst, device, l2_rule=1) as h:
        dmmv.dmmv_set_x(h, x0)
        dmmv.dmmv_residual(h)
        ms = dmmv.dmmv_time_l2(h, 5) / 5
        dmmv.dmmv_solve(h, x0, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dmmv.dmmv_solve(h, x0, 3)
        torch.cuda.synchronize()
        it_ms = (time.perf_counter() - t0) / 3 * 1e3
    peak = 157.3
    return {"kernel": "k_l2_g_mfma" if inst.dtype == np.float32 else "k_l2_g_batched", "flops": flops, "ms": ms,
            "TFLOPs": flops / (ms * 1e-3) / 1e12, "peak_TFLOPs_fp32_matrix": peak,
            "frac": flops / (ms * 1e-3) / 1e12 / peak,
            "ms_per_iteration_with_l2_rule": it_ms,
            "note": "ms_per_iteration_with_l2_rule: dmmv_solve with options.l2_rule = 1 (residual included, 3 "
                    "iterations): score table written, G recomputed, arg-min over (score, l2 change, index)"}


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


def traffic_summary(idx: int, fetch_dir: str, write_dir: str) -> None:
    """Turn the counter CSVs of the two --traffic-probe runs into profiles/hbm_traffic_<workload>.json.
    Both counters are read in KiB per dispatch; each is scaled by what it reads for the probe's plain
    256 MiB copy (whose bytes are known).  Runs on the CPU."""
    import csv
    import glob

    def per_kernel(d, counter):
        files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
        if not files:
            raise SystemExit(f"no *counter_collection.csv under {d}")
        acc = {}
        for path in files:
            with open(path, newline="") as f:
                for row in csv.DictReader(f):
                    if row.get("Counter_Name") != counter:
                        continue
                    name = row["Kernel_Name"].split("(")[0]
                    acc.setdefault(name, []).append((int(row["Grid_Size"]), float(row["Counter_Value"])))
        return acc

    from workloads import CONFIG_NAMES
    fetch, write = per_kernel(fetch_dir, "FETCH_SIZE"), per_kernel(write_dir, "WRITE_SIZE")

    def pick(acc, needle):
        hits = [k for k in acc if needle in k]
        if len(hits) != 1:
            raise SystemExit(f"expected one kernel matching {needle!r}, found {hits}")
        return hits[0], acc[hits[0]]

    copy_bytes = 256 << 20
    # the probe's 256 MiB copy is the largest dispatch of the copy kernel (uploads use it too)
    cf = max(pick(fetch, "copyBuffer")[1])[1]
    cw = max(pick(write, "copyBuffer")[1])[1]
    f_scale = copy_bytes / 1024.0 / cf
    w_scale = copy_bytes / 1024.0 / cw
    kname, kf = pick(fetch, "k_eval_")
    _, kw = pick(write, "k_eval_")
    kf, kw = [v for _, v in kf], [v for _, v in kw]
    fetched = sum(kf) / len(kf) * 1024.0 * f_scale
    written = sum(kw) / len(kw) * 1024.0 * w_scale
    out = {"workload": CONFIG_NAMES[idx], "kernel": kname, "launches": len(kf),
           "fetch_KiB_raw": sum(kf) / len(kf), "write_KiB_raw": sum(kw) / len(kw),
           "fetch_scale": f_scale, "write_scale": w_scale,
           "bytes_fetched": fetched, "bytes_written": written, "bytes_per_launch": fetched + written,
           "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --traffic-probe`, scaled by the "
                     "same counters' reading for a 256 MiB device-to-device copy"}
    path = os.path.join(PROFILES, f"hbm_traffic_{CONFIG_NAMES[idx]}.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out))


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


def l2_probe(idx: int, device: str, reps: int) -> None:
    """For `rocprofv3 --pmc` runs on the contraction behind the l2 changes: `reps` launches of
    g = A^T r (a batch: G = X^T R_mat on the matrix cores) on workload idx, nothing else timed."""
    import torch
    from paper_2508_13437_amd import dmmv
    from workloads import make_config

    inst = make_config(idx)
    x0 = torch.from_numpy(np.ascontiguousarray(inst.x0)).to(device)
    with dmmv.from_instance(inst, device, l2_rule=3) as h:
        dmmv.dmmv_set_x(h, x0)
        dmmv.dmmv_residual(h)
        ms = dmmv.dmmv_time_l2(h, reps) / reps
        torch.cuda.synchronize()
    print(json.dumps({"probe": inst.name, "l2_launches": reps + 1, "ms_per_launch": ms,
                      "multiply_adds_per_launch": float(inst.m) * inst.n * inst.R}))


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
    ap.add_argument("--cpu-budget-others", type=float, default=4.0,
                    help="seconds of oracle time per workload of --others")
    ap.add_argument("--traffic-summary", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), default=None,
                    help="no GPU: read the counter CSVs of two `rocprofv3 --pmc` runs of --traffic-probe "
                         "(FETCH_SIZE, WRITE_SIZE) and write profiles/hbm_traffic_<workload>.json")
    ap.add_argument("--traffic-probe", type=int, default=0, metavar="REPS",
                    help="only launch the evaluation kernel REPS times plus a calibration copy "
                         "(for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--residual-probe", type=int, default=0, metavar="REPS",
                    help="only run the matrix-core batched residual REPS times (for rocprofv3 --pmc runs)")
    ap.add_argument("--l2-probe", type=int, default=0, metavar="REPS",
                    help="only launch the contraction g = A^T r of the l2 changes REPS times on --config (for rocprofv3 --pmc)")
    ap.add_argument("--descent-probe", type=int, default=0, metavar="REPS",
                    help="only run the pruned batched descent REPS times (for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.traffic_summary:
        traffic_summary(args.config, *args.traffic_summary)
        return
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
    if args.l2_probe > 0:
        l2_probe(args.config, device, args.l2_probe)
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
                   "mode": "fixed-work (keep_going): every iteration scores all moves", "loop": head["loop"]},
        "iters_per_sec": head["iters_per_sec"], "us_per_iter": head["us_per_iter"],
        "improving_moves_applied": head["improving_moves_applied"],
        "final_max_violation": head["final_max_violation"],
        "roofline": head["roofline"],
    }
    import torch
    prop = torch.cuda.get_device_properties(device)
    line["device"] = {"name": prop.name, "compute_units": prop.multi_processor_count,
                      "memory_GiB": round(prop.total_memory / 2**30, 1),
                      "gcn_arch": getattr(prop, "gcnArchName", None),
                      "peaks_used": {"hbm_GBs": HBM_PEAK_GBS, "fp32_TFLOPs": 157.3, "fp64_TFLOPs": 78.6}}
    if "residual" in head:
        line["residual"] = head["residual"]
    if "l2" in head:
        line["l2"] = head["l2"]
    for key in ("eval_matrix_core_ms", "eval_vector_unit_ms"):
        if key in head:
            line[key] = head[key]
    if "descent" in head:
        line["descent"] = head["descent"]
    if "alns" in head:
        line["alns"] = head["alns"]
    if "alns_value_search" in head:
        line["alns_value_search"] = head["alns_value_search"]
    if "alns_pruned_local_search" in head:
        line["alns_pruned_local_search"] = head["alns_pruned_local_search"]
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
            # the oracle on a small bounded sample of each (a few seconds): a reported baseline
            o = run_config(idx, default_steps[idx], 1 if idx < 4 else 0, None, device,
                           not args.no_cpu_baseline, args.cpu_budget_others)
            line["other_workloads"].append(o)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
