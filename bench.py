#!/usr/bin/env python3
"""Benchmark of the commitment sweep on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config2]

A step is one pass of the whole hot path over one batch: generate the batch's candidates
on the device (seeded flat-Dirichlet rows or the simplex lattice), sweep them (follower
payoffs, tie-broken best responses, leader value, arg-max), and bring the result (best
value, best index, K best responses) back to the host.  Payoffs and prior are resident in
HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "valu": 78.6, "valu_bf16": 78.6}

# workload -> (config number, candidates per step, note)
WORKLOADS = {
    "config1": (1, None, "m=n=3 K=2 lattice N=100 (5151 candidates)"),
    "config2": (2, 1 << 20, "m=n=8 K=4, 2^20 Dirichlet(1) candidates"),
    "config3": (3, 1 << 24, "m=n=32 K=16 misalignment-structured, 2^24 candidates"),
    "config4_chunk": (4, 1 << 22, "m=64 n=128 K=64 bf16, one 2^22-candidate chunk of the 2^26"),
    "config5_sub": (5, 1 << 16, "m=128 n=256 K=256 integer payoffs, 2^16-candidate sub-range of the 2^24"),
}


def run_workload(name, steps, warmup, want_cpu_baseline=True):
    import numpy as np
    import torch
    from paper_2605_18856_amd import bsse, workloads

    cfg, count, note = WORKLOADS[name]
    game = workloads.game(cfg)
    storage = bsse.BSSE_STORAGE_BF16 if game.storage == "bf16" else bsse.BSSE_STORAGE_F32
    g = bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior, storage=storage)
    path = bsse.bsse_path_name(g)
    lattice = game.candidates == "lattice"
    if lattice:
        count = bsse.bsse_lattice_count(game.m, game.lattice_N)
        Xd = None
    else:
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")

    def step(k):
        if lattice:
            bsse.bsse_lattice(g, game.lattice_N)
            return bsse.bsse_sweep(g)
        # a fresh batch of the seeded sequence every step
        bsse.bsse_dirichlet(g, game.candidate_seed, k * count, count, Xd)
        return bsse.bsse_sweep(g, Xd, count)

    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    bsse.bsse_set_timing(g, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        out = step(warmup + k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms, launches = bsse.bsse_get_timing(g)
    bsse.bsse_set_timing(g, False)

    ms_per_step = (t1 - t0) * 1e3 / steps
    evals = count * game.K
    value = evals / (ms_per_step * 1e-3)
    k_ms = kernel_ms / max(launches, 1)

    flops = evals * (2.0 * game.m * game.n + 2.0 * game.m)       # algorithmic, per launch
    bytes_ = count * 4.0 * game.m                                  # candidate rows read once
    ai = flops / bytes_
    if path.startswith("mfma"):
        bound, unit, peak = "mfma", "TFLOP/s", PEAK_TFLOPS[path]
        achieved = flops / (k_ms * 1e-3) / 1e12
    elif ai > PEAK_TFLOPS["valu"] * 1e12 / (HBM_PEAK_GBS * 1e9):
        bound, unit, peak = "alu", "TFLOP/s", PEAK_TFLOPS["valu"]
        achieved = flops / (k_ms * 1e-3) / 1e12
    else:
        bound, unit, peak = "hbm", "GB/s", HBM_PEAK_GBS
        achieved = bytes_ / (k_ms * 1e-3) / 1e9
    roofline = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": None, "kernel": "fused sweep (" + path + ")",
                "kernel_ms": k_ms, "launches": launches,
                "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": bytes_}

    cpu = None
    if want_cpu_baseline:
        from oracle import sweep as osweep
        cores = len(os.sched_getaffinity(0))
        # bounded sample: calibrate on a few rows, then size the sample for ~12 s of oracle
        # work; when the whole batch takes less, repeat passes over the batch instead
        if lattice:
            Xall = bsse.candidates_to_host(g)
        else:
            Xall = None
        def rows(k):
            Xh = Xall[:k] if lattice else Xd[:k].cpu().numpy()
            return workloads.round_to_bf16(Xh) if game.storage == "bf16" else Xh
        probe = int(min(count, max(16, 2_000_000 // (game.K * game.m * game.n))))
        Xp = rows(probe)
        osweep.sweep(game.A, game.B, game.prior, Xp[:2], per_candidate=False, nthreads=cores)
        c0 = time.perf_counter()
        osweep.sweep(game.A, game.B, game.prior, Xp, per_candidate=False, nthreads=cores)
        per_row = max((time.perf_counter() - c0) / probe, 1e-9)
        sample = int(min(count, max(probe, 12.0 / per_row)))
        passes = max(1, int(12.0 / (per_row * sample))) if sample == count else 1
        passes = min(passes, 2000)
        Xh = rows(sample)
        c0 = time.perf_counter()
        for _ in range(passes):
            ref = osweep.sweep(game.A, game.B, game.prior, Xh, per_candidate=False, nthreads=cores)
        c1 = time.perf_counter()
        cpu = {"value": passes * sample * game.K / (c1 - c0), "unit": "candidate-type evals/s",
               "cores": ref.threads, "kind": "oracle",
               "sample": f"{passes} pass(es) over the first {sample} candidates of the step's "
                         f"batch of {count} ({c1 - c0:.1f} s of oracle time, fp64, OpenMP over candidates)"}
    g.close()
    return {
        "ms_per_step": ms_per_step, "value": value, "path": path, "count": count,
        "game": game, "roofline": roofline, "cpu_baseline": cpu, "note": note,
        "best_index": out.best_index, "best_value": out.best_value,
        "n_tie_evals": out.n_tie_evals,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="config2", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the sweep has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    default_steps = {"config1": 200, "config2": 200, "config3": 20, "config4_chunk": 3, "config5_sub": 3}
    steps = args.steps if args.steps is not None else default_steps[args.workload]
    warmup = args.warmup if args.warmup is not None else max(1, min(10, steps // 4))
    r = run_workload(args.workload, steps, warmup, not args.no_cpu_baseline)
    game = r["game"]
    line = {
        "metric": "candidate-type evals/sec at 1 MI355X",
        "value": r["value"], "unit": "candidate-type evals/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if game.storage == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "description": r["note"], "m": game.m, "n": game.n,
                   "K": game.K, "candidates_per_step": r["count"], "path": r["path"],
                   "step": "generate candidates + sweep + result to host"},
        "roofline": r["roofline"],
        "cpu_baseline": r["cpu_baseline"],
        "result": {"best_index": r["best_index"], "best_value": r["best_value"],
                   "n_tie_evals": r["n_tie_evals"]},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
