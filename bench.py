#!/usr/bin/env python3
"""Benchmark of the commitment sweep on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config4]

A step is one pass of the whole hot path over one whole configuration: every candidate of the
configuration is generated on the device (seeded flat-Dirichlet rows, or the simplex lattice),
swept (follower payoffs, tie-broken best responses, leader value, arg-max) and merged into the
running best, chunk by chunk where the configuration is streamed (config 4: sixteen chunks of
2^22 candidates).  The K timed steps are K such passes over consecutive ranges of the seeded
sequence, chunks of ONE streamed sweep: the result (best value, best index, best responses) comes
back to the host after the last step, inside the timed region; the figure with a result brought
back after every step is reported beside it.  Payoffs and prior are resident in HBM before the
timed region.  Prints ONE JSON line.

The headline workload is config 4 (m = 64, n = 128, K = 64, bf16 storage, 2^26 candidates), the
largest dense configuration; the others are reported under "other_workloads".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "valu": 78.6, "valu_bf16": 78.6,
               # fp32 operands split into bf16 parts run on the bf16 matrix cores: priced against
               # that peak with ALGORITHMIC flops (the kernel executes 3x / 6x as many)
               "mfma_split3": 2500.0, "mfma_split6": 2500.0, "mfma_small_split6": 2500.0}
EXECUTED_FLOP_FACTOR = {"mfma_split3": 3.0, "mfma_split6": 6.0, "mfma_small_split6": 6.0}

# HBM bytes per launch of the fused sweep kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# (profiles/sweep_kernels_hbm_traffic.md; FETCH_SIZE reads half of a known-size copy on this part,
# so it is scaled by 2.0; WRITE_SIZE reads a known-size fill exactly).  Keyed by workload; one
# launch = one chunk.
TRAFFIC_BYTES = {
    "config2": (155.9 * 2.0 + 29.0) * 1024.0,          # rows generated in registers: slots and payoffs only
    "config3": (1050370.0 * 2.0 + 4097.3) * 1024.0,
    "config4": (673309.0 * 2.0 + 270.1) * 1024.0,
    "config5": (1867050.0 * 2.0 + 301.7) * 1024.0,
}

# Matrix and vector instructions a wavefront alternates between in the fused sweep kernel of a
# workload, from the rocprofv3 counters in profiles/ (SQ_INSTS_MFMA and SQ_INSTS_VALU minus it, per
# wavefront and block of one type, rounded to the measurement's granularity of 24): config 4, one
# pass of two candidate tiles: 32 and 2 x 156; config 3, two candidate tiles: 24 and 2 x 105;
# config 5, one tile: 192 and 379.
MIXES = {"config4": (32, 312), "config3": (24, 216), "config5": (192, 384)}

# workload -> (config number, candidates per step, candidates per chunk (= per launch), note)
WORKLOADS = {
    "config1": (1, None, None, "m=n=3 K=2 lattice N=100 (5151 candidates)"),
    "config2": (2, 1 << 20, 1 << 20, "m=n=8 K=4, 2^20 Dirichlet(1) candidates, rows made inside the sweep kernel"),
    "config3": (3, 1 << 24, 1 << 24, "m=n=32 K=16 misalignment-structured, 2^24 candidates in one launch"),
    "config4": (4, 1 << 26, 1 << 22, "m=64 n=128 K=64 bf16, 2^26 candidates streamed in 16 chunks of 2^22"),
    "config5": (5, 1 << 24, 1 << 20, "m=128 n=256 K=256 integer payoffs, 2^24 candidates streamed in 16 chunks of 2^20"),
}
DEFAULT_STEPS = {"config1": (200, 10), "config2": (200, 10), "config3": (20, 3), "config4": (6, 1),
                 "config5": (2, 1)}


def cpu_baseline_leg(game, g, count_chunk, lattice, with_parity):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the
    workload's first chunk (about 12 s of oracle time on all cores, 3 s on one); the GPU's
    per-candidate outputs on the same sample are compared with it (parity counts)."""
    import numpy as np
    import torch
    from oracle import sweep as osweep
    from paper_2605_18856_amd import bsse, workloads

    cores = len(os.sched_getaffinity(0))
    if lattice:
        Xall = bsse.candidates_to_host(g)
        count = Xall.shape[0]
        Xd = None
    else:
        Xall = None
        count = count_chunk
        Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, Xd)
        torch.cuda.synchronize()

    def rows(k):
        return Xall[:k] if lattice else Xd[:k].cpu().numpy()

    def feed(Xh):          # the operand values the kernel is defined to consume
        return workloads.round_to_bf16(Xh) if game.storage == "bf16" else Xh

    A = workloads.round_to_bf16(game.A) if game.storage == "bf16" else game.A
    B = workloads.round_to_bf16(game.B) if game.storage == "bf16" else game.B
    probe = int(min(count, max(16, 2_000_000 // (game.K * game.m * game.n))))
    Xp = feed(rows(probe))
    osweep.sweep(A, B, game.prior, Xp[:2], per_candidate=False, nthreads=cores)
    c0 = time.perf_counter()
    osweep.sweep(A, B, game.prior, Xp, per_candidate=False, nthreads=cores)
    per_row = max((time.perf_counter() - c0) / probe, 1e-9)
    sample = int(min(count, max(probe, 4096, 12.0 / per_row)))
    Xraw = rows(sample)
    Xh = feed(Xraw)
    passes = 0
    c0 = time.perf_counter()
    while True:
        ref = osweep.sweep(A, B, game.prior, Xh, per_candidate=False, nthreads=cores)
        passes += 1
        c1 = time.perf_counter()
        if c1 - c0 >= 10.0 or passes >= 20000:        # (the probe over-estimates the cost per row)
            break
    n1 = int(max(16, min(sample, 3.0 / (per_row * max(cores, 1)))))
    s0 = time.perf_counter()
    p1 = 0
    while True:
        osweep.sweep(A, B, game.prior, Xh[:n1], per_candidate=False, nthreads=1)
        p1 += 1
        s1 = time.perf_counter()
        if s1 - s0 >= 3.0 or p1 >= 20000 or n1 < sample:
            break
    cpu = {"value": passes * sample * game.K / (c1 - c0), "unit": "candidate-type evals/s",
           "single_thread_value": p1 * n1 * game.K / (s1 - s0),
           "cores": ref.threads, "kind": "oracle",
           "extrapolated": bool(sample < count),
           "sample": f"{passes} pass(es) over the first {sample} candidates of the first chunk "
                     f"({count} candidates) of the workload ({c1 - c0:.1f} s of oracle time, fp64, "
                     f"OpenMP over candidates)"}
    if with_parity:
        # the same sample through the library's per-candidate outputs, against the oracle
        from tests import parity
        n = int(min(sample, 8192))
        Xs = torch.from_numpy(np.ascontiguousarray(Xraw[:n])).cuda()
        V = torch.empty(n, dtype=torch.float32, device="cuda")
        br = torch.empty((n, game.K), dtype=torch.int32, device="cuda")
        bsse.bsse_eval(g, Xs, n, V, br)
        torch.cuda.synchronize()
        rep = parity.compare_eval(game, Xraw[:n], V.cpu().numpy(), br.cpu().numpy(), nthreads=cores)
        cpu["parity_counts"] = {"rows": n, "evaluations": rep.n_evals,
                                "best_response_mismatches": rep.br_mismatch,
                                "flagged_gap_below_1e-6": rep.flagged,
                                "bound_explained": rep.bound_explained, "hard": rep.hard_failures,
                                "max_value_err_rel": rep.max_value_err,
                                "value_failures": rep.value_failures}
    return cpu


def run_workload(name, steps, warmup, want_cpu_baseline=True):
    import torch
    from paper_2605_18856_amd import bsse, workloads

    cfg, total, chunk, note = WORKLOADS[name]
    game = workloads.game(cfg)
    storage = bsse.BSSE_STORAGE_BF16 if game.storage == "bf16" else bsse.BSSE_STORAGE_F32
    g = bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior, storage=storage)
    path = bsse.bsse_path_name(g)
    lattice = game.candidates == "lattice"
    if lattice:
        total = chunk = bsse.bsse_lattice_count(game.m, game.lattice_N)
        Xd = None
    else:
        Xd = torch.empty((chunk, game.m), dtype=torch.float32, device="cuda")
    nchunks = total // chunk

    # games on the small-game kernel generate their rows inside the sweep kernel
    fused = name == "config2"

    def step(k):
        # a fresh range of the seeded sequence every step; the lattice is the same set every time
        for c in range(nchunks):
            base = k * total + c * chunk
            if lattice:
                bsse.bsse_lattice(g, game.lattice_N)
                bsse.bsse_sweep_chunk(g, None, 0, 0)
            elif fused:
                bsse.bsse_sweep_dirichlet_chunk(g, game.candidate_seed, base, chunk, base)
            else:
                bsse.bsse_dirichlet(g, game.candidate_seed, base, chunk, Xd)
                bsse.bsse_sweep_chunk(g, Xd, chunk, base)

    def run(first, n, each):
        """n steps; each: a result on the host after every step, else once after the last"""
        out = None
        bsse.bsse_sweep_reset(g)
        for k in range(first, first + n):
            step(k)
            if each:
                out = bsse.bsse_sweep_result(g)
                bsse.bsse_sweep_reset(g)
        return out if each else bsse.bsse_sweep_result(g)

    run(0, warmup, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = run(warmup, steps, False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # the same steps with a result on the host after every step
    run(warmup, steps, True)
    torch.cuda.synchronize()
    ms_per_step_each = (time.perf_counter() - t1) * 1e3 / steps
    # and once more with a HIP event pair around every launch of the sweep kernel (on the stream
    # the library launches it on): the kernel's own duration, for the roofline; not part of
    # `value`, the event pairs cost a few microseconds per launch
    bsse.bsse_set_timing(g, True)
    run(warmup, steps, False)
    torch.cuda.synchronize()
    kernel_ms, launches = bsse.bsse_get_timing(g)
    bsse.bsse_set_timing(g, False)

    ms_per_step = (t1 - t0) * 1e3 / steps
    evals = total * game.K
    value = evals / (ms_per_step * 1e-3)
    k_ms = kernel_ms / max(launches, 1)

    # algorithmic work of ONE launch (= one chunk): 2mn + 2m flops per candidate-type evaluation,
    # 4m bytes per candidate (rows read once; the payoffs stay in cache / LDS and are not counted)
    flops = chunk * game.K * (2.0 * game.m * game.n + 2.0 * game.m)
    bytes_ = 0.0 if fused else chunk * 4.0 * game.m
    flop_peak = PEAK_TFLOPS[path]
    t_hbm = bytes_ / (HBM_PEAK_GBS * 1e9)
    t_flop = flops * EXECUTED_FLOP_FACTOR.get(path, 1.0) / (flop_peak * 1e12)   # what the unit executes
    if t_hbm >= t_flop:
        bound, unit, peak = "hbm", "GB/s", HBM_PEAK_GBS
        achieved = bytes_ / (k_ms * 1e-3) / 1e9
    else:
        bound = "mfma" if path.startswith("mfma") else "alu"
        unit, peak = "TFLOP/s", flop_peak
        achieved = flops / (k_ms * 1e-3) / 1e12
    roofline = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": TRAFFIC_BYTES.get(name),
                "kernel": ("generate + sweep (" if fused else "fused sweep (") + path + ")",
                "kernel_ms": k_ms, "launches": launches, "candidates_per_launch": chunk,
                "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": bytes_}
    if fused:
        # Side figures for the kernel that also makes its rows (no candidate bytes exist, so no
        # memory roofline applies, and `frac` above counts the contraction flops alone): the same
        # kernel time priced with every arithmetic operation of the generator and of the sweep
        # (a builder-defined count: per 4 components one Philox4x32-10 block = 60 operations, ~10
        # per component from word to exponential, m - 1 additions, one division, m scalings; per
        # type 2mn + (n - 1) + n + 2m + 2), and the rate at the step time, where consecutive
        # launches overlap on two streams.
        m, n, K = game.m, game.n, game.K
        ops = chunk * ((m / 4.0) * 60.0 + m * 10.0 + (m - 1) + 1 + m + K * (2.0 * m * n + (n - 1) + n + 2.0 * m + 2.0))
        roofline["frac_counting_every_generator_and_argmax_operation"] = ops / (k_ms * 1e-3) / 1e12 / peak
        roofline["frac_at_step_rate"] = flops / (ms_per_step * 1e-3) / 1e12 / peak
    if path in EXECUTED_FLOP_FACTOR and bound == "mfma":
        # the split path does an fp32-accurate contraction with 3 or 6 bf16 products per term:
        # frac prices the algorithmic flops against the bf16 peak; these fields give the rate the
        # matrix cores actually run at and the comparison with the fp32 matrix-core peak
        roofline["executed_mfma_tflops"] = achieved * EXECUTED_FLOP_FACTOR[path]
        roofline["executed_frac"] = achieved * EXECUTED_FLOP_FACTOR[path] / peak
        roofline["frac_of_fp32_mfma_peak"] = achieved / PEAK_TFLOPS["mfma_f32"]

    cpu = cpu_baseline_leg(game, g, chunk, lattice, True) if want_cpu_baseline else None
    g.close()
    return {
        "ms_per_step": ms_per_step, "value": value, "path": path, "count": total, "chunk": chunk,
        "ms_per_step_each": ms_per_step_each, "fused": fused, "timed_region_s": t1 - t0,
        "game": game, "roofline": roofline, "cpu_baseline": cpu, "note": note,
        "best_index": out.best_index, "best_value": out.best_value,
        "n_tie_evals": out.n_tie_evals,
    }


def hbm_leg():
    """The memory-bound configuration (config-2 game, 32 bytes of candidate row per 4 evaluations)
    with rows READ FROM A BUFFER, on 2^26 candidates (2 GiB, eight times the last-level cache):
    the sweep kernel alone, HIP-event timed, as achieved HBM bandwidth."""
    import torch
    from paper_2605_18856_amd import bsse, workloads
    game = workloads.game(2)
    count = 1 << 26
    g = bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior)
    Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
    bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, Xd)
    bsse.bsse_sweep_reset(g)
    bsse.bsse_sweep_chunk(g, Xd, count, 0)
    bsse.bsse_set_timing(g, True)
    for _ in range(5):
        bsse.bsse_sweep_chunk(g, Xd, count, 0)
    ms, k = bsse.bsse_get_timing(g)
    out = bsse.bsse_sweep_result(g)
    # the same 2^26 rows generated inside the sweep kernel instead of read from the buffer
    bsse.bsse_sweep_reset(g)
    bsse.bsse_sweep_dirichlet_chunk(g, game.candidate_seed, 0, count, 0)
    bsse.bsse_set_timing(g, True)
    for _ in range(5):
        bsse.bsse_sweep_dirichlet_chunk(g, game.candidate_seed, 0, count, 0)
    ms_gen, k_gen = bsse.bsse_get_timing(g)
    out_gen = bsse.bsse_sweep_result(g)
    g.close()
    k_ms = ms / k
    gbs = count * 4.0 * game.m / (k_ms * 1e-3) / 1e9
    return {"workload": "config2 game, 2^26 candidates per launch, rows read from a 2 GiB buffer",
            "kernel_ms": k_ms,
            "evals_per_s": count * game.K / (k_ms * 1e-3), "bound": "hbm", "achieved": gbs,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": count * 4.0 * game.m,
            # rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE of this launch (profiles/sweep_kernels_hbm_traffic.md)
            "traffic": (1048810.0 * 2.0 + 11.4) * 1024.0,
            "best_index": out.best_index,
            "rows_generated_in_the_kernel": {"kernel_ms": ms_gen / k_gen,
                                             "evals_per_s": count * game.K / (ms_gen / k_gen * 1e-3),
                                             "best_index": out_gen.best_index}}


def prior_batch_leg(P=101, steps=20):
    """Prior-robustness batch (not part of `value`): the config-2 game and batch swept for P
    priors in one call, against P plain sweeps of the same batch."""
    import numpy as np
    import torch
    from paper_2605_18856_amd import bsse, workloads

    game = workloads.game(2)
    count = 1 << 20
    g = bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior)
    Xd = torch.empty((count, game.m), dtype=torch.float32, device="cuda")
    bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, Xd)
    rng = np.random.Generator(np.random.PCG64(4000))
    pri = rng.dirichlet(np.ones(game.K), size=P)
    pri = (pri / pri.sum(axis=1, keepdims=True)).astype(np.float32)
    for p in range(P):          # fp32 rows whose sum is within 1e-6 of 1
        pri[p, np.argmax(pri[p])] += np.float32(1.0 - pri[p].astype(np.float64).sum())
    for _ in range(3):
        bsse.bsse_sweep_priors(g, pri, Xd, count)
        bsse.bsse_sweep(g, Xd, count)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        bsse.bsse_sweep_priors(g, pri, Xd, count)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        bsse.bsse_sweep(g, Xd, count)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    ms_batch, ms_sweep = (t1 - t0) * 1e3 / steps, (t2 - t1) * 1e3 / steps
    g.close()
    return {"workload": "config2 game, 2^20 candidates, %d priors per call" % P, "priors": P,
            "ms_per_call": ms_batch, "ms_per_plain_sweep": ms_sweep,
            "candidate_type_prior_evals_per_s": count * game.K * P / (ms_batch * 1e-3),
            "speedup_over_one_sweep_per_prior": P * ms_sweep / ms_batch}


def refinement_leg(steps=10):
    """Survivors, local refinement and the LP polish (not part of `value`) on the config-2 game
    and its 2^20-candidate batch: wall time per call of bsse_sweep_topk (k = 64), bsse_refine
    (8 centres, 3 rounds of 4096-point clouds) and bsse_polish, and the values they reach."""
    import torch
    from paper_2605_18856_amd import bsse, workloads

    game = workloads.game(2)
    count = 1 << 20
    g = bsse.bsse_create(game.m, game.n, game.K, game.A, game.B, game.prior)
    bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, None)        # the handle-owned set
    sweep = bsse.bsse_sweep(g)
    bsse.bsse_sweep_topk(g, 64)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        vals, idx, _ = bsse.bsse_sweep_topk(g, 64)
    t1 = time.perf_counter()
    for _ in range(steps):
        bsse.bsse_sweep(g)
        pol = bsse.bsse_polish(g)
    t2 = time.perf_counter()
    ms_sweep_polish = (t2 - t1) * 1e3 / steps
    t3 = time.perf_counter()
    for _ in range(steps):
        bsse.bsse_sweep(g)
    ms_sweep = (time.perf_counter() - t3) * 1e3 / steps
    t4 = time.perf_counter()
    for _ in range(steps):
        # (the refinement leaves its last local set in the handle: start from the batch again)
        bsse.bsse_dirichlet(g, game.candidate_seed, 0, count, None)
        _, ref_v, _, ref_evals = bsse.bsse_refine(g, 8, 3, cloud_count=4096, seed=7, radius=0.25, shrink=0.25)
    ms_refine = (time.perf_counter() - t4) * 1e3 / steps
    g.close()
    return {"workload": "config2 game, 2^20 candidates (handle-owned set)",
            "sweep_value": sweep.best_value,
            "topk": {"k": 64, "ms_per_call": (t1 - t0) * 1e3 / steps, "kth_value": float(vals[-1])},
            "polish": {"ms_per_call": max(ms_sweep_polish - ms_sweep, 0.0), "value": pol.value,
                       "lp_value": pol.lp_value},
            "refine": {"centres": 8, "rounds": 3, "cloud": 4096, "ms_per_call_with_regeneration": ms_refine,
                       "value": ref_v, "evals": int(ref_evals)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="config4", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="time the named workload only (skip the short extra legs on the other "
                         "configurations and the memory-bound leg)")
    ap.add_argument("--memory-leg", action="store_true",
                    help="with --only: still run the memory-bound leg (the small-game sweep kernel over "
                         "2^26 rows read from a 2 GiB buffer)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run a plain 256 MiB device copy 5 times (a known-size reference "
                         "kernel for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--ceilings", action="store_true",
                    help="(the default unless --only is given) also measure what this box reaches on "
                         "plain kernels (stream read GB/s, bf16 and fp32 MFMA loop TFLOP/s, empty-launch "
                         "latency, MFMAs under the sweep kernel's own mix of matrix and vector "
                         "instructions) and report the fractions against them beside those against the "
                         "vendor peaks; a few seconds, outside every timed region")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured ceilings")
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
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[args.workload][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[args.workload][1]
    if args.copy_reference:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    r = run_workload(args.workload, steps, warmup, not args.no_cpu_baseline)
    game = r["game"]
    line = {
        "metric": "candidate-type evals/sec at 1 MI355X",
        "value": r["value"], "unit": "candidate-type evals/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if game.storage == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "description": r["note"], "m": game.m, "n": game.n,
                   "K": game.K, "candidates_per_step": r["count"], "candidates_per_launch": r["chunk"],
                   "path": r["path"], "timed_region_s": r["timed_region_s"],
                   "step": ("candidates generated inside the sweep kernel" if r["fused"] else
                            "per chunk: generate candidates into a buffer + sweep") +
                           " + merge into the running best; the K steps are consecutive ranges of one "
                           "streamed sweep, result to host after the last",
                   "ms_per_step_with_a_result_after_every_step": r["ms_per_step_each"],
                   "value_with_a_result_after_every_step":
                       r["count"] * game.K / (r["ms_per_step_each"] * 1e-3)},
        "roofline": r["roofline"],
        "cpu_baseline": r["cpu_baseline"],
        "result": {"best_index": r["best_index"], "best_value": r["best_value"],
                   "n_tie_evals": r["n_tie_evals"]},
    }
    if (args.ceilings or not args.only) and not args.no_ceilings:
        from paper_2605_18856_amd import bsse
        c = bsse.bsse_ceilings()
        line["measured_ceilings"] = c
        rf = line["roofline"]
        key = {"GB/s": "stream_read_GBs", "TFLOP/s": "mfma_bf16_TFLOPs" if rf["peak"] == 2500.0 else "mfma_f32_TFLOPs"}[rf["unit"]]
        rf["frac_of_measured_ceiling"] = rf["achieved"] / c[key]
        if args.workload in MIXES:
            # what the bf16 matrix cores keep under this kernel's mix of matrix and vector instructions
            # with nothing else in the way (no loads, dependencies or barriers)
            nm, nv = MIXES[args.workload]
            mix = bsse.bsse_mixed_ceiling(nm, nv) / EXECUTED_FLOP_FACTOR.get(r["path"], 1.0)
            c["mfma_bf16_TFLOPs_under_this_kernels_instruction_mix"] = mix
            c["instruction_mix"] = {"mfma_per_block": nm, "vector_per_block": nv}
            rf["frac_of_mixed_ceiling"] = rf["achieved"] / mix
    if not args.only:
        # short extra legs: the other configurations (not part of `value`), and the sweep
        # kernel alone on a batch far larger than the caches for the memory-bound game
        others = {}
        for w, (st, wu) in {"config1": (50, 5), "config2": (50, 5), "config3": (6, 2),
                            "config4": (2, 1), "config5": (1, 1)}.items():
            if w == args.workload:
                continue
            o = run_workload(w, st, wu, False)
            others[w] = {"value": o["value"], "ms_per_step": o["ms_per_step"], "path": o["path"],
                         "candidates_per_step": o["count"], "candidates_per_launch": o["chunk"],
                         "roofline": {k: o["roofline"][k] for k in
                                      ("bound", "achieved", "peak", "unit", "frac", "kernel_ms", "traffic")}}
            if w in MIXES and not args.no_ceilings:
                from paper_2605_18856_amd import bsse
                nm, nv = MIXES[w]
                mix = bsse.bsse_mixed_ceiling(nm, nv) / EXECUTED_FLOP_FACTOR.get(o["path"], 1.0)
                others[w]["roofline"]["mixed_ceiling"] = mix
                others[w]["roofline"]["instruction_mix"] = {"mfma_per_block": nm, "vector_per_block": nv}
                others[w]["roofline"]["frac_of_mixed_ceiling"] = o["roofline"]["achieved"] / mix
        line["other_workloads"] = others
        line["memory_bound_leg"] = hbm_leg()
        line["prior_batch"] = prior_batch_leg()
        line["refinement"] = refinement_leg()
    elif args.memory_leg:
        line["memory_bound_leg"] = hbm_leg()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
