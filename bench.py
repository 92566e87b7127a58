#!/usr/bin/env python3
"""Benchmark of the Finch selection path (score + top-r + compact over the whole
chunk loop) on one MI355X.

One bench "step" = one full pass of the hot path over one batch: every chunk step
of every problem of the workload (C4 by default: 256 problems x 32 chunk steps,
131072 document tokens).  Inputs are synthetic and already resident in HBM when
the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4]
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

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
COPY_CALIBRATION_BYTES = 1 << 30

# HBM bytes per launch from hardware counters (two rocprofv3 --pmc runs of this
# program on C4 with default options, FETCH_SIZE then WRITE_SIZE, each scaled by what
# the same counter reads for the 1 GiB elementwise copy of --copy-calibration).
# Offline figures (bench.py cannot read counters itself), reported only for a run with
# the options they were taken with, together with the summary they come from.
TRAFFIC_SOURCE = {"owner": "profiles/owner_loop_bf16_C4_hbm_traffic.txt",
                  "rowstats": "profiles/stage_kernels_bf16_C4_hbm_traffic.txt",
                  "colsum": "profiles/stage_kernels_bf16_C4_hbm_traffic.txt",
                  "select": "profiles/stage_kernels_bf16_C4_hbm_traffic.txt",
                  "gather": "profiles/stage_kernels_bf16_C4_hbm_traffic.txt"}
MEASURED_TRAFFIC = {"C4": {
    "rowstats": 2.0 * 159749.1 * 1024 + 1792.0 * 1024,
    "colsum": 2.0 * 159516.2 * 1024 + 4780.0 * 1024,
    "select": 2.0 * 2557.3 * 1024 + 728.0 * 1024,
    "gather": 2.0 * 47163.0 * 1024 + 92928.0 * 1024,
    "owner": 2.0 * 11133278.1 * 1024 + 3149952.0 * 1024,   # one launch = the whole loop
}}


def algorithmic_bytes(w, loop):
    """Bytes the method must move, per kernel class and in total, summed over one
    full chunk loop: every candidate key read once for scoring, Q once per step,
    every kept K and V row read once and written once."""
    e, d = w.elem_bytes, w.head_dim
    per = dict(score_pass=0, select=0, gather=0)
    keys = 0
    for i in range(loop.n_steps):
        for p, (c, m, r) in zip(loop.active[i], loop.step_shapes[i]):
            R = w.group * loop.problems[p]["n_que"]
            N = c + m
            keys += N
            per["score_pass"] += N * d * e + R * d * e
            per["select"] += 4 * N + 4 * min(r, N)
            per["gather"] += min(r, N) * d * e * 4
    total = per["score_pass"] + per["gather"]
    return per, total, keys


def logit_flops(w, loop):
    """Multiply-adds x 2 of the logits the method forms: every (prompt row, candidate key)
    pair once per scoring pass, two passes (document rows, when they are on, not counted)."""
    flops = 0
    for i in range(loop.n_steps):
        for p, (c, m, r) in zip(loop.active[i], loop.step_shapes[i]):
            R = w.group * loop.problems[p]["n_que"]
            flops += 2 * 2 * (c + m) * R * w.head_dim
    return flops


def cpu_baseline(w, next_problem, chunk, budget_s=10.0, seed=12345):
    """The oracle, as it stands, on the host cores, in two legs: BLAS free to use every
    core, then pinned to one thread.  Each leg runs whole chunk loops of problems drawn
    from a seeded shuffle of the workload's problems until about `budget_s` seconds of
    oracle time have been spent, and is extrapolated linearly to the whole job."""
    import random

    from oracle import finch_oracle as O
    host_cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    blas_threads = None
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([int(x.get("num_threads", 1)) for x in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
    order = list(range(w.n_problems))
    random.Random(seed).shuffle(order)
    n_tokens = sum(r.n_cont for r in w.requests)

    def leg(first):
        done, dt = 0, 0.0
        while dt < budget_s and done < len(order):
            pb = next_problem(order[(first + done) % len(order)])
            if pb is None:
                break
            t0 = time.perf_counter()
            O.compress(pb["Q"], pb["K"], pb["V"], chunk, pb["budget"])
            dt += time.perf_counter() - t0
            done += 1
        return done, dt

    done_all, dt_all = leg(0)
    out = dict(value=n_tokens / (dt_all / done_all * w.n_problems), unit="document tokens/s", cores=host_cores,
               blas_threads=blas_threads, kind="oracle")
    sample = (f"all cores: {done_all} of {w.n_problems} problems of {w.name} (seeded shuffle, seed {seed}), full "
              f"chunk loop each, {dt_all:.1f} s of oracle time, extrapolated linearly to all problems")
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            done_1, dt_1 = leg(done_all)
        if done_1:
            out["single_thread_value"] = n_tokens / (dt_1 / done_1 * w.n_problems)
            sample += f"; one thread: the next {done_1} problems of the same shuffle (wrapping round), {dt_1:.1f} s"
    else:
        sample += "; one-thread leg skipped (threadpoolctl not importable: BLAS threads cannot be pinned)"
    out["sample"] = sample
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    # (the first launches after the inputs have been drawn run 5-20 % longer than the steady state)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--path", default="auto", choices=["auto", "separate", "owner"],
                    help="launch path of the library (auto: its own choice)")
    ap.add_argument("--per-step", action="store_true",
                    help="one finch_step call per chunk instead of one finch_loop call")
    ap.add_argument("--reposition", default="off", choices=["off", "half", "interleaved"],
                    help="rotate kept keys to their new slots while compacting (rotary pairing)")
    ap.add_argument("--order", default="ascending", choices=["ascending", "rank"],
                    help="slots of the kept rows in the new cache")
    ap.add_argument("--layer-group", type=int, default=1,
                    help="L > 1: one selection per run of L problems (the KV heads of a layer)")
    ap.add_argument("--constant-budget", action="store_true",
                    help="keep the whole budget k from the first step on")
    ap.add_argument("--doc-rows", action="store_true",
                    help="scoring also takes the rows of each chunk's own tokens (causal mask); "
                         "about G*m more rows per problem, so use few --steps")
    ap.add_argument("--exact-denominator", action="store_true",
                    help="softmax denominators include the prompt's own keys (random ones here)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise copy of 1 GiB (read 1 GiB, write 1 GiB) three "
                         "times, so that a counter run of this command holds a kernel of known traffic")
    ap.add_argument("--phases", action="store_true",
                    help="load the measurement build with phase timers (python -m paper_2408_00167_amd.build "
                         "--phase-timers) and add the time per phase of a step of the one-workgroup-per-"
                         "problem kernels; the timed loop then runs the instrumented kernels")
    args = ap.parse_args()
    if args.phases:
        # (before the binding is imported: it reads the library's path once)
        os.environ["FINCH_LIBRARY"] = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                   "paper_2408_00167_amd", "libfinch_phases.so")
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (problems are independent; there is no "
              "multi-GPU path to measure). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2408_00167_amd as F
    import workloads as W
    from paper_2408_00167_amd.driver import ChunkLoop

    if not os.path.exists(F.LIB_PATH):
        from paper_2408_00167_amd.build import build_library
        build_library(verbose=False, phase_timers=args.phases)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = W.get_workload(args.workload)
    fin = F.Finch(F.FINCH_BF16 if w.dtype == "bf16" else F.FINCH_F32, w.head_dim, w.group, device=dev)
    fin.set_step_path({"auto": F.FINCH_PATH_AUTO, "separate": F.FINCH_PATH_SEPARATE,
                       "owner": F.FINCH_PATH_OWNER}[args.path])

    fin.set_reposition({"off": F.FINCH_ROPE_OFF, "half": F.FINCH_ROPE_HALF,
                        "interleaved": F.FINCH_ROPE_INTERLEAVED}[args.reposition],
                       {"ascending": F.FINCH_ORDER_ASCENDING, "rank": F.FINCH_ORDER_RANK}[args.order], 500000.0)

    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, args.layer_group)

    t_gen = time.perf_counter()
    probs = []
    for b, l, g in W.problems_of(w):
        p = W.make_problem(w, b, l, g, device=dev)
        probs.append(dict(Q=p["Q"], K=p["K"], V=p["V"], n_que=w.requests[b].n_que,
                          budget=w.requests[b].budget))
        if args.doc_rows:
            probs[-1]["Q_doc"] = torch.randn(w.group, w.chunk, w.head_dim, device=dev).to(p["K"].dtype)
        if args.exact_denominator:
            probs[-1]["K_que"] = torch.randn(w.requests[b].n_que, w.head_dim, device=dev).to(p["K"].dtype)
    loop = ChunkLoop(fin, probs, w.chunk, history=False, want_scores=False,
                     constant_budget=args.constant_budget)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    per_kernel_bytes, total_bytes, keys = algorithmic_bytes(w, loop)
    n_tokens = sum(r.n_cont for r in w.requests)

    for _ in range(args.warmup):
        loop.run(per_step=args.per_step)
    torch.cuda.synchronize()
    phase_fn = None
    if args.phases:
        import ctypes
        phase_fn = F.load_library().finch_debug_phases
        phase_fn.argtypes = [ctypes.POINTER(ctypes.c_ulonglong), ctypes.c_int]
        phase_fn.restype = ctypes.c_int
        phase_buf = (ctypes.c_ulonglong * 8)()
        assert phase_fn(phase_buf, 1) == 0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        loop.run(per_step=args.per_step)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = ev0.elapsed_time(ev1) / args.steps
    ms = wall_ms
    phases = None
    if phase_fn is not None:
        # thread 0 of each workgroup has added up its 10 ns ticks per phase over the timed loops
        assert phase_fn(phase_buf, 0) == 0
        names = ["stage_prompt_rows", "pass1_wave0", "pass1_barrier_wait", "merge_row_statistics", "pass2_wave0",
                 "pass2_barrier_wait", "top_r", "compaction"]
        per = args.steps * len(probs) * loop.n_steps
        phases = {n: phase_buf[i] * 0.01 / per for i, n in enumerate(names)}
        phases["sum"] = sum(phases.values())
        phases["unit"] = "us per chunk step, mean over workgroups"

    if args.copy_calibration:
        src = torch.ones(COPY_CALIBRATION_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # Per-kernel durations: the same loop again with HIP events around every launch
    # (on the launch stream).  Kept out of the pass that produced `value` because the
    # event records themselves lengthen the loop.
    roofline, kernels = None, None
    default_options = (args.reposition == "off" and args.order == "ascending" and args.layer_group == 1
                       and not args.constant_budget and not args.doc_rows and not args.exact_denominator)
    if not args.no_profile:
        F.finch_profile(fin.ctx, True)
        prof_steps = min(args.steps, max(1, 8192 // max(1, 5 * loop.n_steps)))
        # (creating the event pool leaves the GPU idle for a moment and the next launches
        # run long again: two passes that are recorded and thrown away)
        for _ in range(min(2, args.warmup)):
            loop.run(per_step=args.per_step)
        torch.cuda.synchronize()
        F.finch_profile_read(fin.ctx)
        torch.cuda.synchronize()
        tp = time.perf_counter()
        for _ in range(prof_steps):
            loop.run(per_step=args.per_step)
        torch.cuda.synchronize()
        prof_ms = (time.perf_counter() - tp) * 1e3 / prof_steps
        prof = F.finch_profile_read(fin.ctx)
        F.finch_profile(fin.ctx, False)
        kernels = {}
        for name, v in prof.items():
            if v["launches"]:
                kernels[name] = dict(avg_us=1e3 * v["ms"] / v["launches"], launches_per_step=v["launches"] // prof_steps,
                                     ms_per_step=v["ms"] / prof_steps)
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        per_kernel_bytes["prompt_lse"] = 0
        klass = {"prompt_lse": "prompt_lse","rowstats": "score_pass", "colsum": "score_pass", "owner": "step",
                 "select": "select", "gather": "gather", "lse": "select"}[dom]
        launches = kernels[dom]["launches_per_step"]
        # a launch that runs all stages: everything the method has to move (keys once)
        per_kernel_bytes["step"] = total_bytes
        bytes_per_launch = per_kernel_bytes[klass] / launches
        achieved = bytes_per_launch / (kernels[dom]["avg_us"] * 1e-6) / 1e9
        roofline = dict(bound="hbm", kernel=dom, achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s",
                        frac=achieved / HBM_PEAK_GBPS,
                        traffic=MEASURED_TRAFFIC.get(w.name, {}).get(dom) if default_options else None,
                        traffic_source=TRAFFIC_SOURCE.get(dom) if default_options and w.name in MEASURED_TRAFFIC else None,
                        bytes_per_launch=bytes_per_launch, avg_launch_us=kernels[dom]["avg_us"],
                        launches_per_step=launches, profiled_ms_per_step=prof_ms,
                        note="priced against HBM as the path's contract asks; counters and microbenchmarks "
                             "(profiles/) show the scoring passes bound by vector/matrix instruction issue, "
                             "not by memory")

    # what the arithmetic side of the same launches amounts to (bf16 runs; information
    # beside the contract's HBM figure: the scoring passes are not bound by memory)
    matrix_pipe = None
    if w.dtype == "bf16" and not args.doc_rows:
        fl = logit_flops(w, loop)
        matrix_pipe = dict(logit_flops=fl, achieved_TFLOPs=fl / (ms * 1e-3) / 1e12, peak_TFLOPs=MFMA_BF16_PEAK_TFLOPS,
                           frac=fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS)
    path_gbps = total_bytes / (ms * 1e-3) / 1e9
    out = {
        "metric": "document tokens compressed/sec (score+topk+compact); achieved HBM GB/s",
        "value": n_tokens / (ms * 1e-3),
        "unit": "document tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "event_ms_per_step": ev_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}", "problems": w.n_problems,
                   "document_tokens": n_tokens, "chunk": w.chunk, "chunk_steps": loop.n_steps,
                   "head_dim": w.head_dim, "group": w.group,
                   "path": args.path, "calls": "finch_step per chunk" if args.per_step else "finch_loop",
                   "reposition": args.reposition, "order": args.order,
                   "exact_denominator": args.exact_denominator, "doc_rows": args.doc_rows,
                   "layer_group": args.layer_group,
                   "constant_budget": args.constant_budget,
                   "prompt_rows": [w.rows(r) for r in w.requests][:4],
                   "budget": [r.budget for r in w.requests][:4], "keys_scored": keys},
        "path": {"algorithmic_bytes": total_bytes, "achieved_GBps": path_gbps,
                 "frac_of_hbm_peak": path_gbps / HBM_PEAK_GBPS},
        "kernels": kernels,
        "roofline": roofline,
        "matrix_pipe": matrix_pipe,
        "setup_s": t_gen,
    }
    if phases is not None:
        out["phases"] = phases
    if not args.no_cpu_baseline:
        order = list(W.problems_of(w))

        def next_problem(i):
            if i >= len(order):
                return None
            b, l, g = order[i]
            p = W.make_problem(w, b, l, g, device=dev)
            return dict(Q=W.to_numpy_storage(p["Q"]), K=W.to_numpy_storage(p["K"]),
                        V=W.to_numpy_storage(p["V"]), budget=w.requests[b].budget)

        out["cpu_baseline"] = cpu_baseline(w, next_problem, w.chunk)
    print(json.dumps(out), flush=True)
    fin.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
