#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: plan -> grouped GEMM -> replica sum.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]
                    (cfg1..cfg5, mlp{1,2}-{column,inner,outer,2d}, bc{512,256,128};
                     --dtype f32, --c-dtype bf16, --merge auto|always|never, --ld-multiple N)

One step = one pass of the whole path over one batch of synthetic input already
resident in HBM: ``dmm_plan`` on the descriptors (host slicing + grouping), then
``dmm_execute`` (work-table upload and the grouped-GEMM launches; when C is
replicated, the replica sum rides in the epilogue of replica 0's macro-tiles).
60 ms of the same steps untimed to bring the device out of its idle state
(SETTLE_MS below), W untimed warm-up steps, then exactly K timed steps between
two device synchronisations; one JSON line on stdout.

The line also carries
  roofline      the grouped-GEMM kernel against the dense bf16 (or fp32) MFMA
                peak: algorithmic FLOPs (2 m n k of the ops behind the launch) / its
                average duration, taken from HIP events the library records around
                the launch on the launch stream (DMM_TIMING) on every one of 24 more
                steps run right after the timed region (which carries no events).
                With a replicated C that is the first of the step's two launches (the
                plain kernel over the macro-tiles of replicas 1, 2, ...);
  roofline_fused_launch   the second launch (replica 0's macro-tiles, whose epilogue adds
                the other replicas' partial sums and stores the sum to every replica):
                its FLOPs against the MFMA peak and the bytes of the sum it also moves;
  per_config    (default workload only) the other configurations, a short run each:
                plan + execute rate, kernel rate and fraction of the MFMA peak of the
                configuration's element type, parity of a sample of rows (cfg1, cfg2, cfg3,
                cfg5 packed and with ld padded to 8, cfg4 with fp32 operands, and 8192^3 in
                128 x 128 tiles dealt block-cyclically, which runs the merged macro-tiles);
  separate_replica_sum   (replicated C) the same plan + execute steps with
                DMM_SEPARATE_REDUCE: one GEMM launch over all macro-tiles, then the
                replica-sum kernel; reported beside `value`, never as it, with
  roofline_gemm_separate   that one GEMM launch against the MFMA peak, and
  roofline_replica_sum   the replica-sum kernel against peak HBM bandwidth:
                (c + 1) * 4 bytes per C element / its average duration;
  cpu_baseline  the CPU oracle (fp64 triple loop, as it stands) timed on the
                host cores on a bounded sample of rows of the same product;
  context       (bf16 workloads) what the vendor library reaches on this very box
                for one dense M x K x N product of the same operands' distribution
                (torch.matmul, bf16 output) and for the same product of zeros.  The
                chip lowers its clock under matrix load, and by how much depends on
                the data, so the published peak is not reachable with random
                operands; these two numbers say how far it is on the day.  Also the
                rate of a register-only MFMA loop on every SIMD (the library's
                dmm_measure_mfma_rate), random and constant operands.  Context only:
                nothing of the product path runs through the vendor library.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
SETTLE_MS = 60.0     # untimed load in front of the warm-up steps: after an idle spell the device runs its first
                     # 25 ms or so of matrix work up to a third slower than it then settles to (measured per step:
                     # 0.92, 1.05, 1.19, 1.19, 1.12, 1.05 ... 0.90 ms at step 20, 0.87 from step 30 on, flat to step
                     # 600), so a handful of warm-up steps alone would leave that transient in the timed region


def settle(one_step, sync, min_ms=SETTLE_MS, min_steps=5):
    """Untimed steps until the device has been under load for `min_ms`; returns how many."""
    n = 0
    t0 = time.perf_counter()
    while n < min_steps or (time.perf_counter() - t0) * 1e3 < min_ms:
        one_step()
        n += 1
        if n % 8 == 0:
            sync()            # (so that wall time is device time: the steps are issued asynchronously)
    sync()
    return n


def parity_sample(prob, cfg, A, B, np, omatmul):
    """Rows of C from the last run against the oracle: the first and last row, one row out of
    every 256-row band (every macro-tile band) and a few random ones, all columns."""
    rng = np.random.default_rng(3)
    M = cfg["M"]
    rows = {0, M - 1} | {int(b + rng.integers(0, min(256, M - b))) for b in range(0, M, 256)}
    rows |= {int(r) for r in rng.integers(0, M, 6)}
    rows = np.array(sorted(rows))
    got = prob.C.gather_rows(rows, 0).astype(np.float64)
    ref = omatmul.matmul(A[rows], B, bf16=(cfg["dtype"] == "bf16"))
    return {"rows_checked": int(len(rows)), "rel_frobenius": float(np.linalg.norm(got - ref) / np.linalg.norm(ref)),
            "tolerance": 2e-3 if cfg["dtype"] == "bf16" else 1e-5}


def short_run(name, ld_multiple, np, torch, workloads, binding, DeviceProblem, omatmul, steps=12, kernel_steps=12, dtype=None):
    """One of the other configurations: `steps` plan + execute steps between two synchronisations,
    then `kernel_steps` more with events around the kernels, then the parity sample."""
    cfg = workloads.config(name)
    if dtype and dtype != cfg["dtype"]:
        cfg = dict(cfg, dtype=dtype, name=f"{cfg['name']}/{dtype}")
    A, B = workloads.make_operands(cfg)
    prob = DeviceProblem(cfg, A, B, ld_multiple=ld_multiple)
    stream = torch.cuda.current_stream().cuda_stream
    fl = workloads.flops(cfg)
    peak = PEAK_TFLOPS[cfg["dtype"]]

    def one(flags):
        plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], 0)
        plan.execute_marshalled(prob.dtype_code, prob.args, flags | prob.c_flags, stream)
        return plan
    inflight = []

    def run(n):                               # n steps, three in flight (destroy waits for the plan's own work)
        for _ in range(n):
            inflight.append(one(0))
            if len(inflight) > 3:
                inflight.pop(0).destroy()
    settle(lambda: run(1), torch.cuda.synchronize)
    run(5)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    while inflight:
        inflight.pop(0).destroy()
    g, r = [], []
    for _ in range(kernel_steps):
        p = one(binding.DMM_TIMING | binding.DMM_SEPARATE_REDUCE)   # one GEMM launch, then the replica-sum kernel
        gm, rm = p.elapsed_ms()
        ran_merged = p.ran_merged()
        p.destroy()
        g.append(gm)
        r.append(rm)
    res = {"workload": f"{cfg['name']}: M={cfg['M']} K={cfg['K']} N={cfg['N']} {cfg['dtype']}, {cfg['what']}",
           "ld_multiple": ld_multiple, "tasks": prob.plan.num_tasks(), "work_items": prob.plan.num_items(),
           "ran_merged": ran_merged, "steps": steps,
           "ms_per_step": round(ms, 4), "value": round(fl / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
           "pct_of_mfma_peak": round(100.0 * fl / (ms * 1e-3) / 1e12 / peak, 2),
           "gemm_kernel": {"launch": "all macro-tiles in one launch", "avg_ms": round(float(np.mean(g)), 4), "median_ms": round(float(np.median(g)), 4),
                           "best_ms": round(float(np.min(g)), 4), "launches_timed": len(g),
                           "achieved": round(fl / (float(np.mean(g)) * 1e-3) / 1e12, 2), "peak": peak, "unit": "TFLOP/s",
                           "frac": round(fl / (float(np.mean(g)) * 1e-3) / 1e12 / peak, 4)},
           "parity": parity_sample(prob, cfg, A, B, np, omatmul)}
    if cfg["C"]["replication"] > 1:
        res["replica_sum_kernel_avg_ms"] = round(float(np.mean(r)), 4)
    prob.close()
    del prob, A, B
    gc.collect()
    torch.cuda.empty_cache()
    return res


def reduce_large(np, torch, workloads, DeviceProblem, stream):
    """The replica sum alone at a size where neither launch overhead nor the last-level cache
    matter: 16 tiles of 4096 x 4096, four replicas: 4 x 1.07 GB read, 1.07 GB written."""
    Mr = Nr = 16384
    rcfg = dict(name="reduce-large", M=Mr, K=64, N=Nr, dtype="bf16", nranks=64,
                A=workloads.block_desc(Mr, 64, 4, 4, replication=4), B=workloads.block_desc(64, Nr, 4, 4, replication=4),
                C=workloads.block_desc(Mr, Nr, 4, 4, replication=4))
    rp = DeviceProblem(rcfg, c_fill=1.0)
    settle(lambda: rp.reduce(0, stream), torch.cuda.synchronize)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
    ev[0].record()
    for i in range(10):
        rp.reduce(0, stream)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ts = [ev[i].elapsed_time(ev[i + 1]) for i in range(10)]
    rbytes = 5 * 4.0 * Mr * Nr
    res = {"kernel": "reduce_replicas_kernel", "bound": "hbm",
           "workload": "c = 4, C 16384 x 16384 fp32 in 4x4 tiles, dmm_reduce_replicas alone",
           "achieved": round(rbytes / (float(np.mean(ts)) * 1e-3) / 1e9, 1),
           "peak": PEAK_HBM_GBS, "unit": "GB/s",
           "frac": round(rbytes / (float(np.mean(ts)) * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
           "avg_ms": round(float(np.mean(ts)), 4), "best_ms": round(min(ts), 4)}
    rp.close()
    del rp
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg4", help="cfg1..cfg5 (default: the 8192^3 2.5D configuration)")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default=None,
                    help="element type of A and B (default: the workload's own)")
    ap.add_argument("--c-dtype", choices=["f32", "bf16"], default="f32",
                    help="element type of the C tiles (bf16: DMM_C_BF16, only for a C with one replica)")
    ap.add_argument("--merge", choices=["auto", "always", "never"], default="auto",
                    help="merged macro-tiles: where they save a tenth of the macro-tiles (auto), wherever the plan "
                         "can have them (DMM_MERGE_ALWAYS), or not at all (DMM_NO_MERGE)")
    ap.add_argument("--ld-multiple", type=int, default=1, help="pad leading dimensions to this many elements")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of C the CPU oracle computes (0 = auto)")
    ap.add_argument("--no-context", action="store_true", help="skip the vendor-library GEMM timing")
    ap.add_argument("--reduce", choices=["fused", "separate"], default="fused",
                    help="replicated C: the replica sum in the GEMM's epilogue (the library's default) or, with "
                         "DMM_SEPARATE_REDUCE, in the kernel of its own, on every step of this run")
    ap.add_argument("--no-separate", action="store_true",
                    help="skip the extra steps with DMM_SEPARATE_REDUCE (one GEMM launch + the replica-sum kernel)")
    ap.add_argument("--no-reduce-large", action="store_true",
                    help="skip the stand-alone replica sum at c = 4 on 16384 x 16384 (5.4 GB moved)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of the other configurations (cfg1, cfg2, cfg3, cfg5 packed and padded)")
    ap.add_argument("--only-reduce-large", action="store_true",
                    help="run nothing but the stand-alone replica sum at c = 4 on 16384 x 16384 (for a kernel trace)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the one-GPU part of the method (all virtual ranks' tiles live on one "
              "MI355X); --gpus must be 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import workloads
    from paper_2510_08874_amd import DMM_TIMING, binding
    from paper_2510_08874_amd.tiles import DeviceProblem

    binding.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dprop = torch.cuda.get_device_properties(0)

    if args.only_reduce_large:
        print(json.dumps({"roofline_replica_sum_large":
                          reduce_large(np, torch, workloads, DeviceProblem, torch.cuda.current_stream().cuda_stream)}), flush=True)
        return 0

    cfg = workloads.config(args.workload)
    if args.dtype and args.dtype != cfg["dtype"]:
        cfg = dict(cfg, dtype=args.dtype, name=f"{cfg['name']}/{args.dtype}")
    if args.merge == "always":
        cfg = dict(cfg, merge_always=True)
    plan_flags = binding.DMM_MERGE_ALWAYS if args.merge == "always" else 0
    exec_flags = binding.DMM_NO_MERGE if args.merge == "never" else 0
    if args.reduce == "separate":
        exec_flags |= binding.DMM_SEPARATE_REDUCE
    A, B = workloads.make_operands(cfg)
    prob = DeviceProblem(cfg, A, B, ld_multiple=args.ld_multiple, c_dtype=args.c_dtype)
    stream = torch.cuda.current_stream().cuda_stream
    c_rep = cfg["C"]["replication"]

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    host_s = [0.0, 0.0]       # host seconds spent issuing (plan + execute), and waiting for finished steps
    DEPTH = 3                 # steps in flight: a plan is read back and destroyed three steps after its launch
    inflight = []
    gemm_ms, red_ms, launch_ms = [], [], []

    KERNEL_STEPS = 24         # steps after the timed region whose kernels are bracketed by HIP events (the
                              # events cost the stream about 20 us per step, so the timed steps carry none)

    def step(record, timed=True):
        h0 = time.perf_counter()
        plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], plan_flags)      # slicing + grouping (host)
        plan.execute_marshalled(prob.dtype_code, prob.args, (DMM_TIMING if timed else 0) | prob.c_flags | exec_flags,
                                stream)                                                  # upload + GEMM + replica sum
        h1 = time.perf_counter()
        inflight.append((plan, record))
        if len(inflight) > DEPTH:
            retire()
        host_s[0] += h1 - h0
        host_s[1] += time.perf_counter() - h1

    def retire():
        plan, record = inflight.pop(0)
        g, r = plan.elapsed_ms()          # waits for that step's events
        two = plan.gemm_launch_ms() if record else None
        plan.destroy()
        if record and g >= 0.0:
            gemm_ms.append(g)
            red_ms.append(r)
            if two[0][0] >= 0.0:
                launch_ms.append(two)

    # The interpreter's cyclic collector stays off inside the loop: one full collection takes tens of
    # milliseconds here (it walks torch's objects) and would show up as a GPU idle gap of that length.
    gc.collect()
    gc.disable()
    settle_steps = settle(lambda: step(False, timed=False), torch.cuda.synchronize)
    for _ in range(args.warmup):
        step(False)
    while inflight:
        retire()
    torch.cuda.synchronize()
    host_s[0] = host_s[1] = 0.0
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(False, timed=False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    while inflight:
        retire()
    # the same steps once more, each with events around its kernels: the roofline figures
    for i in range(KERNEL_STEPS):
        step(True, timed=True)
    while inflight:
        retire()
    torch.cuda.synchronize()

    # the same steps with the replica sum in a kernel of its own (DMM_SEPARATE_REDUCE), for the record
    # and for the roofline of that kernel: one GEMM launch over all macro-tiles, then the sum
    separate = None
    sep_gemm, sep_red = [], []
    if c_rep > 1 and not args.no_separate and args.reduce == "fused":
        def sstep(record):
            plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], plan_flags)
            plan.execute_marshalled(prob.dtype_code, prob.args, (DMM_TIMING if record else 0) | binding.DMM_SEPARATE_REDUCE | exec_flags,
                                    stream)
            inflight.append((plan, record))
            if len(inflight) > DEPTH:
                sretire()

        def sretire():
            p0, rec = inflight.pop(0)
            if rec:
                g, r = p0.elapsed_ms()
                sep_gemm.append(g)
                sep_red.append(r)
            p0.destroy()
        for _ in range(10):
            sstep(False)
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for _ in range(args.steps):
            sstep(False)
        torch.cuda.synchronize()
        tf1 = time.perf_counter()
        for _ in range(KERNEL_STEPS):
            sstep(True)
        while inflight:
            sretire()
        f_ms = (tf1 - tf0) * 1e3 / args.steps
        separate = {"flag": "DMM_SEPARATE_REDUCE", "ms_per_step": round(f_ms, 4),
                    "value": round(workloads.flops(cfg) / (f_ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
                    "note": "same final contents of every C replica, bit for bit; not the default, not `value`"}

    # the same step without re-planning (one plan, tables already resident), for the record
    torch.cuda.synchronize()
    te0 = time.perf_counter()
    for _ in range(args.steps):
        prob.plan.execute_marshalled(prob.dtype_code, prob.args, prob.c_flags | exec_flags, stream)
    exec_only_host_us = (time.perf_counter() - te0) * 1e6 / args.steps     # host time of the calls alone
    torch.cuda.synchronize()
    exec_only_ms = (time.perf_counter() - te0) * 1e3 / args.steps
    tables_reused = prob.plan.table_reused()
    gc.enable()

    # host-only cost of planning, for the record
    tp0 = time.perf_counter()
    for _ in range(20):
        binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], plan_flags).destroy()
    plan_us = (time.perf_counter() - tp0) / 20 * 1e6
    # ... and of writing out the op list, its grouped order and the per-group macro-tiles (a plan with
    # merged macro-tiles runs without them and leaves that to the first accessor call)
    tp0 = time.perf_counter()
    for _ in range(5):
        pl = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], plan_flags)
        pl.num_tasks()
        pl.destroy()
    list_us = (time.perf_counter() - tp0) / 5 * 1e6
    ran_merged = prob.plan.ran_merged()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    fl = workloads.flops(cfg)
    value = fl / (ms_per_step * 1e-3) / 1e12
    peak = PEAK_TFLOPS[cfg["dtype"]]

    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(cfg["name"], {})

    def mfma_line(kernel, flops, times, **more):
        avg, best = float(np.mean(times)), float(np.min(times))
        ach = flops / (avg * 1e-3) / 1e12
        return dict({"kernel": kernel, "bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(ach / peak, 4), "avg_ms": round(avg, 4), "median_ms": round(float(np.median(times)), 4),
                     "best_ms": round(best, 4), "launches_timed": len(times),
                     "best_frac": round(flops / (best * 1e-3) / 1e12 / peak, 4)}, **more)

    es_tag = "2" if cfg["dtype"] == "bf16" else "4"
    fused_launches = prob.plan.ran_fused()        # of the execute-only steps above: same flags as the timed steps
    sum_read = (c_rep - 1) * 4.0 * cfg["M"] * cfg["N"]      # what a fused epilogue reads on top of the plain one
    roof_fused = None
    if fused_launches == 2 and launch_ms:
        # the step's two launches, each against the MFMA peak with the FLOPs of the ops behind it
        f0, f1 = launch_ms[0][0][1], launch_ms[0][1][1]
        roof = mfma_line(f"grouped_gemm_kernel<{es_tag}, false>", f0, [t[0][0] for t in launch_ms],
                         launch="first of the step's two GEMM launches: the macro-tiles of replicas 1.. "
                                f"({f0 / fl:.3f} of the step's FLOPs)", traffic=traffic.get("gemm_bytes"))
        roof_fused = mfma_line(f"grouped_gemm_kernel<{es_tag}, true>", f1, [t[1][0] for t in launch_ms],
                               launch="second launch: replica 0's macro-tiles, whose epilogue adds the other replicas' "
                                      "partial sums", partial_sum_bytes_read=sum_read)
    elif fused_launches == 1:
        roof = mfma_line(f"grouped_gemm_kernel<{es_tag}, true>", fl, gemm_ms,
                         launch="the step's one launch: the macro-tiles of replicas 1.. first, then replica 0's, whose "
                                "epilogue adds the other replicas' partial sums (written by the same workgroup earlier "
                                "in the launch)", partial_sum_bytes_read=sum_read, traffic=traffic.get("gemm_fused_bytes"))
    else:
        roof = mfma_line("grouped_gemm_comp_kernel" if ran_merged else f"grouped_gemm_kernel<{es_tag}, false>", fl, gemm_ms,
                         traffic=traffic.get("gemm_bytes"))
    achieved = roof["achieved"]
    fused_ran = fused_launches > 0

    out = {
        "metric": "plan-execute TFLOP/s and % of MFMA peak per partitioning config (1 GPU)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: M={cfg['M']} K={cfg['K']} N={cfg['N']} {cfg['dtype']}, {cfg['what']}",
                   "virtual_ranks": cfg["nranks"], "tasks": prob.plan.num_tasks(), "groups": prob.plan.num_groups(),
                   "work_items": prob.plan.num_items(), "merged_work_items": prob.plan.num_merged_items(),
                   "ran_merged": ran_merged, "merge": args.merge, "ld_multiple": args.ld_multiple, "c_dtype": args.c_dtype,
                   "step": "dmm_plan + dmm_execute (grouped GEMM" + (" with the replica sum in its epilogue)" if fused_ran
                                                                   else " + replica sum)" if c_rep > 1 else ")"),
                   "kernel_event_steps_after_the_timed_region": KERNEL_STEPS,
                   "settle": f"{settle_steps} untimed steps ({SETTLE_MS:.0f} ms of load) in front of the warm-up steps", "plan_host_us": round(plan_us, 1),
                   "plan_with_op_list_host_us": round(list_us, 1),
                   "execute_only_ms_per_step": round(exec_only_ms, 4),
                   "execute_only_tflops": round(workloads.flops(cfg) / (exec_only_ms * 1e-3) / 1e12, 2),
                   "execute_only_host_us_per_call": round(exec_only_host_us, 1), "execute_only_tables_reused": tables_reused,
                   "host_issue_us_per_step": round(host_s[0] / args.steps * 1e6, 1),
                   "host_wait_us_per_step": round(host_s[1] / args.steps * 1e6, 1)},
        "pct_of_mfma_peak": round(100.0 * value / peak, 2),
        "device": {"name": dprop.name, "gcn_arch": getattr(dprop, "gcnArchName", ""), "compute_units": dprop.multi_processor_count,
                   "peak_used": f"{peak} TFLOP/s = published dense {cfg['dtype']} MFMA peak of MI355X "
                                "(256 CUs x 4 SIMDs x 1024 flop/cycle x 2.4 GHz for bf16)"},
        "roofline": roof,
    }
    if roof_fused:
        out["roofline_fused_launch"] = roof_fused
        out["gemm_both_launches"] = {"avg_ms": round(float(np.mean(gemm_ms)), 4),
                                     "frac_of_mfma_peak": round(fl / (float(np.mean(gemm_ms)) * 1e-3) / 1e12 / peak, 4)}
    if separate:
        out["separate_replica_sum"] = separate
        out["roofline_gemm_separate"] = mfma_line(f"grouped_gemm_kernel<{es_tag}, false>", fl, sep_gemm,
                                                  launch="all macro-tiles in one launch (DMM_SEPARATE_REDUCE)")
    red_times = sep_red if separate else [r for r in red_ms if r >= 0.0]
    if red_times:
        r_avg = float(np.mean(red_times))
        r_best = float(np.min(red_times))
        red_bytes = (c_rep + 1) * 4.0 * cfg["M"] * cfg["N"]
        out["roofline_replica_sum"] = {"kernel": "reduce_replicas_kernel", "bound": "hbm",
                                       "achieved": round(red_bytes / (r_avg * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                                       "unit": "GB/s", "frac": round(red_bytes / (r_avg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                       "avg_ms": round(r_avg, 4), "best_ms": round(r_best, 4), "launches_timed": len(red_times),
                                       "traffic": traffic.get("reduce_bytes")}

    # parity spot check on the output of the timed run, and the CPU baseline
    from oracle import matmul as omatmul
    out["parity"] = parity_sample(prob, cfg, A, B, np, omatmul)

    if not args.no_cpu_baseline:
        n_rows = args.cpu_rows or max(1, min(cfg["M"], int(3.0e12 / (2.0 * cfg["K"] * cfg["N"]))))
        sel = np.arange(n_rows)
        tc0 = time.perf_counter()
        omatmul.matmul(A[sel], B, bf16=(cfg["dtype"] == "bf16"))
        tc = time.perf_counter() - tc0
        out["cpu_baseline"] = {"value": round(2.0 * n_rows * cfg["K"] * cfg["N"] / tc / 1e12, 5), "unit": "TFLOP/s",
                               "cores": omatmul.num_threads(), "kind": "oracle",
                               "sample": f"fp64 i-k-j triple loop on the first {n_rows} of {cfg['M']} rows of C "
                                         f"(all {cfg['N']} columns, K={cfg['K']}), {tc:.1f} s",
                               "seconds": round(tc, 2)}
    prob.close()
    del prob
    gc.collect()
    torch.cuda.empty_cache()

    if args.workload == "cfg4" and not args.dtype and not args.no_per_config and args.ld_multiple == 1 \
            and args.c_dtype == "f32" and args.merge == "auto":
        per = {}
        for name, ldm in (("cfg1", 1), ("cfg2", 1), ("cfg3", 1), ("cfg5", 1), ("cfg5", 8)):
            per[name if ldm == 1 else f"{name}/ld{ldm}"] = short_run(name, ldm, np, torch, workloads, binding, DeviceProblem, omatmul)
        per["cfg4/f32"] = short_run("cfg4", 1, np, torch, workloads, binding, DeviceProblem, omatmul, dtype="f32")
        per["bc128"] = short_run("bc128", 1, np, torch, workloads, binding, DeviceProblem, omatmul)
        per["cfg4"] = {"see": "the top level of this line (value, roofline, parity)"}
        out["per_config"] = per

    if not args.no_reduce_large and c_rep > 1:
        out["roofline_replica_sum_large"] = reduce_large(np, torch, workloads, DeviceProblem, stream)

    if not args.no_context and cfg["dtype"] == "bf16":
        def vendor(kind):
            mk = torch.randn if kind == "normal" else torch.zeros
            a = mk(cfg["M"], cfg["K"], device="cuda", dtype=torch.bfloat16)
            b = mk(cfg["K"], cfg["N"], device="cuda", dtype=torch.bfloat16)
            c = a @ b
            settle(lambda: torch.matmul(a, b, out=c), torch.cuda.synchronize)      # (the same courtesy as above)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                c = a @ b
            e1.record()
            torch.cuda.synchronize()
            del a, b, c
            return round(fl / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e12, 1)
        # this library's own grouped GEMM on the same partitioning with all-zero operands: what its
        # schedule sustains when the data lets the clock stay up
        zp = DeviceProblem(cfg, np.zeros_like(A), np.zeros_like(B), ld_multiple=args.ld_multiple, c_dtype=args.c_dtype)
        zt = []
        settle(lambda: zp.plan.execute_marshalled(zp.dtype_code, zp.args, binding.DMM_SEPARATE_REDUCE | zp.c_flags | exec_flags, stream),
               torch.cuda.synchronize)
        for i in range(30):
            zp.plan.execute_marshalled(zp.dtype_code, zp.args, DMM_TIMING | binding.DMM_SEPARATE_REDUCE | zp.c_flags | exec_flags, stream)
            zt.append(zp.plan.elapsed_ms()[0])
        zp.close()
        del zp
        torch.cuda.empty_cache()
        pipe_rand = binding.dmm_measure_mfma_rate(100.0, True)
        pipe_const = binding.dmm_measure_mfma_rate(100.0, False)
        out["context"] = {"grouped_gemm_zero_data_tflops": round(fl / (float(np.mean(zt)) * 1e-3) / 1e12, 1),
                          "vendor_matmul_bf16_out_normal_data_tflops": vendor("normal"),
                          "vendor_matmul_bf16_out_zero_data_tflops": vendor("zeros"),
                          "mfma_pipe_only_random_operands": {"tflops": round(pipe_rand[0], 1), "shader_mhz": round(pipe_rand[1])},
                          "mfma_pipe_only_constant_operands": {"tflops": round(pipe_const[0], 1), "shader_mhz": round(pipe_const[1])},
                          "gemm_frac_of_pipe_only_random": round(achieved / pipe_rand[0], 4),
                          "note": "zero data: this library's grouped GEMM on the same plan with all-zero operands; "
                                  "vendor: one dense product of the same M, K, N through torch.matmul on this box (not part "
                                  "of the path); pipe only: 100 ms of back-to-back bf16 MFMAs from registers on every SIMD "
                                  "(dmm_measure_mfma_rate): what the matrix pipes sustain at the clock the part settles to"}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
