#!/usr/bin/env python3
"""Benchmark of the MARS verification pass on one MI355X.

One step = one call of ``mars_verify`` (the whole hot path: row reduction, margin test,
acceptance, residual resampling, path and bonus-token selection) over one batch of synthetic
input already resident in HBM.  The workload is the headline configuration: sampling
verification at T = 0.7, B = 16 requests, a 60-node draft tree each, V = 151 936, bf16
logits, dense fp32 draft distribution, theta = 0.9 (960 rows, 291.7 MB of logits per step).
Four independently generated input sets are rotated so that a step never finds its
logits in the 256 MB memory-side cache.

Prints ONE JSON line with the whole-job rows/s, the HBM roofline of the dominant kernel
(the row reduction, timed by itself with HIP events on the stream it runs on) and the CPU
oracle timed on the host cores of the same box.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
N_BUFFERS = 4
PARTIAL_BYTES = 24     # one partial result per (row, split, wave) written by the row reduction
WAVES_PER_GROUP = 8    # waves per work-group of the row reduction


def kernel_source_digest() -> str:
    h = hashlib.sha256()
    for f in ("common.h", "row_reduce.h"):
        with open(os.path.join(ROOT, "paper_2601_15498_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic():
    """HBM bytes per launch of the row reduction from the committed rocprofv3 counter runs, or
    None when there are none or the kernel source has changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "row_reduce_cfg2_traffic.json")
    try:
        with open(path) as fh:
            t = json.load(fh)
    except (OSError, ValueError):
        return None
    if t.get("kernel_source_digest") != kernel_source_digest():
        return None
    return t.get("hbm_bytes_per_launch")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for hardware-counter runs: a few launches of the row reduction on the headline "
                         "workload and of a plain device copy of the same size (the calibration kernel)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU only: the verification pass is per request and needs no "
              "exchange between GPUs; run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from mars_inputs import CONFIGS, make_workload
    from paper_2601_15498_amd import binding as M

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        return 2
    M.lib()
    dev = torch.device("cuda:0")
    spec = dict(CONFIGS[2])
    name = spec.pop("name")
    B, N, V = spec["B"], spec["N"], spec["V"]
    rows = B * N
    elt = 2 if spec["dtype"] == "bf16" else 4
    T = spec["temperature"]

    t_gen = time.perf_counter()
    sets, host0 = [], None
    for k in range(N_BUFFERS):
        w = make_workload(f"{name}_set{k}", seed=2 + 100 * k, **spec)
        if k == 0:
            host0 = w
        sets.append(dict(
            logits=torch.from_numpy(w.logits).to(dev),
            tok=torch.from_numpy(w.draft_tokens).to(dev),
            par=torch.from_numpy(w.tree_parent).to(dev),
            theta=torch.from_numpy(w.theta).to(dev),
            u=torch.from_numpy(w.uniforms).to(dev),
            q=torch.from_numpy(w.draft_probs).to(dev)))
    t_gen = time.perf_counter() - t_gen

    ws = M.alloc_workspace(B, N, V, dev)
    out = M.VerifyOutputs(B, N, dev)

    if args.pmc_probe:
        # Counter runs serialise kernels; keep the run short.  The copy moves exactly the bytes of one
        # logits tensor (read) and as many again (write): the known quantity the counters are scaled by.
        dst = torch.empty_like(sets[0]["logits"])
        for i in range(6):
            dst.copy_(sets[i % N_BUFFERS]["logits"])
            M.mars_row_reduce(sets[i % N_BUFFERS]["logits"], T, ws)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "logits_bytes": rows * V * elt, "launches_each": 6}), flush=True)
        return 0

    def step(i):
        s = sets[i % N_BUFFERS]
        M.mars_verify(s["logits"], s["tok"], s["par"], s["theta"], T, s["u"], s["q"], out, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = rows * args.steps / elapsed
    tau = float(out.accept_len.float().mean().item()) + 1.0

    # Spread of one call: HIP events around each of up to 200 further calls (no host sync between them).
    n_ev = min(args.steps, 200)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for i, (a, b) in enumerate(ev):
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    call_us = np.sort(np.array([a.elapsed_time(b) * 1e3 for a, b in ev]))
    pct = {q: float(call_us[min(n_ev - 1, int(q / 100.0 * n_ev))]) for q in (10, 50, 90)}

    # The dominant kernel by itself: HIP events on the stream the kernel is launched on.
    for i in range(min(args.warmup, 10)):
        M.mars_row_reduce(sets[i % N_BUFFERS]["logits"], T, ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(args.steps):
        M.mars_row_reduce(sets[i % N_BUFFERS]["logits"], T, ws)
    e1.record()
    torch.cuda.synchronize()
    k1_ms = e0.elapsed_time(e1) / args.steps
    splits = max(1, min((1024 + rows - 1) // rows, V // 8192))  # the library's rule: 2 for 960 rows
    algo_bytes = rows * V * elt + rows * splits * WAVES_PER_GROUP * PARTIAL_BYTES
    achieved = algo_bytes / (k1_ms * 1e-3) / 1e9

    result = {
        "metric": "verify rows/s + achieved HBM GB/s vs peak, B=16 tree-60 V=151936 bf16",
        "value": value,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[2]: sampling T=0.7, B=16, 60-node tree per request, V=151936, "
                               "bf16 logits, dense fp32 draft distribution, theta=0.9",
                   "B": B, "N": N, "V": V, "rows_per_step": rows, "logits_dtype": spec["dtype"],
                   "temperature": T, "input_sets_rotated": N_BUFFERS, "mean_tau": tau,
                   "whole_pass_logits_GBps": rows * V * elt / (ms_per_step * 1e-3) / 1e9,
                   "call_us_p10": pct[10], "call_us_median": pct[50], "call_us_p90": pct[90],
                   "input_generation_s": round(t_gen, 1)},
        "roofline": {"bound": "hbm", "kernel": "row_reduce_kernel<bf16, 8 per load, sampling>",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(),
                     "algorithmic_bytes_per_launch": algo_bytes, "avg_launch_us": k1_ms * 1e3},
    }

    if not args.no_cpu_baseline:
        from oracle import mars_ref
        cores = os.cpu_count() or 1
        cores = min(cores, 16) if "OMP_NUM_THREADS" not in os.environ else int(os.environ["OMP_NUM_THREADS"])
        mars_ref.set_threads(cores)
        reps, cpu_s = 0, 0.0
        while reps < 3 or (cpu_s * cores < 10.0 and reps < 20):
            t = time.perf_counter()
            mars_ref.verify(host0.logits, host0.draft_tokens, host0.tree_parent, host0.theta, T,
                            host0.uniforms, host0.draft_probs)
            cpu_s += time.perf_counter() - t
            reps += 1
        mars_ref.set_threads(1)
        t = time.perf_counter()
        mars_ref.verify(host0.logits, host0.draft_tokens, host0.tree_parent, host0.theta, T,
                        host0.uniforms, host0.draft_probs)
        one_s = time.perf_counter() - t
        result["cpu_baseline"] = {"value": rows * reps / cpu_s, "unit": "rows/s", "cores": cores, "kind": "oracle",
                                  "sample": f"the whole configs[2] workload (960 rows, input set 0), {reps} passes, "
                                            f"{cpu_s:.1f} s wall",
                                  "single_thread_value": rows / one_s}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
