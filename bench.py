#!/usr/bin/env python3
"""Benchmark of the MARS verification pass on one MI355X.

One step = one call of the whole hot path (row reduction, margin test, acceptance, residual
resampling, path and bonus-token selection) over one batch of synthetic input already resident in
HBM.  The default workload is the headline configuration: sampling verification at T = 0.7,
B = 16 requests, a 60-node draft tree each, V = 151 936, bf16 logits, dense fp32 draft
distribution, theta = 0.9 (960 rows, 291.7 MB of logits per step).  Four independently generated
input sets are rotated so that a step never finds its logits in the 256 MB memory-side cache.

``--workload`` selects what a step is:
  headline  mars_verify on the headline configuration (the default; the line the metric is quoted on)
  cfg0 / cfg1_greedy / cfg1_sampling / cfg3 / cfg4
            mars_verify on the other stated configurations: a greedy chain of 8 drafts over 32 000 entries
            (fp32); one 60-node tree over 151 936 entries at T = 0 and at T = 1 (one-hot draft); 64 greedy
            chains over 128 256 entries with a threshold per request; 256 trees of 26 nodes over 151 936
            fp32 entries at T = 1 (4 GB of logits, one input set: it exceeds every cache by itself)
  commit    the same through mars_verify_ex with the committed sequence and the kept cache rows
  sweep7    the same with seven thresholds per request (0.84 .. 0.96) from one read of the logits
  margin    mars_margin_stats on the same logits (top-2 statistics per row and their histograms)
  spd       mars_verify on chains of 6 drafts with a dense draft distribution, B = 128, T = 1
  lmhead    mars_lmhead_verify: greedy verification from the last hidden states (H = 4096) and the
            LM-head weight [151 936, 4096], the logits never written to memory; its roofline object
            is the matrix-core one (bf16 MFMA peak) of the fused kernel

``value`` is the throughput of the passes issued one after the other on ONE stream: what one caller of
the library sees.  Beside it the line carries the throughput with the steps issued round-robin on
``--streams`` HIP streams (default 2; 1 = not measured), each with its own workspace and outputs
(``config.overlapped_*``): the library keeps no state and calls with different workspaces may
overlap, so the latency-bound per-request kernel of one step runs beside the bandwidth-bound row
reduction of the next, as a server verifying two micro-batches would have it; and the latency of
single calls (``config.call_us_*``).

Prints ONE JSON line with the whole-job rows/s, two HBM roofline objects -- ``roofline``: the
dominant kernel (the row reduction, timed by itself with HIP events on the stream it runs on);
``roofline_pass``: the whole call, the bytes of the logits over the time of one call -- and the CPU
oracle timed on the host cores of the same machine.
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
N_BUFFERS = 4
PARTIAL_BYTES = 24     # one partial result per (row, split) written by the row reduction
SWEEP = (0.84, 0.86, 0.88, 0.90, 0.92, 0.94, 0.96)
MARGIN_RANGES = (-5.0, 35.0, 0.5, 1.0, 0.0, 1.0)
MARGIN_BINS = (40, 50, 50)

WORKLOADS = {
    "headline": dict(cfg=2, what="configs[2]: sampling T=0.7, B=16, 60-node tree per request, V=151936, "
                                 "bf16 logits, dense fp32 draft distribution, theta=0.9"),
    "commit": dict(cfg=2, what="configs[2] through mars_verify_ex, with the committed sequence and the kept cache rows"),
    "sweep7": dict(cfg=2, what="configs[2] through mars_verify_ex with 7 thresholds per request (0.84..0.96), "
                               "one read of the logits"),
    "margin": dict(cfg=2, what="mars_margin_stats on the logits of configs[2]: top-2 statistics per row, histograms "
                               "of z1, z2/z1, p2/p1 (40/50/50 cells)"),
    "spd": dict(cfg=5, what="chains of 6 drafts (N=7), B=128, V=151936, bf16 logits, dense fp32 draft distribution, "
                            "T=1, theta=0.9"),
    "cfg0": dict(cfg=0, streams=1, what="configs[0]: greedy, B=1, chain of 8 drafts (N=9), V=32000, fp32 logits, "
                                         "theta=0.9 (1.15 MB of logits: a latency, the inputs stay in cache)"),
    "cfg1_greedy": dict(cfg=1, temperature=0.0, streams=1,
                        what="configs[1] at T=0: B=1, a 60-node tree, V=151936, bf16 logits, theta=0.9"),
    "cfg1_sampling": dict(cfg=1, streams=1,
                          what="configs[1] at T=1.0 with a one-hot draft distribution: B=1, a 60-node tree, V=151936, "
                               "bf16 logits, theta=0.9"),
    "cfg3": dict(cfg=3, what="configs[3]: greedy, B=64, chains of 8 drafts (N=9), V=128256, bf16 logits, Gumbel(0,2) "
                             "background, a threshold per request from {0.85, 0.9, 0.95}"),
    "cfg4": dict(cfg=4, buffers=1, steps=40, warmup=4,
                 what="configs[4]: sampling T=1.0, B=256, a 26-node tree per request, V=151936, fp32 logits (4.05 GB, "
                      "one input set), one-hot draft distribution, theta=0.9"),
    "lmhead": dict(cfg=None, what="greedy verification from hidden states: B=16, 60-node tree per request, H=4096, "
                                  "V=151936, bf16 hidden states and LM-head weight, theta=0.9; logits formed, reduced "
                                  "and dropped inside one kernel"),
    "lmhead_sampling": dict(cfg=None, what="sampling verification (T=0.7, dense fp32 q) from hidden states: B=16, 60-node "
                            "tree per request, H=4096, V=151936; the logits are written once by the fused kernel"),
}


def _code_only(text: str) -> str:
    """C++ source with its comments taken out and runs of white space collapsed (string literals
    are left alone): what a counter capture is tied to is the code, not its commentary."""
    out, i, n = [], 0, len(text)
    while i < n:
        c = text[i]
        if c == '"' or c == "'":
            j = i + 1
            while j < n and text[j] != c:
                j += 2 if text[j] == "\\" else 1
            out.append(text[i:j + 1]); i = j + 1
        elif text.startswith("//", i):
            j = text.find("\n", i)
            i = n if j < 0 else j
        elif text.startswith("/*", i):
            j = text.find("*/", i + 2)
            out.append(" "); i = n if j < 0 else j + 2
        else:
            out.append(c); i += 1
    return " ".join("".join(out).split())


def kernel_source_digest(files=("common.h", "row_reduce.h")) -> str:
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2601_15498_amd", "csrc", f), "r", encoding="utf-8") as fh:
            h.update(_code_only(fh.read()).encode("utf-8"))
    return h.hexdigest()[:16]


def measured_traffic():
    """HBM bytes per launch of the row reduction from the committed rocprofv3 counter runs, or
    None when there are none or the kernel source has changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "row_reduce_headline_traffic.json")
    try:
        with open(path) as fh:
            t = json.load(fh)
    except (OSError, ValueError):
        return None
    if t.get("kernel_source_digest") != kernel_source_digest():
        return None
    return t.get("hbm_bytes_per_launch")


def measured_pass_traffic():
    """HBM bytes of a whole pass on the headline workload (row reduction + per-request kernel) from the
    same counter runs, or None when either kernel's source has changed since."""
    k1 = measured_traffic()
    if k1 is None:
        return None
    with open(os.path.join(ROOT, "profiles", "row_reduce_headline_traffic.json")) as fh:
        t = json.load(fh)
    if t.get("tail_source_digest") != kernel_source_digest(("common.h", "tail.h")) or "tail_hbm_bytes_per_launch" not in t:
        return None
    return k1 + t["tail_hbm_bytes_per_launch"]


def measured_lmhead_traffic():
    """Bytes the fused LM-head kernel moves between L2 and the memory side per launch on its benchmark
    workload, from the committed counter runs; None once the kernel source has changed since."""
    try:
        with open(os.path.join(ROOT, "profiles", "lmhead_reduce_traffic.json")) as fh:
            t = json.load(fh)
    except (OSError, ValueError):
        return None
    if t.get("kernel_source_digest") != kernel_source_digest(("common.h", "lmhead.h")):
        return None
    return t.get("hbm_bytes_per_launch")


def main_lmhead(args) -> int:
    """--workload lmhead: one step = one mars_lmhead_verify call (LM head + top-2 + Alg. 1)."""
    import numpy as np
    import torch

    from mars_inputs.lmhead import LMHEAD_CONFIGS, make_lmhead_workload
    from paper_2601_15498_amd import binding as M

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        return 2
    M.lib()
    dev = torch.device("cuda:0")
    spec = dict(LMHEAD_CONFIGS["headline"])
    name = spec.pop("name")
    sampling = args.workload == "lmhead_sampling"
    t_gen = time.perf_counter()
    if sampling:   # lattice inputs (exact fp32 sums), dense draft distribution
        w = make_lmhead_workload(name, seed=2, lattice=True, temperature=0.7, dense_q=True, **spec)
    else:
        w = make_lmhead_workload(name, seed=2, **spec)
    t_gen = time.perf_counter() - t_gen
    B, N, H, V = w.B, w.N, w.H, w.V
    rows = B * N
    d = dict(h=torch.from_numpy(w.hidden).to(dev), w=torch.from_numpy(w.weight).to(dev),
             tok=torch.from_numpy(w.draft_tokens).to(dev), par=torch.from_numpy(w.tree_parent).to(dev),
             th=torch.from_numpy(np.ascontiguousarray(w.theta, np.float32)).to(dev))
    out = M.VerifyOutputs(B, N, dev, want_diag=sampling)
    ws = torch.empty(M.mars_lmhead_workspace_bytes(B, N, V, H), dtype=torch.uint8, device=dev)
    if sampling:
        d["u"] = torch.from_numpy(w.uniforms).to(dev)
        d["q"] = torch.from_numpy(w.draft_probs).to(dev)
        logits_out = torch.empty((B, N, V), dtype=torch.uint16, device=dev)

    def step(stages=0):
        if sampling:
            M.mars_lmhead_verify_sampling(d["h"], d["w"], d["tok"], d["par"], d["th"], w.temperature, d["u"], d["q"],
                                          logits_out, out, ws, stages=stages)
        else:
            M.mars_lmhead_verify(d["h"], d["w"], d["tok"], d["par"], d["th"], out, ws, stages=stages)

    def timed(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    timed(args.warmup)
    elapsed = timed(args.steps)
    tau = float(out.accept_len.float().mean().item() + 1.0)
    statuses = int((out.request_status != 0).sum().item())
    # the fused LM-head kernel by itself: HIP events on the stream it is launched on
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(min(args.warmup, 10)):
        step(M.MARS_STAGE_ROWS)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step(M.MARS_STAGE_ROWS)
    e1.record()
    torch.cuda.synchronize()
    k_ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * rows * H * V
    achieved = flops / (k_ms * 1e-3) / 1e12
    # For context: the same product by the library GEMM, which also has to write the logits (an unfused
    # pipeline then still runs the row reduction and the per-request kernel over them).
    h2 = d["h"].view(torch.bfloat16).reshape(rows, H)
    w2 = d["w"].view(torch.bfloat16)
    for _ in range(3):
        torch.matmul(h2, w2.t())
    torch.cuda.synchronize()
    n_mm = max(4, min(args.steps, 30))
    e0.record()
    for _ in range(n_mm):
        torch.matmul(h2, w2.t())
    e1.record()
    torch.cuda.synchronize()
    gemm_us = e0.elapsed_time(e1) / n_mm * 1e3
    unfused_pass_us = None
    if sampling:   # what follows the library GEMM in an unfused pipeline: the pass over the stored logits
        out2 = M.VerifyOutputs(B, N, dev)
        ws2 = M.alloc_workspace(B, N, V)
        for _ in range(3):
            M.mars_verify(logits_out, d["tok"], d["par"], d["th"], w.temperature, d["u"], d["q"], out2, ws2)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n_mm):
            M.mars_verify(logits_out, d["tok"], d["par"], d["th"], w.temperature, d["u"], d["q"], out2, ws2)
        e1.record()
        torch.cuda.synchronize()
        unfused_pass_us = e0.elapsed_time(e1) / n_mm * 1e3
    result = {
        "metric": f"rows/s + achieved bf16 MFMA TFLOP/s vs peak, workload '{args.workload}'",
        "value": rows * args.steps / elapsed, "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload]["what"], "B": B, "N": N, "H": H, "V": V, "rows_per_step": rows,
                   "streams": 1, "mean_tau": tau, "requests_with_nonzero_status": statuses,
                   "weight_bytes": V * H * 2, "weight_stream_GBps": V * H * 2 / (k_ms * 1e-3) / 1e9,
                   "library_gemm_us": gemm_us, "unfused_pass_behind_the_gemm_us": unfused_pass_us,
                   "logits_bytes_written": rows * V * 2 if sampling else 0,
                   "input_generation_s": round(t_gen, 1)},
        "roofline": {"bound": "mfma", "kernel": "lmhead_reduce_kernel<192, %s>" % ("sampling" if sampling else "greedy"), "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None if sampling else measured_lmhead_traffic(), "algorithmic_flops_per_launch": flops,
                     "algorithmic_bytes_per_launch": V * H * 2 + rows * H * 2 + (rows * V * 2 if sampling else 0),
                     "avg_launch_us": k_ms * 1e3},
    }
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info

        from oracle import lmhead_ref
        sample = 2  # requests
        reps, cpu_s = 0, 0.0
        while reps < 2 or (cpu_s < 10.0 and reps < 20):
            t = time.perf_counter()
            if sampling:
                lmhead_ref.lmhead_verify_sampling(w.hidden[:sample], w.weight, w.draft_tokens[:sample],
                                                  w.tree_parent[:sample], w.theta[:sample], w.temperature,
                                                  w.uniforms[:sample], w.draft_probs[:sample])
            else:
                lmhead_ref.lmhead_verify(w.hidden[:sample], w.weight, w.draft_tokens[:sample], w.tree_parent[:sample],
                                         w.theta[:sample])
            cpu_s += time.perf_counter() - t
            reps += 1
        threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
        result["cpu_baseline"] = {"value": sample * N * reps / cpu_s, "unit": "rows/s", "cores": threads, "kind": "oracle",
                                  "sample": f"the first {sample} requests ({sample * N} rows against the whole weight), "
                                            f"{reps} passes, {cpu_s:.1f} s wall; fp64 matrix product by the BLAS numpy "
                                            "links, then the C oracle"}
    print(json.dumps(result), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 400; 40 for cfg4)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 40; 4 for cfg4)")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="headline")
    ap.add_argument("--streams", type=int, default=None,
                    help="HIP streams of the additional overlapped measurement (default: 2; 1 = none, also the default "
                         "for the single-request workloads, whose figure is a latency)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--row-scan", action="store_true",
                    help="the row reduction alone on 768, 960, 1536 and 2304 rows of the headline shape (random "
                         "bf16 logits), both forms: what a launch costs beyond its bytes, and the rate a further "
                         "768 rows are read at")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for hardware-counter runs: a few launches of the row reduction on the headline "
                         "workload and of a plain device copy of the same size (the calibration kernel)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU only: the verification pass is per request and needs no "
              "exchange between GPUs; run it with --gpus 1", file=sys.stderr)
        return 2

    if args.steps is None:
        args.steps = WORKLOADS[args.workload].get("steps", 400)
    if args.warmup is None:
        args.warmup = WORKLOADS[args.workload].get("warmup", 40)
    if args.workload in ("lmhead", "lmhead_sampling"):
        return main_lmhead(args)

    import numpy as np
    import torch

    from mars_inputs import CONFIGS, make_workload
    from paper_2601_15498_amd import binding as M

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        return 2
    M.lib()
    dev = torch.device("cuda:0")
    wl = args.workload
    spec = dict(CONFIGS[WORKLOADS[wl]["cfg"]])
    name = spec.pop("name")
    B, N, V = spec["B"], spec["N"], spec["V"]
    rows = B * N
    elt = 2 if spec["dtype"] == "bf16" else 4
    if "temperature" in WORKLOADS[wl]:
        spec["temperature"] = WORKLOADS[wl]["temperature"]
    T = spec["temperature"]
    K = len(SWEEP) if wl == "sweep7" else 1
    if wl == "sweep7":
        spec["sweep_thetas"] = SWEEP

    n_buffers = WORKLOADS[wl].get("buffers", N_BUFFERS)
    t_gen = time.perf_counter()
    sets, host0 = [], None
    for k in range(n_buffers):
        w = make_workload(f"{name}_set{k}", seed=2 + 100 * k, **spec)
        if k == 0:
            host0 = w
        theta = np.tile(np.asarray(SWEEP, np.float32)[:, None], (1, B)) if wl == "sweep7" else w.theta
        sets.append(dict(
            logits=torch.from_numpy(w.logits).to(dev),
            tok=torch.from_numpy(w.draft_tokens).to(dev),
            par=torch.from_numpy(w.tree_parent).to(dev),
            theta=torch.from_numpy(np.ascontiguousarray(theta)).to(dev),
            u=None if w.uniforms is None else torch.from_numpy(w.uniforms).to(dev),        # greedy: none drawn
            q=None if w.draft_probs is None else torch.from_numpy(w.draft_probs).to(dev)))  # None: one-hot
    t_gen = time.perf_counter() - t_gen

    n_streams = max(1, args.streams if args.streams is not None else WORKLOADS[wl].get("streams", 2))
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    wss = [M.alloc_workspace(B, N, V, dev, n_theta=K) for _ in range(n_streams)]
    outs = [M.VerifyOutputs(B, N, dev, n_theta=K, want_commit=(wl == "commit")) for _ in range(n_streams)]
    margin_rows = [torch.empty((rows, M.MARGIN_ROW_WORDS), dtype=torch.float32, device=dev) for _ in range(n_streams)]
    margin_counts = [torch.empty((M.margin_counts_len(MARGIN_BINS),), dtype=torch.int32, device=dev)
                     for _ in range(n_streams)]
    ws, out = wss[0], outs[0]
    k1_temperature = 0.0 if wl == "margin" else T  # the statistics need the top-2 only: no sum-exp in that pass

    def step(i, j=0):
        """One pass over input set i with the workspace and outputs of slot j, on the current stream."""
        s = sets[i % n_buffers]
        if wl in ("headline", "spd") or wl.startswith("cfg"):
            M.mars_verify(s["logits"], s["tok"], s["par"], s["theta"], T, s["u"], s["q"], outs[j], wss[j])
        elif wl == "margin":
            M.mars_margin_stats(s["logits"], s["theta"], T, MARGIN_RANGES, MARGIN_BINS, margin_rows[j],
                                margin_counts[j], wss[j])
        else:
            M.mars_verify_ex(s["logits"], s["tok"], s["par"], s["theta"], T, s["u"], s["q"], outs[j], wss[j], n_theta=K)

    if args.row_scan:
        # A launch = a part that does not shrink with the input + bytes at the marginal rate: both come out of
        # launches on 1x, 2x and 3x the 768 rows the chip holds three work-groups per compute unit of.
        del sets
        res = []
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for form, temp in (("sampling", 0.7), ("greedy", 0.0)):
            for n in (48, 60, 96, 144):
                torch.manual_seed(n)
                bufs = [(torch.randn(16, n, V, device=dev) * 3).to(torch.bfloat16) for _ in range(4)]
                w = M.alloc_workspace(16, n, V, dev)
                for z in bufs:
                    M.mars_row_reduce(z, temp, w)
                torch.cuda.synchronize()
                ts = []
                for _ in range(5):
                    ev0.record()
                    for i in range(40):
                        M.mars_row_reduce(bufs[i % 4], temp, w)
                    ev1.record()
                    torch.cuda.synchronize()
                    ts.append(ev0.elapsed_time(ev1) / 40 * 1e3)
                res.append({"form": form, "rows": 16 * n, "bytes": 16 * n * V * 2, "us_min": round(min(ts), 2),
                            "us_median": round(sorted(ts)[2], 2)})
                del bufs, w
        for form in ("sampling", "greedy"):
            r = {x["rows"]: x for x in res if x["form"] == form}
            step_us = (r[2304]["us_min"] - r[768]["us_min"]) / 2
            res.append({"form": form, "us_per_further_768_rows": round(step_us, 2),
                        "marginal_GBps": round(768 * V * 2 / step_us / 1e3, 1),
                        "us_of_a_768_row_launch_beyond_that_rate": round(r[768]["us_min"] - step_us, 2)})
        print(json.dumps({"row_scan": res}), flush=True)
        return 0

    if args.pmc_probe:
        # Counter runs serialise kernels; keep the run short.  The copy moves exactly the bytes of one
        # logits tensor (read) and as many again (write): the known quantity the counters are scaled by.
        dst = torch.empty_like(sets[0]["logits"])
        for i in range(6):
            dst.copy_(sets[i % n_buffers]["logits"])
            M.mars_row_reduce(sets[i % n_buffers]["logits"], k1_temperature, ws)
        for i in range(6):  # and the whole pass, so that the per-request kernel is counted too
            step(i)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "logits_bytes": rows * V * elt, "launches_each": 6}), flush=True)
        return 0

    def timed(n_steps, n_str):
        """Wall time of n_steps passes issued round-robin over n_str streams (0: the current stream)."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if n_str == 1:  # (one context for the whole loop: entering one per step costs the host ~6 us)
            with torch.cuda.stream(streams[0]):
                for i in range(n_steps):
                    step(i, 0)
        else:
            for i in range(n_steps):
                if n_str == 0:
                    step(i)
                else:
                    with torch.cuda.stream(streams[i % n_str]):
                        step(i, i % n_str)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # The figure of the line: the passes one after the other on one stream.
    timed(args.warmup, 1)
    elapsed = timed(args.steps, 1)
    ms_per_step = elapsed / args.steps * 1e3
    value = rows * args.steps / elapsed
    tau = None if wl == "margin" else (out.accept_len.float().reshape(K, B).mean(dim=1) + 1.0).tolist()
    # Beside it: the same passes round-robin over several streams (calls overlap).
    overlapped = None
    if n_streams > 1:
        timed(min(args.warmup, 10), n_streams)
        overlapped = timed(args.steps, n_streams)
    statuses = 0 if wl == "margin" else int(sum((o.request_status != 0).sum().item() for o in outs))

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
        M.mars_row_reduce(sets[i % n_buffers]["logits"], k1_temperature, ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(args.steps):
        M.mars_row_reduce(sets[i % n_buffers]["logits"], k1_temperature, ws)
    e1.record()
    torch.cuda.synchronize()
    k1_ms = e0.elapsed_time(e1) / args.steps
    target = min(768, max(128, (rows * V) >> 16))                # the library's rule for the work-groups it aims for
    splits = max(1, min((target + rows - 1) // rows, V // 8192))  # 960 rows: one work-group per row
    algo_bytes = rows * V * elt + rows * splits * PARTIAL_BYTES
    achieved = algo_bytes / (k1_ms * 1e-3) / 1e9
    # What the memory system gives a plain kernel on the same tensors: a device copy (as many bytes written as read).
    dst = torch.empty_like(sets[0]["logits"])
    for i in range(3):
        dst.copy_(sets[i % n_buffers]["logits"])
    torch.cuda.synchronize()
    n_copy = max(4, min(args.steps, 50))
    e0.record()
    for i in range(n_copy):
        dst.copy_(sets[i % n_buffers]["logits"])
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 2.0 * rows * V * elt / (e0.elapsed_time(e1) / n_copy * 1e-3) / 1e9
    del dst
    traffic = measured_traffic() if wl in ("headline", "commit", "sweep7") else None
    pass_bytes = rows * V * elt  # the logits, read once; everything else a pass touches is noise next to them
    pass_gbps = pass_bytes / (ms_per_step * 1e-3) / 1e9

    metric = "verify rows/s + achieved HBM GB/s vs peak, B=16 tree-60 V=151936 bf16"
    if wl != "headline":
        metric = f"rows/s + achieved HBM GB/s vs peak, workload '{wl}'"
    k1_name = "row_reduce_kernel<%s, %d per load, %s>" % (spec["dtype"], 16 // elt,
                                                          "top-2 only" if k1_temperature == 0.0 else "sampling")
    result = {
        "metric": metric,
        "value": value,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",   # the arithmetic of the path (statistics and probabilities in fp32); storage: logits_dtype
        "data": "synthetic",
        "config": {"workload": WORKLOADS[wl]["what"],
                   "B": B, "N": N, "V": V, "rows_per_step": rows, "logits_dtype": spec["dtype"],
                   "temperature": T, "thresholds_per_request": K, "input_sets_rotated": n_buffers, "mean_tau": tau,
                   "streams": 1, "requests_with_nonzero_status": statuses,
                   "overlapped_streams": n_streams if overlapped else None,
                   "overlapped_ms_per_step": overlapped / args.steps * 1e3 if overlapped else None,
                   "overlapped_rows_per_s": rows * args.steps / overlapped if overlapped else None,
                   "pass_hbm_traffic_GBps": (measured_pass_traffic() / (ms_per_step * 1e-3) / 1e9
                                             if wl == "headline" and measured_pass_traffic() else None),
                   "call_us_p10": pct[10], "call_us_median": pct[50], "call_us_p90": pct[90],
                   "device_copy_GBps": copy_gbps,
                   "input_generation_s": round(t_gen, 1)},
        "roofline": {"bound": "hbm", "kernel": k1_name,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_stale": bool(traffic is None and wl in ("headline", "commit", "sweep7")),
                     "algorithmic_bytes_per_launch": algo_bytes, "avg_launch_us": k1_ms * 1e3},
        # the whole call against the same roofline: the logits are read once per pass, whatever else it does
        "roofline_pass": {"bound": "hbm", "what": "one call on one stream, all kernels", "achieved": pass_gbps,
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": pass_gbps / HBM_PEAK_GBS,
                          "algorithmic_bytes_per_call": pass_bytes, "ms_per_call": ms_per_step},
    }

    if not args.no_cpu_baseline:
        from oracle import mars_ref
        found = os.cpu_count() or 1
        cores = min(found, 16) if "OMP_NUM_THREADS" not in os.environ else int(os.environ["OMP_NUM_THREADS"])

        def oracle_pass():
            h = host0
            if wl == "margin":
                mars_ref.margin_stats(h.logits, h.theta, T, MARGIN_RANGES, MARGIN_BINS)
            elif wl == "sweep7":
                mars_ref.verify_sweep(h.logits, h.draft_tokens, h.tree_parent,
                                      np.tile(np.asarray(SWEEP, np.float32)[:, None], (1, B)), T, h.uniforms,
                                      h.draft_probs)
            else:
                o = mars_ref.verify(h.logits, h.draft_tokens, h.tree_parent, h.theta, T, h.uniforms, h.draft_probs)
                if wl == "commit":
                    mars_ref.commit(h.draft_tokens, o["accept_len"], o["path_idx"], o["bonus_token"])

        mars_ref.set_threads(cores)
        reps, cpu_s = 0, 0.0
        while reps < 3 or (cpu_s * cores < 10.0 and reps < 20):
            t = time.perf_counter()
            oracle_pass()
            cpu_s += time.perf_counter() - t
            reps += 1
        mars_ref.set_threads(1)
        t = time.perf_counter()
        oracle_pass()
        one_s = time.perf_counter() - t
        result["cpu_baseline"] = {"value": rows * reps / cpu_s, "unit": "rows/s", "cores": cores,
                                  "host_cores_found": found, "kind": "oracle",
                                  "sample": f"the whole workload ({rows} rows, input set 0), {reps} passes, "
                                            f"{cpu_s:.1f} s wall",
                                  "single_thread_value": rows / one_s}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
