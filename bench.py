#!/usr/bin/env python3
"""Benchmark of the APMSqueeze compressed-momentum step on one MI355X.

A "step" is one pass of the whole hot path (apms_compress -> apms_server_reduce -> apms_apply,
Algorithm 1 lines 6-11) over one batch of fresh synthetic gradients for all n simulated workers.
Inputs are generated in HBM before the timed region of each step; the timed region is bracketed by
HIP events on the stream the kernels are launched on.  In the deferred modes the timed region starts
with nothing pending and the closing apms_finalize (which completes the last step's error update and
momentum gather) is inside the timed total.

Prints ONE JSON line on stdout (progress goes to stderr):
  value      parameters per second of the whole job (d_pad * steps / timed seconds)
  roofline   HBM roofline of the dominant kernel (the worker-side compress kernel)
  cpu_baseline  the CPU oracle, as it stands, timed on a bounded sample of the same workload
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure

# HBM bytes per launch of the compress kernel measured with rocprofv3 PMC counters (FETCH_SIZE and
# WRITE_SIZE runs, each scaled by what the counter reads for a plain copy of known size); the summary
# with the commands is profiles/bench_bert-large-flat_hbm_traffic.txt.  Reported only for the workload
# and error mode it was measured on.
MEASURED_COMPRESS_TRAFFIC = {("bert-large-flat", "deferred"): 88.458e9, ("bert-large-flat", "deferred-errors"): 87.763e9}

METRIC = "compressed-momentum step params/sec & HBM GB/s (% of peak), BERT-Large d, 1 GPU"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def call_bytes(n, gather_deferred=False):
    """Bytes per parameter per step each CALL has to move (fp32 state resident in HBM: m_i, g_i, delta_i
    per worker; sign words 1 bit per element; scales negligible).

    Eager gather (the accounting the workload was specified with, 344.25 B at n = 16):
      apms_compress       16.125 n        read m, g, delta; write delta; write n/8 B of signs
      apms_server_reduce  8 + (n+1)/8     read n sign streams; read + write server error; write signs
      apms_apply          12.125 + 4 n    read signs, v, x; write x; write m to n slices
    Deferred gather (apms_compress carries out the previous step's gather and uses the decoded momentum
    instead of reading m back, 282.25 B at n = 16):
      apms_compress       16.25 n         read g, delta, n/8 B of server signs; write delta, m, n/8 B of signs
      apms_apply          12.125          read signs, v, x; write x
    """
    server = 8.0 + (n + 1) / 8.0
    if gather_deferred:
        return {"compress": 16.25 * n, "server_reduce": server, "apply": 12.125}
    return {"compress": 16.125 * n, "server_reduce": server, "apply": 12.125 + 4.0 * n}


def cpu_baseline(wl, run, g, sample_elems, steps):
    """Time the CPU oracle (single thread, as it stands) on the first `sample_elems` parameters of the
    workload: same state bits, copied from HBM, treated as one chunk."""
    import numpy as np
    import oracle
    S, n = sample_elems, wl.n
    st = oracle.State(S, n, S, run.x[:S].cpu().numpy(), run.m[:, :S].cpu().numpy(), run.v[:S].cpu().numpy())
    gs = np.ascontiguousarray(g[:, :S].cpu().numpy())
    st.step(gs, wl.beta, wl.lr, wl.eps)               # page in, untimed
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step(gs, wl.beta, wl.lr, wl.eps)
    dt = time.perf_counter() - t0
    return {
        "value": S * steps / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
        "sample": "first %d parameters x %d workers of %s as one chunk, %d steps, %.1f s" % (S, n, wl.name, steps, dt),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert-large-flat")
    ap.add_argument("--mode", choices=["deferred", "deferred-errors", "eager", "implicit"], default="deferred",
                    help="deferred: error buffers and the momentum gather are written one call later "
                         "(apms_set_deferral); eager: every buffer is final when its call's work ends; implicit: as "
                         "deferred, but m[n][d] is never written (departs from the benchmark's state model)")
    ap.add_argument("--compress-tiles", type=int, default=0)
    ap.add_argument("--server-tiles", type=int, default=0)
    ap.add_argument("--algo", choices=["momentum", "gradient", "topk"], default="momentum",
                    help="momentum: APMSqueeze with the 1-bit compressor (the benchmark); gradient: the APGSqueeze "
                         "variant of Section 5.3; topk: APMSqueeze with the top-k compressor of Section 5.1 (eager)")
    ap.add_argument("--topk-percent", type=float, default=1.0, help="kept fraction of every chunk, in percent")
    ap.add_argument("--grad-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="element type of the gradient input (f32 is the benchmark's configuration)")
    ap.add_argument("--occupancy-pad", default="", help="e.g. compress=65536,apply=0 (apms_set_occupancy_pad)")
    ap.add_argument("--chunk-elems", type=int, default=0,
                    help="chunk length (the unit that has its own scale and server) instead of the workload's own, "
                         "which is d_pad / n as in the paper; a labelled variant, e.g. 65536")
    ap.add_argument("--placement", choices=["tuned", "packed"], default="tuned",
                    help="tuned: the worker error and the gradient are the pair of several successively "
                         "allocated buffers that the worker kernel runs fastest on (the chip's HBM regions; "
                         "fp32 gradients, buffers of 4 GB and more); packed: as first allocated")
    ap.add_argument("--reuse-grad", action="store_true", help="do not redraw gradients between steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of n*d floats (a kernel of known HBM traffic, for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 23)
    ap.add_argument("--cpu-steps", type=int, default=8)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (n workers are simulated as n state slices in HBM); "
                 "--gpus N with N > 1 is not supported")

    import torch
    from paper_2008_11343_amd import binding as B
    from paper_2008_11343_amd import workloads as W
    from paper_2008_11343_amd.runner import DeviceRun

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    wl = {w.name: w for w in W.CONFIGS}[args.workload]
    if args.chunk_elems:
        import dataclasses
        wl = dataclasses.replace(wl, chunk=args.chunk_elems, name="%s-chunk%d" % (wl.name, args.chunk_elems))
    dev = "cuda:0"
    d, n, L = wl.d_pad, wl.n, wl.L
    log("workload %s: d_pad=%d n=%d chunk=%d (%d chunks), %s gradients, mode=%s" %
        (wl.name, d, n, L, wl.C, wl.grad, args.mode))
    deferral = {"deferred": B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER, "deferred-errors": B.APMS_DEFER_ERRORS,
                "eager": 0,
                "implicit": B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER | B.APMS_IMPLICIT_MOMENTUM}[args.mode]
    warm = None
    gdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.grad_dtype]
    # the run owns every buffer, the gradient input included, so that it can place them in HBM
    run = DeviceRun(d, n, L, dev, deferred=deferral, place=args.placement == "tuned",
                    grad_dtype=gdt)
    if run.placement:
        log("placement: pair %d of %s ms; worker-kernel occupancy pad %d of %s ms" % (
            run.placement["chosen_pair"], run.placement["worker_kernel_ms_by_pair"],
            run.placement["occupancy_pad_compress"], run.placement["worker_kernel_ms_by_occupancy_pad"]))
    if wl.warmup_steps:
        # full pipeline: Adam warm-up on the averaged gradients (Algorithm 1 line 2), then freeze v
        W.device_state_(wl, dict(x=run.x, m=run.m[0], v=run.v), warm_start=True)
    else:
        W.device_state_(wl, dict(x=run.x, m=run.m, v=run.v, werr=run.werr, serr=run.serr))
    if args.compress_tiles or args.server_tiles:
        B.apms_set_tiles_per_block(run.ctx, args.compress_tiles, args.server_tiles)
    kernel_ids = {"compress": B.APMS_KERNEL_COMPRESS, "server": B.APMS_KERNEL_SERVER,
                  "apply": B.APMS_KERNEL_APPLY, "finalize": B.APMS_KERNEL_FINALIZE, "warmup": B.APMS_KERNEL_WARMUP}
    for item in filter(None, args.occupancy_pad.split(",")):
        name, val = item.split("=")
        B.apms_set_occupancy_pad(run.ctx, kernel_ids[name], int(val))
    topk_K = max(1, int(L * args.topk_percent / 100.0))
    if args.algo == "topk":
        if deferral or args.grad_dtype != "f32":
            sys.exit("bench.py: --algo topk is eager and fp32 only (use --mode eager)")
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        run.idx, run.val = torch.zeros(n, wl.C, topk_K, **i32), torch.zeros(n, wl.C, topk_K, **f32)
        run.sidx, run.sval = torch.zeros(wl.C, topk_K, **i32), torch.zeros(wl.C, topk_K, **f32)
        B.apms_topk_reserve(run.ctx, topk_K)
    plan = B.apms_get_plan(run.ctx)
    g = run.g
    g32 = g if gdt == torch.float32 else torch.empty(n, d, dtype=torch.float32, device=dev)   # generation buffer
    gbytes = g.element_size()
    stream = torch.cuda.current_stream()

    def draw(step):
        W.device_grad_(wl, step, g32)
        if g is not g32:
            g.copy_(g32)                    # round to nearest even, untimed (input generation)

    def one_step(step, events=None):
        if step == 0 or not args.reuse_grad:
            draw(wl.warmup_steps + step)
        if events is not None:
            events[0].record(stream)
        if args.algo == "gradient":
            B.apms_compress_gradient(run.ctx, g, run._grad_format(g), run.werr, run.packed, run.scales)
        elif args.algo == "topk":
            B.apms_topk_compress(run.ctx, run.m, g, run.werr, run.idx, run.val, topk_K, wl.beta)
        else:
            run.compress(g, wl.beta)
        if events is not None:
            events[1].record(stream)
        if args.algo == "topk":
            B.apms_topk_server_reduce(run.ctx, run.idx, run.val, topk_K, run.serr, run.sidx, run.sval)
        else:
            run.server_reduce()
        if events is not None:
            events[2].record(stream)
        if args.algo == "topk":
            B.apms_topk_apply(run.ctx, run.sidx, run.sval, topk_K, run.v, run.x, run.m, wl.lr, wl.eps)
        elif args.algo == "gradient":
            B.apms_apply_gradient(run.ctx, run.spacked, run.sscales, run.v, run.x, run.m, wl.lr, wl.beta, wl.eps)
        else:
            run.apply(wl.lr, wl.eps)
        if events is not None:
            events[3].record(stream)

    if wl.warmup_steps:
        wev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * wl.warmup_steps)]
        for t in range(1, wl.warmup_steps + 1):
            draw(t - 1)
            wev[2 * t - 2].record(stream)
            run.warmup_step(g, 1e-3, wl.beta, wl.beta2, wl.eps, t)
            wev[2 * t - 1].record(stream)
        run.freeze()
        torch.cuda.synchronize()
        wms = sorted(wev[2 * i].elapsed_time(wev[2 * i + 1]) for i in range(wl.warmup_steps))
        warm = {"steps": wl.warmup_steps, "ms_per_step_median": wms[len(wms) // 2],
                "GBps": d * (gbytes * n + 24.0) / (wms[len(wms) // 2] * 1e-3) / 1e9}
        log("Adam warm-up: %d steps, median %.3f ms (%.0f GB/s), then freeze" % (warm["steps"], warm["ms_per_step_median"], warm["GBps"]))
    if args.calibration_copy:
        W.device_grad_(wl, 0, g32)
        run.werr.copy_(g32)
        run.werr.zero_()
        torch.cuda.synchronize()
        log("calibration copy done: %d bytes read, %d bytes written" % (4 * n * d, 4 * n * d))
    for s in range(args.warmup):
        one_step(s)
    run.finalize()          # the timed region starts from a state with nothing pending
    torch.cuda.synchronize()
    log("warm-up done (%d steps)" % args.warmup)

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    fin = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    for s in range(args.steps):
        one_step(args.warmup + s, ev[s])
    fin[0].record(stream)
    run.finalize()
    fin[1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0

    t_c = [e[0].elapsed_time(e[1]) for e in ev]
    t_s = [e[1].elapsed_time(e[2]) for e in ev]
    t_a = [e[2].elapsed_time(e[3]) for e in ev]
    t_fin = fin[0].elapsed_time(fin[1])
    total_ms = sum(t_c) + sum(t_s) + sum(t_a) + t_fin
    ms_per_step = total_ms / args.steps
    value = d * args.steps / (total_ms * 1e-3)
    ab = call_bytes(n, gather_deferred=bool(deferral & B.APMS_DEFER_GATHER))
    ab["compress"] -= (4 - gbytes) * n             # 16-bit gradients: 2n fewer bytes read
    if deferral & B.APMS_IMPLICIT_MOMENTUM:
        ab["compress"] -= 4.0 * n                  # m is not written
    if args.algo == "topk":
        # algorithmic: worker reads m, g, delta and writes delta and its K-entry lists (the selection's extra
        # read of u and its slots are implementation, not counted); server reads the n lists, reads and
        # writes its error, writes its list; gather writes dense m to n slices and takes the model step
        kf = topk_K / L
        ab["compress"] = (16.0 + 8.0 * kf) * n
        ab["server_reduce"] = 8.0 * kf * n + 8.0 + 8.0 * kf
        ab["apply"] = 4.0 * n + 12.0 + 8.0 * kf
    if args.algo == "gradient":
        # worker: read g, delta; write delta, n/8 signs.  apply: read + write m per worker, n/8 signs, v, x, x
        ab["compress"] = (8.0 + gbytes) * n + n / 8.0
        ab["apply"] = 8.125 * n + 12.0
    spec_bytes = sum(call_bytes(n).values())       # the workload's own accounting (eager gather)
    mean = lambda xs: sum(xs) / len(xs)
    median = lambda xs: sorted(xs)[len(xs) // 2] if len(xs) % 2 else 0.5 * sum(sorted(xs)[len(xs) // 2 - 1:len(xs) // 2 + 1])
    step_bytes = d * sum(ab.values())
    compress_ms = mean(t_c)
    achieved = d * ab["compress"] / (compress_ms * 1e-3) / 1e9
    log("ms/step %.3f (compress %.3f, server_reduce %.3f, apply %.3f, final finalize %.3f total); wall %.2f s" %
        (ms_per_step, compress_ms, mean(t_s), mean(t_a), t_fin, wall))

    out = {
        "metric": METRIC, "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": "%s: d_pad=%d n=%d chunk=%d" % (wl.name, d, n, L),
            "algo": args.algo, "topk_K_per_chunk": topk_K if args.algo == "topk" else None, "mode": args.mode, "grad_dtype": args.grad_dtype, "gradients": wl.grad + (", reused" if args.reuse_grad else ", fresh each step"),
            "worker_params_per_s": value * n,
            "bytes_per_param_step": sum(ab.values()),
            "step_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
            "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "bytes_per_param_step_eager_accounting": spec_bytes,
            "step_GBps_eager_accounting": d * spec_bytes / (ms_per_step * 1e-3) / 1e9,
            "ms": {"compress": compress_ms, "server_reduce": mean(t_s), "apply": mean(t_a),
                   "final_finalize_total": t_fin},
            "ms_per_step_median": median([a + b + c for a, b, c in zip(t_c, t_s, t_a)]),
            "GBps": {"compress": achieved,
                     "server_reduce": d * ab["server_reduce"] / (mean(t_s) * 1e-3) / 1e9,
                     "apply": d * ab["apply"] / (mean(t_a) * 1e-3) / 1e9},
            "plan": {k: plan[k] for k in ("compress_tiles_per_block", "compress_grid", "server_tiles_per_block",
                                          "server_grid", "apply_grid", "occupancy_pad")},
            "wall_s_including_input_generation": wall,
            "adam_warmup": warm,
            "placement": run.placement,
            "device": torch.cuda.get_device_name(0),
        },
        "roofline": {
            "kernel": ("apms_topk_compress (all passes of the worker selection)" if args.algo == "topk" else
                       "compress_kernel<momentum: %s, gradient: %s> (apms_compress%s)" % (
                           "none" if args.algo == "gradient" else
                           "pending gather" if deferral & B.APMS_DEFER_GATHER else "read m",
                           args.grad_dtype, "_gradient" if args.algo == "gradient" else "")),
            "bound": "hbm", "achieved": achieved,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_COMPRESS_TRAFFIC.get((wl.name, args.mode)) if (args.grad_dtype == "f32" and args.algo == "momentum") else None,
            "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/bench_bert-large-flat_hbm_traffic.txt",
            "bytes_per_launch": d * ab["compress"],
            "avg_launch_ms": compress_ms,
        },
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(wl, run, g32, min(args.cpu_sample, L), args.cpu_steps)
    run.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
