#!/usr/bin/env python3
"""Benchmark of the APMSqueeze compressed-momentum step on one MI355X.

A "step" is one pass of the whole hot path (apms_compress -> apms_server_reduce -> apms_apply,
Algorithm 1 lines 6-11) over one batch of fresh synthetic gradients for all n simulated workers.
Inputs are generated in HBM before the timed region of each step; the timed region is bracketed by
HIP events on the stream the kernels are launched on.  In the deferred modes the timed region starts
with nothing pending and the closing apms_finalize (which completes the last step's error update and
momentum gather) is inside the timed total.

The headline workload is measured twice in one invocation (--placement both, the default): with every
buffer where the allocator first puts it ("packed": what a caller who just allocates gets) and with the
worker error and gradient buffers placed by timing ("tuned", see runner.DeviceRun).  `value`,
`ms_per_step` and `roofline` are the tuned run's; the packed run's figures are in `config.packed` and
`roofline.frac_packed`.

Prints ONE JSON line on stdout (progress goes to stderr):
  value      parameters per second of the whole job (d_pad * steps / timed seconds)
  roofline   HBM roofline of the dominant kernel (the worker-side compress kernel)
  cpu_baseline  the CPU oracle, as it stands, timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
CU_COUNT, CLOCK_GHZ, LANES_PER_CU = 256, 2.4, 64     # VALU issue: 4 SIMDs x 16 lanes per CU and cycle
# fp32 VALU operations per decoded worker element in the server kernel's inner loop (shift to the sign
# bit, bit-field insert of the sign into the scale, add); the rest of the kernel is per element, not per
# worker, and is left out, so this is a lower bound on the work
SERVER_VALU_OPS_PER_WORKER_ELEM = 3

METRIC = "compressed-momentum step params/sec & HBM GB/s (% of peak), BERT-Large d, 1 GPU"
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_bert-large-flat_hbm_traffic.txt")
KERNEL_SOURCES = ["kernels.hip", "apms_device.h", "apms_launch.h"]


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


def kernel_source_hash():
    """sha256 over the sources of the 1-bit kernels: a traffic measurement is quoted only for the code it was
    taken on."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2008_11343_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the tracked rocprofv3 PMC summary (FETCH_SIZE + WRITE_SIZE runs,
    each scaled by what the counter reads for a plain copy of known size), or (None, reason)."""
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None, "no traffic summary under profiles/"
    sha = re.search(r"^kernel_sources_sha256 (\w+)$", text, re.M)
    if not sha or sha.group(1) != kernel_source_hash():
        return None, "the kernels changed since profiles/%s was measured" % os.path.basename(TRAFFIC_SUMMARY)
    for line in text.splitlines():
        mt = re.match(r"^traffic_bytes_per_launch\s+(\S.*?)\s+(\d+)$", line)
        if mt and mt.group(1) == kernel:
            return float(mt.group(2)), "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/%s" % os.path.basename(TRAFFIC_SUMMARY)
    return None, "kernel not in the traffic summary"


def cpu_baseline(wl, state, g, sample_elems, steps):
    """Time the CPU oracle, as it stands, on the first `sample_elems` parameters of the workload (same state
    bits, copied from HBM): single-threaded as one chunk, and with its optional threads over independent
    (worker, chunk) problems on all host cores with the sample cut into 8 chunks."""
    import numpy as np
    import oracle
    S, n = sample_elems, wl.n
    x, m, v = (state[k][..., :S].cpu().numpy() for k in ("x", "m", "v"))
    gs = np.ascontiguousarray(g[:, :S].cpu().numpy())

    def timed(L, threads, nsteps):
        oracle.set_threads(threads)
        try:
            st = oracle.State(S, n, L, x, m, v)
            st.step(gs, wl.beta, wl.lr, wl.eps)               # page in, untimed
            t0 = time.perf_counter()
            for _ in range(nsteps):
                st.step(gs, wl.beta, wl.lr, wl.eps)
            return time.perf_counter() - t0
        finally:
            oracle.set_threads(1)

    dt1 = timed(S, 1, steps)
    cores = oracle.host_cores()
    chunks = 8 if S % (8 * 32) == 0 else 1
    dtn = timed(S // chunks, cores, 2 * steps)
    return {
        "value": S * steps / dt1, "unit": "params/s", "cores": 1, "kind": "oracle",
        "sample": "first %d parameters x %d workers of %s as one chunk, %d steps, %.1f s" % (S, n, wl.name, steps, dt1),
        "all_cores": {"value": S * 2 * steps / dtn, "unit": "params/s", "cores": cores, "kind": "oracle",
                      "sample": "the same sample as %d chunks, the oracle's threads over independent (worker, chunk) "
                                "problems on the %d cores of this process's affinity mask, %d steps, %.1f s" %
                                (chunks, cores, 2 * steps, dtn)},
    }


def region_map(args):
    """Where the big buffers lie in HBM, and what that does to the fused worker kernel: 44 buffers of a
    quarter-size problem (n = 16, 5.44 GB each) are allocated one after the other, and the gather-carrying
    worker call is timed in its fused form with the momentum, the worker error and the gradient in chosen
    ones of them.  Prints a table (stderr) and one JSON line (stdout)."""
    import torch
    from paper_2008_11343_amd import binding as B
    n = 16
    d = 340000768 // 4 // (n * 4096) * (n * 4096)
    L = d // n
    f = dict(dtype=torch.float32, device="cuda:0")
    i32 = dict(dtype=torch.int32, device="cuda:0")
    nb = 44
    blocks = [torch.zeros(n, d, **f) for _ in range(nb)]
    gib = lambda t: (blocks[0].data_ptr() - t.data_ptr()) / 2.0 ** 30     # the allocator hands out descending addresses
    x = torch.empty(d, **f).normal_(0, 0.02)
    v = torch.ones(d, **f)
    serr = torch.zeros(d, **f)
    packed, spacked = torch.zeros(n, d // 32, **i32), torch.zeros(d // 32, **i32)
    scales, sscales = torch.zeros(n, n, **f), torch.zeros(n, **f)

    def worker_ms(m, werr, g, form, reps=5):
        ctx = B.apms_create(d, n, L, 0)
        B.apms_set_deferral(ctx, B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER)
        B.apms_set_gather_mode(ctx, form)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
        for r in range(reps):
            ev[r][0].record()
            B.apms_compress(ctx, m, g, werr, packed, scales, 0.9)
            ev[r][1].record()
            B.apms_server_reduce(ctx, packed, scales, serr, spacked, sscales)
            B.apms_apply(ctx, spacked, sscales, v, x, m, 1e-4, 1e-8)
        B.apms_finalize(ctx, werr, serr, m)
        torch.cuda.synchronize()
        B.apms_destroy(ctx)
        ts = sorted(e[0].elapsed_time(e[1]) for e in ev[1:])
        return ts[len(ts) // 2]

    gcols = list(range(0, nb, 4))
    rows = []
    log("quarter-size problem: d=%d n=%d, %d buffers of %.2f GB; column = buffer of the gradient (offset from the first "
        "buffer in GiB: %s)" % (d, n, nb, n * d * 4 / 1e9, " ".join("%.0f" % gib(blocks[k]) for k in gcols)))
    for form, fname in ((B.APMS_GATHER_FUSED, "fused"), (B.APMS_GATHER_SPLIT, "split")):
        for mi, wj in ((0, 21), (0, 40), (21, 0), (21, 40), (40, 0), (40, 21), (0, 10), (21, 30), (40, 33)):
            if form == B.APMS_GATHER_SPLIT and (mi, wj) not in ((0, 21), (0, 10), (21, 30)):
                continue
            times = [None if gk in (mi, wj) else worker_ms(blocks[mi], blocks[wj], blocks[gk], form) for gk in gcols]
            rows.append({"form": fname, "m_GiB": gib(blocks[mi]), "err_GiB": gib(blocks[wj]), "ms_by_gradient_buffer": times})
            log("%-5s m at %5.0f GiB, error at %5.0f GiB: " % (fname, gib(blocks[mi]), gib(blocks[wj])) +
                " ".join("  -- " if t is None else "%5.2f" % t for t in times))
    print(json.dumps({"experiment": "region-map", "d": d, "n": n, "buffer_GB": n * d * 4 / 1e9,
                      "gradient_buffer_GiB": [gib(blocks[k]) for k in gcols], "rows": rows}), flush=True)


def measure(args, wl, place, want_state=False):
    """One measurement: allocate, initialise, warm up, time args.steps steps.  Returns a dict of raw results."""
    import torch
    from paper_2008_11343_amd import binding as B
    from paper_2008_11343_amd import workloads as W
    from paper_2008_11343_amd.runner import DeviceRun

    dev = "cuda:0"
    d, n, L = wl.d_pad, wl.n, wl.L
    deferral = {"deferred": B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER, "deferred-errors": B.APMS_DEFER_ERRORS,
                "eager": 0,
                "implicit": B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER | B.APMS_IMPLICIT_MOMENTUM}[args.mode]
    gdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.grad_dtype]
    # the run owns every buffer, the gradient input included, so that it can place them in HBM
    run = DeviceRun(d, n, L, dev, deferred=deferral, place=place, grad_dtype=gdt)
    if run.placement:
        log("placement: pair %d of %s ms (fused worker kernel)" % (
            run.placement["chosen_pair"], run.placement["fused_worker_kernel_ms_by_pair"]))
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
    if args.gather != "auto":
        B.apms_set_gather_mode(run.ctx, {"split": B.APMS_GATHER_SPLIT, "fused": B.APMS_GATHER_FUSED}[args.gather])
    topk_K = max(1, int(L * args.topk_percent / 100.0))
    if args.algo == "topk":
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        run.idx, run.val = torch.zeros(n, wl.C, topk_K, **i32), torch.zeros(n, wl.C, topk_K, **f32)
        run.sidx, run.sval = torch.zeros(wl.C, topk_K, **i32), torch.zeros(wl.C, topk_K, **f32)
        B.apms_topk_reserve(run.ctx, topk_K)
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

    warm = None
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
    # settling: with the gather deferred the library times its candidate forms of the gather-carrying worker
    # call on its first gathers (APMS_GATHER_AUTO) and then keeps the fastest; those steps are ordinary steps,
    # run before the warm-up so that the timed region sees the settled choice
    settle = 0
    auto = (args.algo == "momentum" and (deferral & B.APMS_DEFER_GATHER)
            and not (deferral & B.APMS_IMPLICIT_MOMENTUM) and args.gather == "auto")
    if auto:
        while B.apms_get_plan(run.ctx)["gather_choice"] < 0 and settle < 16:
            one_step(settle)
            torch.cuda.synchronize()
            settle += 1
    for s in range(args.warmup):
        one_step(settle + s)
    run.finalize()          # the timed region starts from a state with nothing pending
    torch.cuda.synchronize()
    plan = B.apms_get_plan(run.ctx)
    log("settling %d steps, warm-up %d steps done; gather form: %s%s, measured [split, fused, fused uncapped] = %s ms" % (
        settle, args.warmup, {-1: "undecided", 0: "split", 1: "fused"}[plan["gather_choice"]],
        " uncapped" if plan["gather_uncapped"] else "", ["%.2f" % t for t in plan["gather_ms"]]))

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    fin = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    for s in range(args.steps):
        one_step(settle + args.warmup + s, ev[s])
    fin[0].record(stream)
    run.finalize()
    fin[1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    res = {
        "t_c": [e[0].elapsed_time(e[1]) for e in ev], "t_s": [e[1].elapsed_time(e[2]) for e in ev],
        "t_a": [e[2].elapsed_time(e[3]) for e in ev], "t_fin": fin[0].elapsed_time(fin[1]), "wall": wall,
        "plan": plan, "placement": run.placement, "warm": warm, "settle": settle, "deferral": deferral,
        "gbytes": gbytes, "topk_K": topk_K,
    }
    res["total_ms"] = sum(res["t_c"]) + sum(res["t_s"]) + sum(res["t_a"]) + res["t_fin"]
    res["ms_per_step"] = res["total_ms"] / args.steps
    log("ms/step %.3f (compress %.3f, server_reduce %.3f, apply %.3f, final finalize %.3f total); wall %.2f s" % (
        res["ms_per_step"], sum(res["t_c"]) / args.steps, sum(res["t_s"]) / args.steps, sum(res["t_a"]) / args.steps,
        res["t_fin"], wall))
    if want_state:
        S = min(args.cpu_sample, L)
        res["state"] = {"x": run.x[:S].clone(), "m": run.m[:, :S].clone(), "v": run.v[:S].clone()}
        res["g32"] = g32[:, :S].clone()
    run.close()
    del run, g, g32
    gc.collect()
    torch.cuda.empty_cache()
    return res


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
                         "variant of Section 5.3; topk: APMSqueeze with the top-k compressor of Section 5.1 "
                         "(--mode eager or deferred-errors)")
    ap.add_argument("--topk-percent", type=float, default=1.0, help="kept fraction of every chunk, in percent")
    ap.add_argument("--grad-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="element type of the gradient input (f32 is the benchmark's configuration)")
    ap.add_argument("--occupancy-pad", default="", help="e.g. compress=65536,apply=0 (apms_set_occupancy_pad)")
    ap.add_argument("--gather", choices=["auto", "split", "fused"], default="auto",
                    help="form of the gather-carrying worker call (apms_set_gather_mode); auto is the library's default")
    ap.add_argument("--chunk-elems", type=int, default=0,
                    help="chunk length (the unit that has its own scale and server) instead of the workload's own, "
                         "which is d_pad / n as in the paper; a labelled variant, e.g. 65536")
    ap.add_argument("--placement", choices=["both", "tuned", "packed"], default="both",
                    help="packed: every buffer as first allocated; tuned: the worker error and the gradient are the "
                         "pair of several successively allocated buffers that the fused worker kernel runs fastest "
                         "on (the chip's HBM regions; fp32 gradients, buffers of 4 GB and more, gather deferred); "
                         "both: measure packed, then tuned, report tuned as the value and packed beside it")
    ap.add_argument("--reuse-grad", action="store_true", help="do not redraw gradients between steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of n*d floats (a kernel of known HBM traffic, for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--region-map", action="store_true",
                    help="instead of the benchmark: time the fused and the split worker call with the momentum, the "
                         "error and the gradient in different parts of HBM (the experiment behind --placement)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 23)
    ap.add_argument("--cpu-steps", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (n workers are simulated as n state slices in HBM); "
                 "--gpus N with N > 1 is not supported")

    import torch
    from paper_2008_11343_amd import binding as B
    from paper_2008_11343_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    if args.region_map:
        region_map(args)
        return
    wl = {w.name: w for w in W.CONFIGS}[args.workload]
    if args.chunk_elems:
        import dataclasses
        wl = dataclasses.replace(wl, chunk=args.chunk_elems, name="%s-chunk%d" % (wl.name, args.chunk_elems))
    if args.algo == "topk" and args.grad_dtype != "f32":
        sys.exit("bench.py: --algo topk takes fp32 gradients")
    d, n, L = wl.d_pad, wl.n, wl.L
    log("workload %s: d_pad=%d n=%d chunk=%d (%d chunks), %s gradients, mode=%s" %
        (wl.name, d, n, L, wl.C, wl.grad, args.mode))

    placeable = (args.algo in ("momentum", "topk") and args.mode == "deferred" and args.grad_dtype == "f32"
                 and 4 * n * d >= (4 << 30))
    packed = None
    if args.placement == "both" and placeable:
        log("-- packed: every buffer as first allocated")
        packed = measure(args, wl, place=False)
        log("-- tuned: worker error and gradient placed by timing")
    res = measure(args, wl, place=(args.placement != "packed") and placeable, want_state=not args.no_cpu_baseline)

    deferral, gbytes, topk_K, plan = res["deferral"], res["gbytes"], res["topk_K"], res["plan"]
    t_c, t_s, t_a, t_fin = res["t_c"], res["t_s"], res["t_a"], res["t_fin"]
    ms_per_step = res["ms_per_step"]
    value = d * args.steps / (res["total_ms"] * 1e-3)
    gather_deferred = bool(deferral & B.APMS_DEFER_GATHER)
    ab = call_bytes(n, gather_deferred=gather_deferred)
    ab["compress"] -= (4 - gbytes) * n             # 16-bit gradients: 2n fewer bytes read
    if deferral & B.APMS_IMPLICIT_MOMENTUM:
        ab["compress"] -= 4.0 * n                  # m is not written
    if args.algo == "topk":
        # algorithmic: worker reads m, g, delta and writes delta and its K-entry lists (the selection's extra
        # read of u and its slots are implementation, not counted); server reads the n lists, reads and
        # writes its error, writes its list; gather writes dense m to n slices and takes the model step
        # with the gather deferred the worker call decodes the server's list instead of reading m and writes m
        # (not with implicit momentum), and the gather call is the model step alone
        kf = topk_K / L
        ab["compress"] = (16.0 + 8.0 * kf) * n
        ab["server_reduce"] = 8.0 * kf * n + 8.0 + 8.0 * kf
        ab["apply"] = 4.0 * n + 12.0 + 8.0 * kf
        if gather_deferred:
            ab["compress"] += 8.0 * kf * n - (4.0 * n if deferral & B.APMS_IMPLICIT_MOMENTUM else 0.0)
            ab["apply"] -= 4.0 * n
    if args.algo == "gradient":
        # worker: read g, delta; write delta, n/8 signs.  apply: read + write m per worker, n/8 signs, v, x, x
        ab["compress"] = (8.0 + gbytes) * n + n / 8.0
        ab["apply"] = 8.125 * n + 12.0
    spec = call_bytes(n)                           # the workload's own accounting (eager gather)
    spec_bytes = sum(spec.values())
    mean = lambda xs: sum(xs) / len(xs)
    median = lambda xs: sorted(xs)[len(xs) // 2] if len(xs) % 2 else 0.5 * sum(sorted(xs)[len(xs) // 2 - 1:len(xs) // 2 + 1])
    step_bytes = d * sum(ab.values())
    compress_ms = mean(t_c)
    # roofline of the dominant kernel: algorithmic bytes per launch = the worker step's per-parameter figure of the
    # workload's own accounting (16.125 n: three fp32 streams in, one out, one bit of signs per worker element;
    # the deferred design moves 16.25 n, see config.GBps) x d, over the HIP-event time of the call
    plain = args.algo == "momentum" and args.grad_dtype == "f32" and not deferral & B.APMS_IMPLICIT_MOMENTUM
    algo_compress = spec["compress"] if plain else ab["compress"]
    achieved = d * algo_compress / (compress_ms * 1e-3) / 1e9
    fused = plan["gather_choice"] == B.APMS_GATHER_FUSED
    kname = None
    if args.algo == "topk":
        kernel = "apms_topk_compress (all passes of the worker selection)"
    elif args.algo == "gradient":
        kernel = "compress_kernel<momentum: none, gradient: %s> (apms_compress_gradient)" % args.grad_dtype
    elif not gather_deferred:
        kernel = "compress_kernel<momentum: read m, gradient: %s> (apms_compress)" % args.grad_dtype
        kname = "apms::compress_kernel<0, 0>"
    elif fused or deferral & B.APMS_IMPLICIT_MOMENTUM:
        kernel = "compress_kernel<momentum: pending gather%s, gradient: %s> (apms_compress)" % (
            ", m not written" if deferral & B.APMS_IMPLICIT_MOMENTUM else " written to m", args.grad_dtype)
        kname = "apms::compress_kernel<1, 0>[fused]"
    else:
        kernel = ("apms_compress as two kernels: apply_kernel<write m only> (the gather as a fill) + "
                  "compress_kernel<momentum: pending gather, m not written, gradient: %s>" % args.grad_dtype)
        kname = "apms_compress[split]"
    traffic, traffic_source = (None, "not measured for this configuration")
    if kname and plain and wl.name == "bert-large-flat" and (deferral & B.APMS_DEFER_ERRORS):
        traffic, traffic_source = measured_traffic(kname)

    # per call: which roof bounds it.  The server step decodes n sign streams per element: at large n its
    # inner loop's VALU work passes what the chip can issue in the time HBM needs for the bytes.
    server_hbm_s = d * ab["server_reduce"] / (HBM_PEAK_GBS * 1e9)
    server_alu_s = d * n * SERVER_VALU_OPS_PER_WORKER_ELEM / (CU_COUNT * LANES_PER_CU * CLOCK_GHZ * 1e9)
    server_bound = "alu" if (args.algo != "topk" and server_alu_s > server_hbm_s) else "hbm"
    calls = {
        "compress": {"bound": "hbm", "frac": d * ab["compress"] / (compress_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "server_reduce": {"bound": server_bound,
                          "frac": (server_alu_s if server_bound == "alu" else server_hbm_s) / (mean(t_s) * 1e-3),
                          "hbm_floor_ms": server_hbm_s * 1e3},
        "apply": {"bound": "hbm", "frac": d * ab["apply"] / (mean(t_a) * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if args.algo != "topk":                                   # the 1-bit server kernel's instruction count per element
        calls["server_reduce"].update(
            valu_floor_ms=server_alu_s * 1e3,
            valu_model="%d fp32 VALU ops per decoded worker element x n x d over %d CUs x %d lanes x %.1f GHz" % (
                SERVER_VALU_OPS_PER_WORKER_ELEM, CU_COUNT, LANES_PER_CU, CLOCK_GHZ))

    out = {
        "metric": METRIC, "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": "%s: d_pad=%d n=%d chunk=%d" % (wl.name, d, n, L),
            "algo": args.algo, "topk_K_per_chunk": topk_K if args.algo == "topk" else None, "mode": args.mode,
            "grad_dtype": args.grad_dtype, "gradients": wl.grad + (", reused" if args.reuse_grad else ", fresh each step"),
            "placement_of_value": "tuned" if res["placement"] else "packed",
            "worker_params_per_s": value * n,
            "bytes_per_param_step": sum(ab.values()),
            "step_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
            "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "bytes_per_param_step_eager_accounting": spec_bytes,
            "step_GBps_eager_accounting": d * spec_bytes / (ms_per_step * 1e-3) / 1e9,
            "ms": {"compress": compress_ms, "server_reduce": mean(t_s), "apply": mean(t_a),
                   "final_finalize_total": t_fin},
            "ms_per_step_median": median([a + b + c for a, b, c in zip(t_c, t_s, t_a)]),
            "GBps": {"compress": d * ab["compress"] / (compress_ms * 1e-3) / 1e9,
                     "server_reduce": d * ab["server_reduce"] / (mean(t_s) * 1e-3) / 1e9,
                     "apply": d * ab["apply"] / (mean(t_a) * 1e-3) / 1e9},
            "calls": calls,
            "plan": {k: plan[k] for k in ("compress_tiles_per_block", "compress_grid", "server_tiles_per_block",
                                          "server_grid", "apply_grid", "occupancy_pad", "gather_mode",
                                          "gather_choice", "gather_uncapped", "gather_ms")},
            "settle_steps": res["settle"],
            "wall_s_including_input_generation": res["wall"],
            "adam_warmup": res["warm"],
            "placement": res["placement"],
            "device": torch.cuda.get_device_name(0),
        },
        "roofline": {
            "kernel": kernel,
            "bound": "hbm", "achieved": achieved,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic, "traffic_source": traffic_source,
            "bytes_per_launch": d * algo_compress,
            "avg_launch_ms": compress_ms,
            "avg_launch_ms_is": "HIP-event time of the apms_compress call on the launch stream: the kernel(s) named "
                                "above plus the scales kernel (one workgroup per (worker, chunk), microseconds)",
        },
    }
    if packed is not None:
        pc = mean(packed["t_c"])
        out["config"]["packed"] = {
            "what": "the same workload and step count with every buffer where the allocator first puts it: what a "
                    "caller who just allocates gets",
            "value": d * args.steps / (packed["total_ms"] * 1e-3), "ms_per_step": packed["ms_per_step"],
            "ms": {"compress": pc, "server_reduce": mean(packed["t_s"]), "apply": mean(packed["t_a"]),
                   "final_finalize_total": packed["t_fin"]},
            "step_frac_of_hbm_peak": step_bytes / (packed["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "gather_choice": packed["plan"]["gather_choice"], "gather_uncapped": packed["plan"]["gather_uncapped"],
            "gather_ms": packed["plan"]["gather_ms"],
        }
        out["config"]["ms_per_step_packed"] = packed["ms_per_step"]
        out["roofline"]["frac_packed"] = d * algo_compress / (pc * 1e-3) / 1e9 / HBM_PEAK_GBS
        out["roofline"]["avg_launch_ms_packed"] = pc
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(wl, res["state"], res["g32"], min(args.cpu_sample, L), args.cpu_steps)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
