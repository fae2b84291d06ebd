#!/usr/bin/env python3
"""Benchmark of the gradient data-reduction hot path on one MI355X.

A step = one nsml_compress + one nsml_decompress over one worker's whole synthetic gradient,
inputs resident in HBM.  Prints ONE JSON line:
  value     GB/s of input fp32 gradient per step (4n / t_step), whole job (one GPU)
  roofline  the dominant kernel (ef_emit: reads grad and residual, writes the accumulator:
            12 algorithmic bytes per element) against the 8 TB/s HBM peak, its duration
            measured with HIP events by the library on the stream it is launched on
  cpu_baseline  the CPU oracle timed on this host's cores on a bounded sample of the workload
Workloads (all synthetic, seeded; see paper_2506_16235_amd/workloads.py):
  llama7b   6,738,415,616 elements in 258 buckets of 25 Mi, Student-t(3)*1e-4, ratio 0.001,
            int4, residual carried across steps      (default: the largest single-GPU config)
  bert      109,482,240 elements in 199 per-tensor buckets, Laplace(0,1e-4), 95 % zero
            embedding rows, ratio 0.01 int8 (override with --ratio / --bits)
  resnet50  25,557,032 elements in 161 buckets, N(0, sigma_l), ratio 0.05 int8
  cfg1      1,048,576 elements, one bucket, N(0,1e-3), ratio 0.01 int8
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

HBM_PEAK_GBS = 8000.0
EF_HIST_BYTES_PER_ELEM = 12.0     # read grad, read residual, write accumulator

DEFAULTS = {          # workload -> (ratio, bits, distinct gradients kept in HBM)
    "llama7b": (0.001, 4, 2),
    "bert": (0.01, 8, 2),
    "resnet50": (0.05, 8, 4),
    "cfg1": (0.01, 8, 1),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_grads(workload, count, dev):
    import torch
    from paper_2506_16235_amd import workloads as W
    grads = []
    off = None
    for s in range(count):
        t0 = time.time()
        if workload == "llama7b":
            g, off = W.llama7b_grad(s, dev)
        elif workload == "bert":
            g, off = W.bert_grad(s, dev)
        elif workload == "resnet50":
            g, off = W.resnet50_grad(s, dev)
        else:
            g, off = W.cfg1(dev)
        torch.cuda.synchronize()
        log(f"[bench] gradient {s} of {workload}: {g.numel()} elements in {time.time() - t0:.1f}s")
        grads.append(g)
    return grads, off


def cpu_baseline(workload, grads, off, ratio, bits, chunk):
    """The oracle, as it stands, timed on this host's cores on a bounded sample of the same
    workload sized for roughly 10-30 s of CPU work: whole buckets (one bucket per thread), and
    for the workloads that fit, several steps with the residual carried."""
    import numpy as np
    import oracle
    cores = min(16, os.cpu_count() or 1)
    sizes = (off[1:] - off[:-1]).astype(np.int64)
    if workload == "llama7b":
        pick = list(range(min(4 * cores, len(sizes))))
        steps = 1
        what = f"first {len(pick)} of {len(sizes)} buckets (25 Mi elements each), 1 step"
    else:
        pick = list(range(len(sizes)))
        steps = {"bert": 10, "resnet50": 40, "cfg1": 100}[workload]
        what = f"all {len(sizes)} buckets, {steps} steps with the residual carried"
    lo, hi = int(off[pick[0]]), int(off[pick[-1] + 1])
    gs = [g[lo:hi].cpu().numpy() for g in grads]
    sub_off = (off[pick[0]:pick[-1] + 2] - off[pick[0]]).astype(np.uint64)
    r = np.zeros_like(gs[0])
    oracle.lib()
    t0 = time.perf_counter()
    for s in range(steps):
        g = gs[s % len(gs)]
        idx, val, sc = oracle.compress(g, r, sub_off, ratio, bits, chunk, nthreads=cores)
        oracle.decompress(idx, val, sc, g.size, sub_off, ratio, bits, chunk, nthreads=cores)
    dt = time.perf_counter() - t0
    used = min(cores, len(pick))
    out = {"value": round(4.0 * gs[0].size * steps / dt / 1e9, 4), "unit": "GB/s", "cores": used,
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"{what}; {gs[0].size} elements per step, compress+decompress, one bucket per thread"}
    if workload != "llama7b":
        # the same on one thread (the three small configurations only), fewer steps
        steps1 = {"bert": 1, "resnet50": 4, "cfg1": 20}[workload]
        r = np.zeros_like(gs[0])
        t0 = time.perf_counter()
        for s in range(steps1):
            g = gs[s % len(gs)]
            idx, val, sc = oracle.compress(g, r, sub_off, ratio, bits, chunk, nthreads=1)
            oracle.decompress(idx, val, sc, g.size, sub_off, ratio, bits, chunk, nthreads=1)
        dt1 = time.perf_counter() - t0
        out["single_thread"] = {"value": round(4.0 * gs[0].size * steps1 / dt1 / 1e9, 4), "unit": "GB/s",
                                "seconds": round(dt1, 2), "steps": steps1}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama7b", choices=sorted(DEFAULTS))
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--chunk", type=int, default=2048)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step per distinct gradient in a HIP graph and time graph replays")
    ap.add_argument("--prune", action="store_true",
                    help="time nsml_compress_pruned (weight-magnitude pruning first) instead of nsml_compress")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB copy kernel (k_calib_copy): the yardstick for "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one worker's pipeline on ONE GPU; a run with "
              "--gpus > 1 is not defined (no collectives are part of the path).", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2506_16235_amd import binding as nsml

    dev = "cuda:0"
    ratio, bits, ngrads = DEFAULTS[args.workload]
    ratio = args.ratio if args.ratio is not None else ratio
    bits = args.bits if args.bits is not None else bits
    chunk = args.chunk

    grads, off = make_grads(args.workload, ngrads, dev)
    n = grads[0].numel()
    B = len(off) - 1
    ctx = nsml.Context(n, B, chunk)
    k_b, K, vb, ns = nsml.payload_layout(off, ratio, bits, chunk)
    payload = 4 * K + vb + 4 * ns
    idx, val, sc = ctx.alloc_payload(off, ratio, bits)
    residual = torch.zeros(n, dtype=torch.float32, device=dev)
    dense = torch.empty(n, dtype=torch.float32, device=dev)
    log(f"[bench] {args.workload}: n={n} B={B} ratio={ratio} bits={bits} K={K} payload={payload} B "
        f"workspace={ctx.workspace_bytes / 2**30:.2f} GiB")

    step_no = [0]
    weights = None
    if args.prune:
        gen = torch.Generator(device=dev)
        gen.manual_seed(99)
        weights = torch.empty(n, dtype=torch.float32, device=dev)
        for lo in range(0, n, 1 << 28):
            hi = min(n, lo + (1 << 28))
            weights[lo:hi] = torch.randn(hi - lo, generator=gen, device=dev) * 0.02

    def step():
        g = grads[step_no[0] % len(grads)]
        step_no[0] += 1
        if weights is not None:
            ctx.compress_pruned(g, residual, weights, off, ratio, bits, idx, val, sc)
        else:
            ctx.compress(g, residual, off, ratio, bits, idx, val, sc)
        ctx.decompress(idx, val, sc, n, off, ratio, bits, dense)

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        nsml.calibration_copy(a, b)
        torch.cuda.synchronize()
        del a, b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    eager_step = step
    if args.graph:
        # one graph per distinct gradient buffer; the residual, payload and dense buffers are shared
        graphs = []
        cap_stream = torch.cuda.Stream()
        for gi in range(len(grads)):
            gr = torch.cuda.CUDAGraph()
            step_no[0] = gi
            with torch.cuda.stream(cap_stream):
                with torch.cuda.graph(gr, stream=cap_stream):
                    eager_step()
            graphs.append(gr)
        torch.cuda.synchronize()
        step_no[0] = 0

        def step():
            graphs[step_no[0] % len(graphs)].replay()
            step_no[0] += 1
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()

    # ---- the timed region: exactly K steps between two synchronisations
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # ---- the same K steps again with every kernel bracketed by HIP events (library side,
    #      on the launch stream) for the per-kernel durations
    ctx.profile_enable(True)
    ctx.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        eager_step()
    torch.cuda.synchronize()
    wall_prof = time.perf_counter() - t0
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    kernels = {k: {"launches": c, "avg_ms": round(ms / c, 5)} for k, (c, ms) in prof.items()}
    cand_buckets, dense_buckets = ctx.path_stats()      # of the last step, outside the timed region
    ef = prof.get("ef_emit")
    ef_ms = ef[1] / ef[0]
    achieved = EF_HIST_BYTES_PER_ELEM * n / (ef_ms * 1e-3) / 1e9

    traffic = None
    step_traffic = None
    # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, calibrated on a
    # plain copy); the figure is kept in the committed profile summary of this workload
    tpath = os.path.join(ROOT, "profiles", f"ef_emit_{args.workload}.txt")
    if os.path.exists(tpath):
        import re
        m = re.search(r"hbm_bytes_per_launch:\s*([0-9.eE+]+)", open(tpath).read())
        traffic = float(m.group(1)) if m else None
        m = re.search(r"hbm_bytes_per_step:\s*([0-9.eE+]+)", open(tpath).read())
        step_traffic = float(m.group(1)) if m else None

    value = 4.0 * n / (ms_per_step * 1e-3) / 1e9
    floor_bytes = 16.0 * n + 2.0 * payload
    out = {
        "metric": "compress+decompress GB/s of fp32 gradient per step; % of HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "elements": n, "buckets": B, "ratio": ratio,
                   "bits": bits, "chunk": chunk, "survivors": K, "payload_bytes": payload,
                   "distinct_gradients": len(grads), "residual": "carried across steps",
                   "weight_pruning": bool(args.prune), "hip_graph": bool(args.graph)},
        "hbm_roofline_frac": round(floor_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "floor_bytes_per_step": floor_bytes,
        "measured_hbm_bytes_per_step": step_traffic,
        "measured_hbm_gbs": round(step_traffic / (ms_per_step * 1e-3) / 1e9, 1) if step_traffic else None,
        "roofline": {"kernel": "ef_emit", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "avg_ms": round(ef_ms, 5),
                     "algorithmic_bytes_per_launch": EF_HIST_BYTES_PER_ELEM * n},
        "selection_paths": {"candidate_buckets": cand_buckets, "dense_fallback_buckets": dense_buckets},
        "kernels": kernels,
        "ms_per_step_profiled": round(wall_prof / args.steps * 1e3, 4),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, grads, off, ratio, bits, chunk)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
