#!/usr/bin/env python3
"""Benchmark of the gradient data-reduction hot path on one MI355X.

A step = one nsml_compress + one nsml_decompress over one worker's whole synthetic gradient,
inputs resident in HBM.  Prints ONE JSON line:
  value     GB/s of input fp32 gradient per step (4n / t_step), whole job (one GPU)
  roofline  the dominant kernel (ef_emit: reads grad and residual, writes the accumulator:
            12 algorithmic bytes per element) against the 8 TB/s HBM peak, its duration
            measured with HIP events by the library on the stream it is launched on
  cpu_baseline  the CPU oracle timed on this host's cores on a bounded sample of the workload
  other_workloads  the same step timed on the other benchmark configurations (the 110 M-element
            gradient at its six (ratio, bits) combinations, the ResNet-50 shape, the 1 Mi-element
            vector), each with its fraction of the 8 TB/s floor model and its kernel times
Workloads (all synthetic, seeded; see paper_2506_16235_amd/workloads.py):
  llama7b   6,738,415,616 elements in 258 buckets of 25 Mi, Student-t(3)*1e-4, ratio 0.001,
            int4, residual carried across steps      (default: the largest single-GPU config)
  bert      109,482,240 elements in 199 per-tensor buckets, Laplace(0,1e-4), 95 % zero
            embedding rows, ratio 0.01 int8 (override with --ratio / --bits)
  resnet50  25,557,032 elements in 161 buckets, N(0, sigma_l), ratio 0.05 int8
  cfg1      1,048,576 elements, one bucket, N(0,1e-3), ratio 0.01 int8
Other modes: --ceilings times plain streaming kernels (read, fill, add, copy) of the library's
access shape; --source-hash prints the hash that ties a profile summary to the kernel sources.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
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
    "llama419m": (0.5, 8, 2),        # the first 16 Llama buckets: the high-ratio measurements
}
STREAMING = ("ef_emit", "decomp", "whist")      # the kernels that move whole gradients


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    """sha256 over the library's sources: a profile summary taken on other sources is stale."""
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(ROOT, "paper_2506_16235_amd", "csrc", "*.h*")) +
                    glob.glob(os.path.join(ROOT, "paper_2506_16235_amd", "csrc", "*.c"))):
        h.update(os.path.basename(p).encode())
        h.update(open(p, "rb").read())
    return h.hexdigest()[:16]


def make_grads(workload, count, dev):
    import torch
    from paper_2506_16235_amd import workloads as W
    grads = []
    off = None
    for s in range(count):
        t0 = time.time()
        if workload == "llama7b":
            g, off = W.llama7b_grad(s, dev)
        elif workload == "llama419m":
            g, off = W.llama_part_grad(s, dev)
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
    host_cpus = os.cpu_count() or 1
    cores = min(16, host_cpus)
    sizes = (off[1:] - off[:-1]).astype(np.int64)
    if workload in ("llama7b", "llama419m"):
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
           "host_cpu_count": host_cpus, "thread_cap": 16,
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"{what}; {gs[0].size} elements per step, compress+decompress, one bucket per thread"}
    if workload not in ("llama7b", "llama419m"):
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


class Job:
    """One workload resident in HBM: gradients, residual, payload and dense buffers, a context."""

    def __init__(self, workload, grads, off, ratio, bits, chunk, prune=False):
        import torch
        from paper_2506_16235_amd import binding as nsml
        self.nsml, self.torch = nsml, torch
        self.workload, self.grads, self.off = workload, grads, off
        self.ratio, self.bits, self.chunk = ratio, bits, chunk
        dev = grads[0].device
        self.n = grads[0].numel()
        self.B = len(off) - 1
        self.ctx = nsml.Context(self.n, self.B, chunk)
        k_b, self.K, vb, ns = nsml.payload_layout(off, ratio, bits, chunk)
        self.payload = 4 * self.K + vb + 4 * ns
        self.idx, self.val, self.sc = self.ctx.alloc_payload(off, ratio, bits)
        self.residual = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.dense = torch.empty(self.n, dtype=torch.float32, device=dev)
        self.step_no = 0
        self.weights = None
        if prune:
            gen = torch.Generator(device=dev)
            gen.manual_seed(99)
            self.weights = torch.empty(self.n, dtype=torch.float32, device=dev)
            for lo in range(0, self.n, 1 << 28):
                hi = min(self.n, lo + (1 << 28))
                self.weights[lo:hi] = torch.randn(hi - lo, generator=gen, device=dev) * 0.02

    def step(self):
        g = self.grads[self.step_no % len(self.grads)]
        self.step_no += 1
        c = self.ctx
        if self.weights is not None:
            c.compress_pruned(g, self.residual, self.weights, self.off, self.ratio, self.bits, self.idx, self.val, self.sc)
        else:
            c.compress(g, self.residual, self.off, self.ratio, self.bits, self.idx, self.val, self.sc)
        c.decompress(self.idx, self.val, self.sc, self.n, self.off, self.ratio, self.bits, self.dense)

    def timed(self, steps, warmup, step_fn=None):
        """W untimed steps, then exactly K steps between two synchronisations -> ms per step."""
        torch = self.torch
        fn = step_fn or self.step
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def profiled(self, steps):
        """The same steps with every kernel bracketed by HIP events (library side, on the launch
        stream) -> ({kernel: (launches, total ms)}, wall ms per step)."""
        torch = self.torch
        self.ctx.profile_enable(True)
        self.ctx.profile_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps * 1e3
        prof = self.ctx.profile_read()
        self.ctx.profile_enable(False)
        return prof, wall

    def floor_bytes(self):
        """What one step must move at least: grad and residual read, accumulator written, dense
        output written, the payload written and read; with pruning also the weights read once."""
        return (20.0 if self.weights is not None else 16.0) * self.n + 2.0 * self.payload

    def summary(self, ms_per_step, prof, steps):
        per_step = {k: ms / steps for k, (c, ms) in prof.items() if c >= steps}
        streaming = {k: round(v, 5) for k, v in per_step.items() if k in STREAMING}
        small = {k: v for k, v in per_step.items() if k not in STREAMING}
        return {
            "elements": self.n, "buckets": self.B, "ratio": self.ratio, "bits": self.bits,
            "ms_per_step": round(ms_per_step, 4),
            "gbs_input": round(4.0 * self.n / (ms_per_step * 1e-3) / 1e9, 1),
            "hbm_roofline_frac": round(self.floor_bytes() / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
            "ef_emit_ms": streaming.get("ef_emit"), "decomp_ms": streaming.get("decomp"),
            "small_kernels_ms": round(sum(small.values()), 5), "small_kernel_launches": len(small),
            "kernel_ms_per_step": {k: round(v, 5) for k, v in sorted(per_step.items(), key=lambda kv: -kv[1])},
        }


def other_workloads(chunk, dev):
    """The remaining benchmark configurations, a few steps each (bounded: about 10 s)."""
    out = {}
    plan = [("bert", [(0.1, 8), (0.1, 4), (0.01, 8), (0.01, 4), (0.001, 8), (0.001, 4)], 30, 5),
            ("resnet50", [(0.05, 8)], 50, 5), ("cfg1", [(0.01, 8)], 100, 10),
            ("llama419m", [(0.5, 8), (1.0, 8), (0.13, 8)], 10, 3)]
    import torch
    for workload, combos, steps, warm in plan:
        grads, off = make_grads(workload, DEFAULTS[workload][2], dev)
        for ratio, bits in combos:
            job = Job(workload, grads, off, ratio, bits, chunk)
            ms = job.timed(steps, warm)
            prof, _ = job.profiled(steps)
            fast, fb = job.ctx.path_stats()
            key = f"{workload}_r{ratio:g}_b{bits}"
            out[key] = job.summary(ms, prof, steps)
            out[key]["selection_paths"] = {"candidate_buckets": fast, "dense_fallback_buckets": fb}
            out[key]["steps"] = steps
            log(f"[bench] {key}: {ms:.4f} ms/step, frac {out[key]['hbm_roofline_frac']}")
            job.ctx.close()
            del job
        del grads
        torch.cuda.empty_cache()
    return out


def ceilings(dev, gib=4, reps=10):
    """What this machine sustains for the plain access patterns of the streaming kernels."""
    import torch
    from paper_2506_16235_amd import binding as nsml
    n = gib * (1 << 30) // 4
    a = torch.zeros(n, dtype=torch.float32, device=dev)
    b = torch.zeros(n, dtype=torch.float32, device=dev)
    moved = {"read": 1, "fill": 1, "add": 3, "copy": 2}
    out = {"array_gib": gib, "reps": reps, "unit": "GB/s", "peak": HBM_PEAK_GBS}
    for mode in ("read", "fill", "add", "copy"):
        for nt in (False, True):
            nsml.calibration_stream(mode, a, b, nt)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                nsml.calibration_stream(mode, a, b, nt)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            out[f"{mode}{'_nt' if nt else ''}"] = round(moved[mode] * n * 4 / (ms * 1e-3) / 1e9, 1)
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
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the extra timings of the other benchmark configurations")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step per distinct gradient in a HIP graph and time graph replays")
    ap.add_argument("--prune", action="store_true",
                    help="time nsml_compress_pruned (weight-magnitude pruning first) instead of nsml_compress")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB copy kernel (k_calib_copy): the yardstick for "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--ceilings", action="store_true",
                    help="time the plain streaming kernels (k_calib_read/fill/add/copy2) and print their GB/s")
    ap.add_argument("--source-hash", action="store_true", help="print the kernel-source hash and exit")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="nsml_set_option setting applied to every context (tuning experiments), may repeat")
    args = ap.parse_args()
    if args.source_hash:
        print(kernel_source_hash())
        return 0
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one worker's pipeline on ONE GPU; a run with "
              "--gpus > 1 is not defined (no collectives are part of the path).", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2506_16235_amd import binding as nsml

    dev = "cuda:0"
    for kv in args.opt:
        name, _, value = kv.partition("=")
        nsml.Context.default_options[name] = int(value)
    if args.ceilings:
        print(json.dumps({"stream_ceilings": ceilings(dev)}), flush=True)
        return 0
    ratio, bits, ngrads = DEFAULTS[args.workload]
    ratio = args.ratio if args.ratio is not None else ratio
    bits = args.bits if args.bits is not None else bits
    chunk = args.chunk

    grads, off = make_grads(args.workload, ngrads, dev)
    job = Job(args.workload, grads, off, ratio, bits, chunk, prune=args.prune)
    n, B, K, payload = job.n, job.B, job.K, job.payload
    log(f"[bench] {args.workload}: n={n} B={B} ratio={ratio} bits={bits} K={K} payload={payload} B "
        f"workspace={job.ctx.workspace_bytes / 2**30:.2f} GiB")

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        nsml.calibration_copy(a, b)
        torch.cuda.synchronize()
        del a, b

    step_fn = None
    if args.graph:
        for _ in range(args.warmup):
            job.step()
        torch.cuda.synchronize()
        # one graph per distinct gradient buffer; the residual, payload and dense buffers are shared
        graphs = []
        cap_stream = torch.cuda.Stream()
        for gi in range(len(grads)):
            gr = torch.cuda.CUDAGraph()
            job.step_no = gi
            with torch.cuda.stream(cap_stream):
                with torch.cuda.graph(gr, stream=cap_stream):
                    job.step()
            graphs.append(gr)
        torch.cuda.synchronize()
        job.step_no = 0

        def step_fn():
            graphs[job.step_no % len(graphs)].replay()
            job.step_no += 1

    # ---- the timed region: W warm-up steps, then exactly K steps between two synchronisations
    ms_per_step = job.timed(args.steps, args.warmup, step_fn)
    # ---- the same K steps again with every kernel bracketed by HIP events
    prof, wall_prof = job.profiled(args.steps)
    kernels = {k: {"launches": c, "avg_ms": round(ms / c, 5)} for k, (c, ms) in prof.items()}
    cand_buckets, dense_buckets = job.ctx.path_stats()      # of the last step, outside the timed region
    ef = prof.get("ef_emit")
    ef_ms = ef[1] / ef[0]
    achieved = EF_HIST_BYTES_PER_ELEM * n / (ef_ms * 1e-3) / 1e9

    # HBM bytes per launch come from rocprofv3 --pmc runs made offline (FETCH_SIZE, WRITE_SIZE,
    # calibrated on a plain copy) and kept in the committed profile summary of this workload; they
    # are reported only while that summary was taken on the kernel sources of this build
    traffic = step_traffic = None
    src_hash = kernel_source_hash()
    prof_hash = None
    tpath = os.path.join(ROOT, "profiles", f"ef_emit_{args.workload}{'_pruned' if args.prune else ''}.txt")
    if os.path.exists(tpath):
        text = open(tpath).read()
        m = re.search(r"kernel_sources_sha256:\s*([0-9a-f]+)", text)
        prof_hash = m.group(1) if m else None
        if prof_hash == src_hash:
            m = re.search(r"hbm_bytes_per_launch:\s*([0-9.eE+]+)", text)
            traffic = float(m.group(1)) if m else None
            m = re.search(r"hbm_bytes_per_step:\s*([0-9.eE+]+)", text)
            step_traffic = float(m.group(1)) if m else None

    value = 4.0 * n / (ms_per_step * 1e-3) / 1e9
    floor_bytes = job.floor_bytes()
    out = {
        "metric": "compress+decompress GB/s of fp32 gradient per step; % of HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "elements": n, "buckets": B, "ratio": ratio,
                   "bits": bits, "chunk": chunk, "survivors": K, "payload_bytes": payload,
                   "distinct_gradients": len(grads), "residual": "carried across steps",
                   "weight_pruning": bool(args.prune), "hip_graph": bool(args.graph),
                   "options": dict(nsml.Context.default_options)},
        "hbm_roofline_frac": round(floor_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "floor_bytes_per_step": floor_bytes,
        "profiled_offline": {"hbm_bytes_per_step": step_traffic,
                             "hbm_gbs": round(step_traffic / (ms_per_step * 1e-3) / 1e9, 1) if step_traffic else None,
                             "summary": os.path.relpath(tpath, ROOT) if os.path.exists(tpath) else None,
                             "summary_kernel_sources": prof_hash, "this_build_kernel_sources": src_hash,
                             "note": None if prof_hash == src_hash else
                             "the committed rocprofv3 summary was taken on other kernel sources: byte counts withheld"},
        "roofline": {"kernel": "ef_emit", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "avg_ms": round(ef_ms, 5),
                     "algorithmic_bytes_per_launch": EF_HIST_BYTES_PER_ELEM * n},
        "selection_paths": {"candidate_buckets": cand_buckets, "dense_fallback_buckets": dense_buckets},
        "kernels": kernels,
        "ms_per_step_profiled": round(wall_prof, 4),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, grads, off, ratio, bits, chunk)
    if not args.no_other_workloads and args.workload == "llama7b" and not args.prune and not args.graph:
        job.ctx.close()
        del job
        torch.cuda.empty_cache()
        # the same step preceded by the weight-magnitude pruning of Algorithm 2 Step 2
        pj = Job(args.workload, grads, off, ratio, bits, chunk, prune=True)
        pms = pj.timed(4, 2)
        pprof, _ = pj.profiled(4)
        band, wdense = pj.ctx.prune_stats()
        out["pruned_variant"] = pj.summary(pms, pprof, 4)
        out["pruned_variant"]["weight_buckets"] = {"from_band": band, "dense_passes": wdense}
        log(f"[bench] pruned variant: {pms:.3f} ms/step")
        pj.ctx.close()
        del pj, grads
        torch.cuda.empty_cache()
        out["other_workloads"] = other_workloads(chunk, dev)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
