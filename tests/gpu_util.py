"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same
bits and compare every output.

Bars (from the build contract): indices, survivor counts and value codes bit-exact; scales and
decoded values within 1e-6 of the chunk absmax (in practice they are bit-equal, which is also
asserted, because both sides do the same single IEEE operations); residual and dense output
bit-exact."""
from __future__ import annotations

import sys

import numpy as np
import torch

import oracle
from paper_2506_16235_amd import binding as nsml

DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def compare_payload(off, ratio, bits, chunk, got, want, v_abs_by_bucket=None, buckets=None):
    """got / want: (idx, val, scales) as numpy arrays (uint32, uint8, float32).  Compares whole
    payloads, or only the slices of `buckets`."""
    k_b, K, vb, ns = oracle.layout(off, ratio, bits, chunk)
    gi, gv, gs = got
    wi, wv, ws = want
    B = len(off) - 1
    P = np.concatenate([[0], np.cumsum(k_b)]).astype(np.int64)
    per = {32: lambda k: 4 * k, 16: lambda k: 2 * k, 8: lambda k: k, 4: lambda k: (k + 1) // 2}[bits]
    V = np.concatenate([[0], np.cumsum([per(int(k)) for k in k_b])]).astype(np.int64)
    nsc = [(-(-int(k) // chunk)) if bits <= 8 else 0 for k in k_b]
    S = np.concatenate([[0], np.cumsum(nsc)]).astype(np.int64)
    todo = range(B) if buckets is None else buckets
    for b in todo:
        a, z = P[b], P[b + 1]
        assert np.array_equal(gi[a:z], wi[a:z]), f"idx differ in bucket {b}"
        assert np.array_equal(gv[V[b]:V[b + 1]], wv[V[b]:V[b + 1]]), f"codes differ in bucket {b}"
        if bits <= 8:
            g_s, w_s = gs[S[b]:S[b + 1]], ws[S[b]:S[b + 1]]
            qmax = 127.0 if bits == 8 else 7.0
            absmax = w_s.astype(np.float64) * qmax
            assert np.all(np.abs(g_s.astype(np.float64) - w_s) <= 1e-6 * absmax), f"scales off in bucket {b}"
            assert np.array_equal(g_s.view(np.uint32), w_s.view(np.uint32)), f"scale bits differ in bucket {b}"
    return k_b, K, vb, ns


class Case:
    """One gradient on the GPU and its copy on the host."""

    def __init__(self, g_dev: torch.Tensor, off, chunk=2048, max_buckets=None, ctx=None):
        self.g = g_dev
        self.off = np.ascontiguousarray(off, dtype=np.uint64)
        self.n = g_dev.numel()
        self.chunk = chunk
        self.ctx = ctx or nsml.Context(self.n, max_buckets or (len(self.off) - 1), chunk)
        self.r = torch.zeros_like(g_dev)
        self.g_host = g_dev.cpu().numpy()
        self.r_host = np.zeros(self.n, dtype=np.float32)

    def set_grad(self, g_dev):
        self.g = g_dev
        self.g_host = g_dev.cpu().numpy()

    def set_residual(self, r_host: np.ndarray):
        self.r_host = r_host.astype(np.float32).copy()
        self.r = torch.from_numpy(self.r_host).to(DEV)

    def step(self, ratio, bits, threads=16, check_dense=True):
        """One compress + decompress on both sides; asserts parity; returns payload sizes."""
        ctx, off, chunk = self.ctx, self.off, self.chunk
        idx, val, sc = ctx.compress(self.g, self.r, off, ratio, bits)
        dense = ctx.decompress(idx, val, sc, self.n, off, ratio, bits)
        torch.cuda.synchronize()
        ctx.path_stats()                      # raises if a device-side consistency check tripped
        w_idx, w_val, w_sc = oracle.compress(self.g_host, self.r_host, off, ratio, bits, chunk, nthreads=threads)
        k_b, K, vb, ns = oracle.layout(off, ratio, bits, chunk)
        got = (idx.cpu().numpy().view(np.uint32)[:K], val.cpu().numpy()[:vb], sc.cpu().numpy()[:ns])
        compare_payload(off, ratio, bits, chunk, got, (w_idx, w_val, w_sc))
        r_gpu = self.r.cpu().numpy()
        assert np.array_equal(r_gpu.view(np.uint32), self.r_host.view(np.uint32)), "residual differs"
        if check_dense:
            w_dense = oracle.decompress(w_idx, w_val, w_sc, self.n, off, ratio, bits, chunk, nthreads=threads)
            d_gpu = dense.cpu().numpy()
            assert np.array_equal(d_gpu.view(np.uint32), w_dense.view(np.uint32)), "dense differs"
        return K, vb, ns
