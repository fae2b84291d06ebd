"""Seeded synthetic gradients and bandwidth traces for the five benchmark configurations.

This module holds input generators only: tensor-size tables of public model
architectures, random value distributions and a random bandwidth trace.  None of
the method's arithmetic (accumulation, selection, coding, controller) lives here,
so both the HIP path and the CPU checker can be fed from it.  It imports neither.

The paper trains ResNet18/VGG16 on CIFAR-100 (Sec. 5.1); no dataset or trained
model is available or needed here.  The gradients below are stand-ins with the
sizes, bucket structure and value distributions the benchmark definition fixes.

Seeds: seed(cfg, step, bucket) = (cfg << 40) | (step << 20) | bucket, one torch
generator per bucket on the requested device (CPU and GPU streams differ; a run
always copies the same bits to whoever needs them).
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np
import torch

CHUNK = 2048


def make_seed(cfg: int, step: int, bucket: int) -> int:
    return (int(cfg) << 40) | (int(step) << 20) | int(bucket)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def offsets_of(sizes: Sequence[int]) -> np.ndarray:
    off = np.zeros(len(sizes) + 1, dtype=np.uint64)
    off[1:] = np.cumsum(np.asarray(sizes, dtype=np.uint64))
    return off


# ------------------------------------------------------------------ shapes

def resnet50_sizes() -> List[int]:
    """Parameter tensors of torchvision-style ResNet-50, in module order: 161 tensors,
    25,557,032 elements (conv weight, then BN gamma, BN beta; downsample after conv3)."""
    s: List[int] = [64 * 3 * 7 * 7, 64, 64]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            s += [planes * inplanes * 1 * 1, planes, planes]
            s += [planes * planes * 3 * 3, planes, planes]
            s += [planes * 4 * planes * 1 * 1, planes * 4, planes * 4]
            if blk == 0:
                s += [planes * 4 * inplanes, planes * 4, planes * 4]
            inplanes = planes * 4
    s += [1000 * 2048, 1000]
    return s


def bert_base_sizes() -> List[int]:
    """Parameter tensors of BERT-base (uncased) encoder + pooler: 199 tensors,
    109,482,240 elements.  Tensor 0 is the 30522 x 768 word embedding."""
    H, I, V = 768, 3072, 30522
    s: List[int] = [V * H, 512 * H, 2 * H, H, H]
    for _ in range(12):
        s += [H * H, H] * 4          # q, k, v, attention output
        s += [H, H]                  # attention LayerNorm
        s += [I * H, I, H * I, H]    # intermediate, output
        s += [H, H]                  # output LayerNorm
    s += [H * H, H]                  # pooler
    return s


def llama7b_sizes() -> List[int]:
    """Parameter tensors of Llama-7B: 291 tensors, 6,738,415,616 elements."""
    H, F, V, L = 4096, 11008, 32000, 32
    s: List[int] = [V * H]
    for _ in range(L):
        s += [H * H] * 4 + [F * H, F * H, H * F] + [H, H]
    s += [H, V * H]
    return s


LLAMA_BUCKET = 25 * (1 << 20)   # "25M-element buckets" read as 25 Mi elements


def llama7b_bucket_offsets(bucket: int = LLAMA_BUCKET) -> np.ndarray:
    """The flattened Llama-7B gradient cut every `bucket` elements (last one short)."""
    n = sum(llama7b_sizes())
    cuts = list(range(0, n, bucket)) + [n]
    return np.asarray(cuts, dtype=np.uint64)


# ------------------------------------------------------------ distributions

def _normal(n: int, sigma: float, gen, device) -> torch.Tensor:
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32).mul_(sigma)


def _laplace(n: int, b: float, gen, device) -> torch.Tensor:
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float32).sub_(0.5)
    mag = (1.0 - 2.0 * u.abs()).clamp_min_(2.0 ** -24).log_().mul_(-b)
    return mag.mul_(torch.sign(u))


def _student_t3(n: int, scale: float, gen, device) -> torch.Tensor:
    z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    c = torch.zeros(n, device=device, dtype=torch.float32)
    for _ in range(3):
        w = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        c.addcmul_(w, w)
    return z.div_(c.div_(3.0).sqrt_()).mul_(scale)


# ------------------------------------------------------------------ configs

def cfg1(device="cpu") -> Tuple[torch.Tensor, np.ndarray]:
    """1,048,576 elements, N(0, sigma=1e-3), seed 0, one bucket."""
    n = 1 << 20
    g = _normal(n, 1e-3, _gen(device, 0), device)
    return g, offsets_of([n])


def resnet50_sigmas(cfg: int = 2) -> np.ndarray:
    """Per-layer sigma, log-uniform in [1e-5, 1e-2], fixed for the whole run."""
    rng = np.random.default_rng(make_seed(cfg, 0, 0))
    return 10.0 ** rng.uniform(-5.0, -2.0, size=len(resnet50_sizes()))


def resnet50_grad(step: int, device="cpu", cfg: int = 2, out: torch.Tensor | None = None):
    """ResNet-50-shaped gradient for `step`: bucket l ~ N(0, sigma_l)."""
    sizes = resnet50_sizes()
    off = offsets_of(sizes)
    sig = resnet50_sigmas(cfg)
    g = out if out is not None else torch.empty(int(off[-1]), device=device, dtype=torch.float32)
    for b, nb in enumerate(sizes):
        g[int(off[b]):int(off[b + 1])] = _normal(nb, float(sig[b]),
                                                 _gen(device, make_seed(cfg, step, b)), device)
    return g, off


BERT_VOCAB, BERT_HIDDEN, BERT_NONZERO_ROWS = 30522, 768, 1526


def bert_grad(step: int = 0, device="cpu", out: torch.Tensor | None = None):
    """BERT-base-shaped gradient: Laplace(0, 1e-4); 95 % of the word-embedding rows are
    exactly zero (1,526 of 30,522 rows, chosen by a seeded permutation, are non-zero)."""
    cfg = 3
    sizes = bert_base_sizes()
    off = offsets_of(sizes)
    g = out if out is not None else torch.empty(int(off[-1]), device=device, dtype=torch.float32)
    for b, nb in enumerate(sizes):
        gen = _gen(device, make_seed(cfg, step, b))
        if b == 0:
            emb = g[:nb].view(BERT_VOCAB, BERT_HIDDEN)
            emb.zero_()
            rows = torch.randperm(BERT_VOCAB, generator=gen, device=device)[:BERT_NONZERO_ROWS]
            emb[rows] = _laplace(BERT_NONZERO_ROWS * BERT_HIDDEN, 1e-4, gen, device).view(
                BERT_NONZERO_ROWS, BERT_HIDDEN)
        else:
            g[int(off[b]):int(off[b + 1])] = _laplace(nb, 1e-4, gen, device)
    return g, off


def llama7b_grad(step: int, device="cpu", out: torch.Tensor | None = None,
                 buckets: Sequence[int] | None = None, bucket: int = LLAMA_BUCKET):
    """Llama-7B-shaped gradient: Student-t(nu=3) * 1e-4, generated bucket by bucket.
    `buckets` restricts generation to some buckets (others are left untouched)."""
    cfg = 4
    off = llama7b_bucket_offsets(bucket)
    g = out if out is not None else torch.empty(int(off[-1]), device=device, dtype=torch.float32)
    todo = range(len(off) - 1) if buckets is None else buckets
    for b in todo:
        lo, hi = int(off[b]), int(off[b + 1])
        g[lo:hi] = _student_t3(hi - lo, 1e-4, _gen(device, make_seed(cfg, step, b)), device)
    return g, off


def llama_part_grad(step: int, device="cpu", nbuckets: int = 16, bucket: int = LLAMA_BUCKET):
    """The first `nbuckets` buckets of the Llama-7B-shaped gradient as a gradient of its own
    (16 buckets: 419,430,400 elements), the mid-size case the high-ratio measurements use."""
    off = llama7b_bucket_offsets(bucket)[:nbuckets + 1]
    g = torch.empty(int(off[-1]), device=device, dtype=torch.float32)
    for b in range(nbuckets):
        g[int(off[b]):int(off[b + 1])] = llama7b_bucket_values(step, b, device, bucket)
    return g, off


def llama7b_bucket_values(step: int, b: int, device="cpu", bucket: int = LLAMA_BUCKET):
    """The values of one Llama bucket, standalone (same bits as llama7b_grad writes)."""
    off = llama7b_bucket_offsets(bucket)
    nb = int(off[b + 1] - off[b])
    return _student_t3(nb, 1e-4, _gen(device, make_seed(4, step, b)), device)


def scaled_model_like(sizes: Sequence[int], divisor: int, floor: int = 1) -> List[int]:
    """Shrink every tensor of a size table (keeps the bucket count and the mix of tiny and
    large buckets) so the CPU checker finishes in seconds."""
    return [max(floor, int(math.ceil(s / divisor))) for s in sizes]


# ------------------------------------------------------------ network trace

def bandwidth_trace(steps: int = 200, seed: int = make_seed(5, 0, 0)) -> np.ndarray:
    """Piecewise-constant link bandwidth in bits/s per step: segments of 5..30 steps,
    level log-uniform in 1..100 Gb/s, one segment in ten is a congestion drop to 1..5 Gb/s."""
    rng = np.random.default_rng(seed)
    bw = np.empty(steps, dtype=np.float64)
    i = 0
    while i < steps:
        seg = int(rng.integers(5, 31))
        if rng.random() < 0.10:
            level = rng.uniform(1e9, 5e9)
        else:
            level = 10.0 ** rng.uniform(9.0, 11.0)
        bw[i:i + seg] = level
        i += seg
    return bw


RTPROP0 = 0.010   # seconds of propagation delay in the simulated link


def simulated_tx_seconds(payload_bytes: float, bw_bits_per_s: float) -> float:
    """Transmission time the simulated link reports for one payload."""
    return RTPROP0 + 8.0 * payload_bytes / bw_bits_per_s
