"""GPU parity on seeded random configurations: bucket layouts, ratios, value widths, chunk sizes,
value distributions (heavy tails, ties, mostly zeros), with and without weight pruning, under
random choices of the library's internal geometry switches.  Three error-feedback steps each,
every output compared with the oracle bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_16235_amd import binding as nsml
from paper_2506_16235_amd import workloads as W
from gpu_util import DEV, compare_payload, say

pytestmark = pytest.mark.gpu


def _case(seed, pruned, monkeypatch):
    rs = np.random.RandomState(seed)
    st = int(rs.choice([0, 1, 2, 4, 8, 16]))
    sw = int(rs.choice([0, 4, 8, 16]))
    rs.choice([0, 4, 16, 64])                 # (keeps the stream of the later draws as it was)
    for k, v in (("span_tiles", st), ("seg_waves", sw)):
        monkeypatch.setitem(nsml.Context.default_options, k, v)
    rs.randint(0, 2)                          # (keeps the stream of the later draws as it was)
    monkeypatch.setitem(nsml.Context.default_options, "force_dense", 1 if rs.rand() < 0.15 else 0)
    monkeypatch.setitem(nsml.Context.default_options, "rescan", 1 if rs.rand() < 0.25 else 0)
    B = int(rs.randint(1, 9))
    sizes = []
    for _ in range(B):
        kind = rs.randint(0, 6)
        sizes.append(int([0, rs.randint(1, 70), rs.randint(70, 9000), rs.randint(9000, 300000),
                          rs.randint(262144, 700000), rs.randint(700000, 2500000)][kind]))
    if sum(sizes) == 0:
        sizes[0] = 5
    off = W.offsets_of(sizes)
    n = int(off[-1])
    chunk = int(rs.choice([8, 64, 256, 2048]))
    bits = int(rs.choice([4, 8, 16, 32]))
    dist = int(rs.randint(0, 4))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    say("random case", seed, "pruned" if pruned else "plain", sizes, "chunk", chunk, "bits", bits, "dist", dist,
        "geometry", st, sw)

    def grad():
        g = torch.randn(n, generator=gen, device=DEV) * 1e-3
        if dist == 1:
            g = g * torch.exp(torch.randn(n, generator=gen, device=DEV) * 2)      # heavy tails
        if dist == 2:
            g = torch.round(g * 3e3) / 3e3                                             # ties
        if dist == 3:
            g[torch.rand(n, generator=gen, device=DEV) < 0.9] = 0.0                  # mostly zeros
        return g

    ctx = nsml.Context(n, B, chunk)
    r = torch.zeros(n, device=DEV)
    r_h = np.zeros(n, dtype=np.float32)
    for _ in range(3):
        ratio = float(rs.choice([0.001, 0.005, 0.01, 0.03, 0.1, 0.3, 1.0]))
        g = grad()
        if pruned:
            w = torch.randn(n, generator=gen, device=DEV) * 0.05
            if rs.rand() < 0.4:
                q = float(rs.choice([40, 2000, 20000]))
                w = torch.round(w * q) / q
            idx, val, sc = ctx.compress_pruned(g, r, w, off, ratio, bits)
        else:
            idx, val, sc = ctx.compress(g, r, off, ratio, bits)
        dense = ctx.decompress(idx, val, sc, n, off, ratio, bits)
        torch.cuda.synchronize()
        ctx.path_stats()
        if pruned:
            ctx.prune_stats()
            w_idx, w_val, w_sc = oracle.compress_pruned(g.cpu().numpy(), r_h, w.cpu().numpy(), off, ratio, bits,
                                                        chunk, nthreads=8)
        else:
            w_idx, w_val, w_sc = oracle.compress(g.cpu().numpy(), r_h, off, ratio, bits, chunk, nthreads=8)
        k_b, K, vb, ns = oracle.layout(off, ratio, bits, chunk)
        got = (idx.cpu().numpy().view(np.uint32)[:K], val.cpu().numpy()[:vb], sc.cpu().numpy()[:ns])
        compare_payload(off, ratio, bits, chunk, got, (w_idx, w_val, w_sc))
        assert np.array_equal(r.cpu().numpy().view(np.uint32), r_h.view(np.uint32)), "residual differs"
        w_dense = oracle.decompress(w_idx, w_val, w_sc, n, off, ratio, bits, chunk, nthreads=8)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), w_dense.view(np.uint32)), "dense differs"


@pytest.mark.parametrize("seed", range(100, 118))
def test_random_configuration(seed, monkeypatch):
    _case(seed, False, monkeypatch)


@pytest.mark.parametrize("seed", range(200, 212))
def test_random_configuration_pruned(seed, monkeypatch):
    _case(seed, True, monkeypatch)
