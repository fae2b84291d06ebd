"""GPU parity for the pruned variant (Algorithm 2 Step 2 + Step 3) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_16235_amd import binding as nsml
from paper_2506_16235_amd import workloads as W
from gpu_util import DEV, compare_payload

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "dense", "miss"])
def path(request, monkeypatch):
    """auto: the paths the library picks; dense: every bucket through the dense passes; miss: the
    staged band of weight magnitudes is put beside the threshold on purpose, so every bucket takes
    the repeat of the weight pass."""
    monkeypatch.setitem(nsml.Context.default_options, "force_dense", 1 if request.param == "dense" else 0)
    monkeypatch.setitem(nsml.Context.default_options, "wband_miss", 1 if request.param == "miss" else 0)
    return request.param


def _rand(n, seed, sigma=1e-3):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return torch.randn(n, generator=g, device=DEV) * sigma


def _run(sizes, ratio, bits, chunk, steps=2, ties=False, seed=0, stats=None, drift=None):
    off = W.offsets_of(sizes)
    n = int(off[-1])
    ctx = nsml.Context(n, len(sizes), chunk)
    r = torch.zeros(n, device=DEV)
    r_h = np.zeros(n, dtype=np.float32)
    for step in range(steps):
        g = _rand(n, seed + 10 * step)
        if drift is None or step == 0:
            w = _rand(n, seed + 10 * step + 1, sigma=0.05)
        else:
            w = w + _rand(n, seed + 10 * step + 1, sigma=drift)      # an optimizer step's worth of change
        if ties == "few":
            w = (w * 20000).round() / 20000      # some hundred equal |w| at the threshold, of both signs
        elif ties:
            w = (w * 40).round() / 40            # many equal |w|, zeros included
            g = (g * 2e3).round() / 2e3
        idx, val, sc = ctx.compress_pruned(g, r, w, off, ratio, bits)
        dense = ctx.decompress(idx, val, sc, n, off, ratio, bits)
        torch.cuda.synchronize()
        ctx.path_stats()                         # raise if a device-side consistency check tripped
        ws = ctx.prune_stats()
        if stats is not None:
            stats.append(ws)
        w_idx, w_val, w_sc = oracle.compress_pruned(g.cpu().numpy(), r_h, w.cpu().numpy(), off, ratio,
                                                    bits, chunk, nthreads=8)
        k_b, K, vb, ns = oracle.layout(off, ratio, bits, chunk)
        got = (idx.cpu().numpy().view(np.uint32)[:K], val.cpu().numpy()[:vb], sc.cpu().numpy()[:ns])
        compare_payload(off, ratio, bits, chunk, got, (w_idx, w_val, w_sc))
        assert np.array_equal(r.cpu().numpy().view(np.uint32), r_h.view(np.uint32))
        w_dense = oracle.decompress(w_idx, w_val, w_sc, n, off, ratio, bits, chunk)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), w_dense.view(np.uint32))


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_ragged_buckets(bits):
    _run([1, 64, 2048, 0, 4095, 4097, 3, 17889, 8192, 12289, 1, 50001, 7, 131072 + 5], 0.05, bits, 64)


@pytest.mark.parametrize("ratio", [0.001, 0.01, 0.3, 1.0])
def test_ratios(ratio):
    _run([300_000, 17, 200_003], ratio, 8, 256)


def test_many_equal_weights_and_gradients():
    _run([100_000, 150_001, 49_999], 0.02, 4, 128, ties=True)
    _run([100_000, 150_001, 49_999], 0.4, 32, 128, ties=True, seed=5)


def test_equal_weights_at_the_threshold_decided_from_the_band(path):
    """Weights on a grid fine enough that the threshold's level-0 digit holds a few per cent of a
    bucket (so the weight stage works from the staged band, not the dense passes) and coarse enough
    that some hundred weights equal the threshold: which of them are kept is decided by index."""
    stats = []
    _run([300_000, 1_000_003, 70_000], 0.01, 8, 256, ties="few", seed=21, stats=stats)
    for band, dense in stats:
        assert (band, dense) == ((3, 0) if path == "auto" else (0, 3))


def test_weights_that_move_little_between_steps(path):
    """From the second step on the band of weight magnitudes is a narrow one around the threshold
    of the step before; with weights that drift by 1e-5 of their spread it holds the new threshold
    (the buckets are decided from the band), with weights replaced by new ones it misses and the
    weight pass is repeated: either way the result is the oracle's."""
    stats = []
    _run([300_000, 2_000_003, 70_000, 5], 0.01, 8, 256, steps=4, seed=77, stats=stats, drift=5e-7)
    if path == "auto":
        assert all(dense <= 1 for band, dense in stats[1:]), stats      # the 5-element bucket may go either way
    _run([300_000, 2_000_003, 70_000], 0.01, 4, 256, steps=3, seed=78, drift=1e-2)


def test_clustered_survivors_with_pruning():
    """Runs of large gradients longer than a staging segment holds, under pruning: the segments
    that overflow are read from the dense accumulator, minus the pruned parameters."""
    n0 = 1_200_000
    off = W.offsets_of([n0, 30_001])
    n = int(off[-1])
    ctx = nsml.Context(n, 2, 256)
    r = torch.zeros(n, device=DEV)
    r_h = np.zeros(n, dtype=np.float32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(909)
    for step, ratio in enumerate((0.05, 0.03)):
        g = W._laplace(n, 1e-6, gen, DEV)
        for start in range(5_000 + 911 * step, n0 - 4_000, 50_000):
            g[start:start + 3_500] = W._laplace(3_500, 1e-3, gen, DEV)
        w = _rand(n, 500 + step, sigma=0.05)
        idx, val, sc = ctx.compress_pruned(g, r, w, off, ratio, 8)
        torch.cuda.synchronize()
        ctx.path_stats()
        w_idx, w_val, w_sc = oracle.compress_pruned(g.cpu().numpy(), r_h, w.cpu().numpy(), off, ratio, 8, 256, nthreads=8)
        k_b, K, vb, ns = oracle.layout(off, ratio, 8, 256)
        got = (idx.cpu().numpy().view(np.uint32)[:K], val.cpu().numpy()[:vb], sc.cpu().numpy()[:ns])
        compare_payload(off, ratio, 8, 256, got, (w_idx, w_val, w_sc))
        assert np.array_equal(r.cpu().numpy().view(np.uint32), r_h.view(np.uint32))


def test_large_single_bucket():
    _run([5_000_000], 0.01, 8, 2048, steps=2)
