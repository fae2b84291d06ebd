"""Pins for the oracle's pruned variant (Algorithm 2 Step 2: pruning_rate = 0.5 * (1 - ratio),
smallest |weight| pruned, their gradients excluded from the sparsification that follows)."""
import numpy as np
import pytest

import oracle

F32 = np.float32


def _keys(a):
    return np.ascontiguousarray(a, dtype=F32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def _beats(key):
    """beats[i, j]: j comes before i in (magnitude descending, index ascending) order."""
    key = key.astype(np.int64)
    n = len(key)
    ii, jj = np.arange(n)[:, None], np.arange(n)[None, :]
    return (key[None, :] > key[:, None]) | ((key[None, :] == key[:, None]) & (jj < ii))


def test_pruning_rate_values():
    # Sec. 4.2 Step 2: rate = 0.5 * (1 - ratio): nothing pruned at ratio 1, 49.5 % at ratio 0.01
    assert oracle.pruned_count(1.0, 1000) == 0
    assert oracle.pruned_count(0.01, 1000) == 495
    assert oracle.pruned_count(0.5, 1001) == 250          # floor(0.25 * 1001)
    assert oracle.pruned_count(0.001, 3) == 1             # floor(1.4985)
    assert oracle.pruned_count(0.3, 1) == 0


@pytest.mark.parametrize("seed", range(5))
def test_rank_definitions(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 900))
    w = (rng.integers(-6, 7, size=n) * 0.5).astype(F32)          # many equal |w|
    a = (rng.integers(-9, 10, size=n) * 0.25).astype(F32)
    for ratio in (0.01, 0.2, 0.6, 1.0):
        keep = oracle.keep_mask(w, ratio)
        m = n - oracle.pruned_count(ratio, n)
        # kept = fewer than m parameters beat it in |w|
        assert np.array_equal(keep, _beats(_keys(w)).sum(1) < m)
        r = np.zeros(n, F32)
        idx, val, _ = oracle.compress_pruned(a, r, w, [0, n], ratio, 32)
        k = oracle.k_of(ratio, n)
        # survivor = kept, and fewer than k KEPT parameters beat it in |a|
        beats_kept = (_beats(_keys(a)) & keep[None, :]).sum(1)
        want = np.nonzero(keep & (beats_kept < k))[0].astype(np.uint32)
        assert np.array_equal(idx, want) and len(idx) == k
        assert np.array_equal(val.view(F32), a[idx])
        # pruned parameters keep their accumulated gradient for later steps
        assert np.array_equal(r[~keep], a[~keep])


def test_ratio_one_equals_unpruned_path():
    rng = np.random.default_rng(9)
    n = 5000
    g = rng.standard_normal(n).astype(F32)
    w = rng.standard_normal(n).astype(F32)
    for bits in (4, 8, 16, 32):
        r1, r2 = np.zeros(n, F32), np.zeros(n, F32)
        a = oracle.compress(g, r1, [0, n], 1.0, bits, 64)
        b = oracle.compress_pruned(g, r2, w, [0, n], 1.0, bits, 64)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
        assert np.array_equal(r1, r2)


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_pruned_payload_is_the_plain_coding_of_the_survivors(bits):
    """Conservation law and batching hold exactly as for the unpruned path."""
    rng = np.random.default_rng(bits)
    n, off = 20000, [0, 3, 9000, 9000, 20000]
    g = (rng.standard_normal(n) * 1e-3).astype(F32)
    res = (rng.standard_normal(n) * 1e-3).astype(F32)
    w = rng.standard_normal(n).astype(F32)
    acc = (g + res).astype(F32)
    r = res.copy()
    idx, val, sc = oracle.compress_pruned(g, r, w, off, 0.05, bits, 256, nthreads=2)
    d = oracle.decompress(idx, val, sc, n, off, 0.05, bits, 256)
    assert np.array_equal((d + r).astype(F32), acc)
    k_b, K, vb, ns = oracle.layout(off, 0.05, bits, 256)
    assert (len(idx), len(val), len(sc)) == (K, vb, ns)
    p = 0
    for b in range(4):
        lo, hi = off[b], off[b + 1]
        kb = int(k_b[b])
        if hi > lo:
            keep = oracle.keep_mask(w[lo:hi], 0.05)
            assert np.all(keep[idx[p:p + kb]])
        p += kb
