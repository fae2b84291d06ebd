"""Invariants the build contract fixes for the whole compress/decompress round trip."""
import numpy as np
import pytest

import oracle

F32 = np.float32


def _data(seed, n, sigma=1e-3):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * sigma).astype(F32)
    res = (rng.standard_normal(n) * sigma).astype(F32)
    return g, res


def test_identity_ratio1_bits32():
    g, res = _data(0, 10000)
    acc = (g + res).astype(F32)
    r = res.copy()
    idx, val, sc = oracle.compress_bucket(g, r, 1.0, 32)
    assert np.array_equal(idx, np.arange(10000, dtype=np.uint32))
    assert np.array_equal(val.view(F32).view(np.uint32), acc.view(np.uint32))
    assert len(sc) == 0
    assert np.all(r == 0)
    d = oracle.decompress(idx, val, sc, 10000, [0, 10000], 1.0, 32)
    assert np.array_equal(d.view(np.uint32), acc.view(np.uint32))


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
@pytest.mark.parametrize("ratio", [0.001, 0.05, 0.6])
def test_error_feedback_conservation(bits, ratio):
    """decompressed + new residual == grad + old residual, exactly, element by element."""
    g, res = _data(bits * 7 + int(ratio * 1000), 50000)
    g[::5] = 0
    res[::10] = 0                       # some exact zeros in the accumulator
    acc = (g + res).astype(F32)
    r = res.copy()
    off = [0, 17, 30000, 50000]
    idx, val, sc = oracle.compress(g, r, off, ratio, bits, 2048)
    d = oracle.decompress(idx, val, sc, 50000, off, ratio, bits, 2048)
    assert np.array_equal((d + r).astype(F32), acc)
    # and what is not sent stays, untouched, in the residual
    sent = d != 0
    assert np.array_equal(r[~sent & (acc != 0)], acc[~sent & (acc != 0)])


def test_batched_equals_loop_of_single_buckets():
    g, res = _data(4, 30000)
    off = [0, 1, 65, 2113, 2113, 20000, 30000]
    for bits in (4, 8, 16, 32):
        r_b = res.copy()
        idx, val, sc = oracle.compress(g, r_b, off, 0.07, bits, 256, nthreads=3)
        k_b, K, vb, ns = oracle.layout(off, 0.07, bits, 256)
        r_s = res.copy()
        I, V, S = [], [], []
        for b in range(len(off) - 1):
            lo, hi = off[b], off[b + 1]
            if hi == lo:
                continue
            rs = r_s[lo:hi].copy()
            i, v, s = oracle.compress_bucket(g[lo:hi], rs, 0.07, bits, 256)
            r_s[lo:hi] = rs
            I.append(i), V.append(v), S.append(s)
        assert np.array_equal(idx, np.concatenate(I))
        assert np.array_equal(val, np.concatenate(V))
        assert np.array_equal(sc, np.concatenate(S))
        assert np.array_equal(r_b.view(np.uint32), r_s.view(np.uint32))
        assert len(idx) == K and len(val) == vb and len(sc) == ns


def test_multi_step_error_feedback():
    """Carried residual: the step-wise conservation law holds at every step and every element
    is eventually sent (nothing is lost for good)."""
    n = 4096
    rng = np.random.default_rng(8)
    r = np.zeros(n, F32)
    total_sent = np.zeros(n, np.float64)
    total_g = np.zeros(n, np.float64)
    ever = np.zeros(n, bool)
    for step in range(40):
        g = (rng.standard_normal(n) * 1e-3).astype(F32)
        acc = (g + r).astype(F32)
        idx, val, sc = oracle.compress_bucket(g, r, 0.1, 8)
        d = oracle.decompress(idx, val, sc, n, [0, n], 0.1, 8)
        assert np.array_equal((d + r).astype(F32), acc)
        ever[idx] = True
        total_sent += d
        total_g += g
    assert np.allclose(total_sent + r, total_g, rtol=0, atol=1e-6)
    assert ever.mean() > 0.95


def test_threads_do_not_change_bytes():
    g, res = _data(12, 40000)
    off = np.linspace(0, 40000, 33).astype(np.uint64)
    outs = []
    for t in (1, 4):
        r = res.copy()
        outs.append(oracle.compress(g, r, off, 0.02, 4, 128, nthreads=t) + (r,))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_bad_arguments():
    g = np.zeros(8, F32)
    with pytest.raises(ValueError):
        oracle.compress(g, g.copy(), [0, 8], 0.0, 8)
    with pytest.raises(ValueError):
        oracle.compress(g, g.copy(), [0, 8], 1.5, 8)
    with pytest.raises(ValueError):
        oracle.compress(g, g.copy(), [0, 8], 0.5, 5)
    with pytest.raises(ValueError):
        oracle.compress(g, g.copy(), [0, 7], 0.5, 8)
