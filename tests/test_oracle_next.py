"""Pins for the oracle's two companion functions: the gradient L2 norm used by the density test
of Algorithm 2 Step 1 and the receiver-side accumulation of payloads."""
import math

import numpy as np

import oracle

F32 = np.float32


def test_l2norm_closed_forms():
    g = np.array([3.0, 4.0, 0.0, -12.0, 5.0], dtype=F32)
    tot, per = oracle.l2norm(g, [0, 2, 2, 5])
    assert per.tolist() == [5.0, 0.0, 13.0]
    assert tot == math.sqrt(25.0 + 169.0)
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100_000) * 1e-3).astype(F32)
    tot, per = oracle.l2norm(x, [0, 100_000])
    assert abs(tot - math.sqrt(math.fsum((x.astype(np.float64) ** 2).tolist()))) <= 1e-12 * tot
    assert abs(tot - np.linalg.norm(x.astype(np.float64))) <= 1e-12 * tot


def test_accumulate_sums_payloads_of_several_workers():
    """Each call adds exactly one worker's sparse gradient; elements nobody sent stay untouched."""
    n, off, ratio = 6000, [0, 1000, 1000, 6000], 0.05
    rng = np.random.default_rng(3)
    dense = np.full(n, 0.25, dtype=F32)
    want = dense.astype(np.float64).copy()
    touched = np.zeros(n, bool)
    for w in range(3):
        g = (rng.standard_normal(n) * 1e-2).astype(F32)
        for bits in (8, 4, 16, 32):
            idx, val, sc = oracle.compress(g, np.zeros(n, F32), off, ratio, bits, 64)
            d = oracle.decompress(idx, val, sc, n, off, ratio, bits, 64)
            before = dense.copy()
            oracle.decompress_accumulate(idx, val, sc, dense, off, ratio, bits, 64)
            assert np.array_equal(dense, (before + d).astype(F32))
            sent = np.zeros(n, bool)
            k_b, K, _, _ = oracle.layout(off, ratio, bits, 64)
            p = 0
            for b in range(3):
                sent[off[b] + idx[p:p + int(k_b[b])].astype(np.int64)] = True
                p += int(k_b[b])
            assert np.array_equal(dense[~sent].view(np.uint32), before[~sent].view(np.uint32))
            touched |= sent
            want += d
    assert np.allclose(dense, want, rtol=0, atol=1e-6)
    assert np.all(dense[~touched] == F32(0.25))
