"""Pins for the oracle's selection step (Algorithm 2 Step 3: top-k by magnitude; ties go to
the lower index; exactly k survivors).  None of these re-uses the oracle's sort."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _keys(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def _rank_definition(a, k):
    """Element i survives iff fewer than k elements beat it, where j beats i when
    |a_j| > |a_i|, or |a_j| == |a_i| and j < i.  O(n^2), no sorting."""
    key = _keys(a).astype(np.int64)
    n = len(key)
    gt = key[None, :] > key[:, None]
    eq_before = (key[None, :] == key[:, None]) & (np.arange(n)[None, :] < np.arange(n)[:, None])
    rank = gt.sum(1) + eq_before.sum(1)
    return np.nonzero(rank < k)[0].astype(np.uint32)


def test_k_golden():
    for line in open(os.path.join(GOLD, "k_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, ratio, k = line.split()
        assert oracle.k_of(float(ratio), int(n)) == int(k), line


def test_hand_example():
    rows = {}
    for line in open(os.path.join(GOLD, "hand_example_int8.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, rest = line.split(":")
        rows[name.strip()] = rest.split()
    g = np.array(rows["grad"], dtype=np.float32)
    r = np.zeros_like(g)
    idx, val, sc = oracle.compress_bucket(g, r, float(rows["ratio"][0]), int(rows["bits"][0]))
    assert idx.tolist() == [int(x) for x in rows["idx"]]
    assert val.view(np.int8).tolist() == [int(x) for x in rows["codes"]]
    assert sc.tolist() == [np.float32(1.0) / np.float32(127.0)]
    g2 = np.array(rows["grad2"], dtype=np.float32)
    idx2, _, _ = oracle.compress_bucket(g2, np.zeros_like(g2), float(rows["ratio2"][0]), 32)
    assert idx2.tolist() == [int(x) for x in rows["idx2"]]


@pytest.mark.parametrize("seed", range(6))
def test_rank_definition_random(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 1500))
    # few distinct magnitudes => many ties, both signs, zeros of both signs
    levels = rng.integers(2, 40)
    a = (rng.integers(-levels, levels + 1, size=n) * 0.125).astype(np.float32)
    a[rng.random(n) < 0.1] = -0.0
    res = (rng.integers(-2, 3, size=n) * 0.125).astype(np.float32)
    g = (a - res).astype(np.float32)
    for ratio in (0.001, 0.03, 0.5, 0.97, 1.0):
        r = res.copy()
        idx, val, _ = oracle.compress_bucket(g, r, ratio, 32)
        acc = (g + res).astype(np.float32)
        k = oracle.k_of(ratio, n)
        assert len(idx) == k
        assert np.array_equal(idx, _rank_definition(acc, k))
        assert np.array_equal(val.view(np.float32).view(np.uint32), acc[idx].view(np.uint32))


def test_exhaustive_tie_patterns():
    """Every vector of length <= 6 over {+0, -0, 1, -1, 2} and every k."""
    alphabet = np.array([0.0, -0.0, 1.0, -1.0, 2.0], dtype=np.float32)
    for n in range(1, 7):
        ks = sorted(set(range(1, n + 1)))
        for combo in itertools.product(range(5), repeat=n):
            a = alphabet[list(combo)]
            for k in ks:
                ratio = k / n
                if oracle.k_of(ratio, n) != k:       # rounding of k/n*n above k: skip
                    continue
                idx, _, _ = oracle.compress_bucket(a, np.zeros(n, np.float32), ratio, 32)
                assert np.array_equal(idx, _rank_definition(a, k)), (a, k)


def test_matches_numpy_stable_sort():
    rng = np.random.default_rng(11)
    n = 4096
    a = rng.standard_normal(n).astype(np.float32)
    a[7::7] = -a[6::7][: len(a[7::7])]       # planted duplicate magnitudes
    for ratio in (0.01, 0.1, 0.9):
        k = oracle.k_of(ratio, n)
        order = np.argsort(-(_keys(a).astype(np.int64)), kind="stable")
        want = np.sort(order[:k]).astype(np.uint32)
        idx, _, _ = oracle.compress_bucket(a, np.zeros(n, np.float32), ratio, 32)
        assert np.array_equal(idx, want)


def test_separation_invariant_large():
    rng = np.random.default_rng(5)
    n = 200_000
    a = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    a[rng.random(n) < 0.3] = 0.0
    a = np.round(a, 4).astype(np.float32)      # ties everywhere
    for ratio in (0.0005, 0.01, 0.1, 0.75):
        idx, _, _ = oracle.compress_bucket(a, np.zeros(n, np.float32), ratio, 32)
        k = oracle.k_of(ratio, n)
        assert len(idx) == k and np.all(np.diff(idx.astype(np.int64)) > 0)
        key = _keys(a)
        inside = np.zeros(n, bool)
        inside[idx] = True
        t = key[inside].min()
        assert key[~inside].max(initial=0) <= t
        # among elements equal to the threshold, the chosen ones are exactly the lowest indices
        eq = np.nonzero(key == t)[0]
        chosen = inside[eq]
        assert np.all(chosen[: chosen.sum()]) and not np.any(chosen[chosen.sum():])


def test_zeros_are_selected_to_reach_k():
    a = np.zeros(100, np.float32)
    a[[5, 50]] = [1.0, -2.0]
    idx, val, _ = oracle.compress_bucket(a, np.zeros(100, np.float32), 0.1, 32)
    assert idx.tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 8, 50]
