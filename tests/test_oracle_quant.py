"""Pins for the oracle's value coding: per-chunk absmax int8 / int4 codes, nibble packing,
the binary16 cast (the paper's own quantizer, Sec. 4.2 Step 1) and decompression."""
import numpy as np
import pytest

import oracle

F32 = np.float32


def _case(seed, n=20000, ratio=0.3, sigma=1e-3):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * sigma).astype(F32)
    res = (rng.standard_normal(n) * sigma * 0.5).astype(F32)
    return g, res


@pytest.mark.parametrize("bits,qmax", [(8, 127), (4, 7)])
@pytest.mark.parametrize("chunk", [2048, 64, 7])
def test_quantizer_properties(bits, qmax, chunk):
    g, res = _case(bits * 10 + chunk)
    acc = (g + res).astype(F32)
    r = res.copy()
    idx, val, scales = oracle.compress(g, r, [0, len(g)], 0.3, bits, chunk)
    k = len(idx)
    v = acc[idx]
    q = oracle.unpack_codes(val, k, bits)
    assert len(scales) == -(-k // chunk)
    assert q.min() >= -qmax and q.max() <= qmax
    for c in range(len(scales)):
        sl = slice(c * chunk, min(k, (c + 1) * chunk))
        m = np.abs(v[sl]).max()
        # scale is the correctly rounded quotient absmax / qmax
        assert scales[c] == F32(m) / F32(qmax)
        exact = float(m) / qmax
        assert abs(float(scales[c]) - exact) <= exact * 2.0 ** -24
        # the absmax element gets the extreme code
        j = np.argmax(np.abs(v[sl]))
        assert abs(q[sl][j]) == qmax and np.sign(q[sl][j]) == np.sign(v[sl][j])
        # rounding error at most half a step (plus the rounding of the quotient itself)
        deq = q[sl].astype(np.float64) * float(scales[c])
        err = np.abs(v[sl].astype(np.float64) - deq)
        assert err.max() <= 0.5 * float(scales[c]) * (1 + 2.0 ** -20)
        # codes are the nearest integer of v / scale evaluated in binary32
        t = (v[sl] / scales[c]).astype(F32)
        assert np.array_equal(q[sl], np.clip(np.rint(t), -qmax, qmax).astype(np.int32))


def test_round_half_even_and_all_codes_int4():
    # values chosen so that v/scale lands exactly on k and on k + 0.5 (scale = 1 exactly)
    v = np.array([7, -7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3, -4, 5, -6, 6.5, -6.5, 0, 1],
                 dtype=F32)
    idx, val, sc = oracle.compress_bucket(v, np.zeros_like(v), 1.0, 4)
    assert sc.tolist() == [1.0]
    q = oracle.unpack_codes(val, len(v), 4)
    assert q.tolist() == [7, -7, 0, 2, 2, 0, -2, -2, 3, -4, 5, -6, 6, -6, 0, 1]
    # packing: even survivor in the low nibble, two's complement
    raw = val.view(np.uint8)
    assert raw[0] == ((7 & 0xF) | ((-7 & 0xF) << 4))
    assert raw[4] == ((3 & 0xF) | ((-4 & 0xF) << 4))


def test_nibble_roundtrip_all_15_codes_and_odd_tail():
    codes = list(range(-7, 8))
    v = np.array(codes, dtype=F32)          # absmax 7 -> scale 1
    idx, val, sc = oracle.compress_bucket(v, np.zeros_like(v), 1.0, 4)
    assert len(val) == 8 and (val[-1] >> 4) == 0      # odd tail: high nibble zero
    assert oracle.unpack_codes(val, 15, 4).tolist() == codes
    d = oracle.decompress(idx, val, sc, 15, [0, 15], 1.0, 4)
    assert d.tolist() == [float(c) for c in codes]


def test_int8_exact_grid():
    codes = np.arange(-127, 128, dtype=np.int32)
    v = codes.astype(F32)
    idx, val, sc = oracle.compress_bucket(v, np.zeros_like(v), 1.0, 8)
    assert sc.tolist() == [1.0]
    assert np.array_equal(oracle.unpack_codes(val, 255, 8), codes)


def test_all_zero_chunk_has_zero_scale():
    g = np.zeros(5000, F32)
    g[:10] = 1.0
    r = np.zeros_like(g)
    idx, val, sc = oracle.compress(g, r, [0, 5000], 1.0, 8, 2048)
    assert sc[0] != 0 and sc[1] == 0.0 and sc[2] == 0.0
    assert not np.any(oracle.unpack_codes(val, 5000, 8)[2048:])
    d = oracle.decompress(idx, val, sc, 5000, [0, 5000], 1.0, 8, 2048)
    assert np.all(d[2048:] == 0) and not np.any(np.signbit(d[2048:]))


def test_fp16_matches_numpy_cast():
    rng = np.random.default_rng(3)
    xs = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.9, 65520.0, 1e5, -1e5, 2.0 ** -24, 2.0 ** -25,
          2.0 ** -25 * 1.0001, 2.0 ** -26, 2.0 ** -14, 2.0 ** -14 * 0.999, 6.1e-5, 5.96e-8,
          1.0 + 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5]
    xs += list((rng.standard_normal(4000) * 10.0 ** rng.uniform(-9, 5, 4000)))
    # every half bit pattern's exact value and the midpoints between neighbours
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = (h[:-1] + h[1:]) / 2
    xs += list(h[::37]) + list(mids[::41]) + list(-mids[::43])
    with np.errstate(over="ignore"):
        for x in xs:
            x32 = F32(x)
            want = np.array([x32]).astype(np.float16).view(np.uint16)[0]
            got = oracle.f32_to_f16_bits(float(x32))
            assert got == want, (x, hex(got), hex(want))
    for hb in list(range(0, 0x7C01, 13)) + [0x8000, 0x8001, 0xFBFF, 0xFC00, 0x03FF, 0x0400]:
        want = np.array([hb], dtype=np.uint16).view(np.float16).astype(F32)[0]
        assert F32(oracle.f16_bits_to_f32(hb)).view(np.uint32) == want.view(np.uint32)


def test_fp16_payload():
    g, res = _case(99, n=5000)
    acc = (g + res).astype(F32)
    r = res.copy()
    idx, val, sc = oracle.compress(g, r, [0, 5000], 0.2, 16)
    assert len(sc) == 0 and len(val) == 2 * len(idx)       # half the bytes of fp32 values
    h = val.view(np.float16)
    assert np.array_equal(h.view(np.uint16), acc[idx].astype(np.float16).view(np.uint16))
    d = oracle.decompress(idx, val, sc, 5000, [0, 5000], 0.2, 16)
    assert np.array_equal(d[idx], h.astype(F32))


@pytest.mark.parametrize("bits", [4, 8, 16, 32])
def test_decompress_places_values_and_zeros(bits):
    g, res = _case(bits, n=9000)
    r = res.copy()
    off = [0, 100, 100, 4000, 9000]          # includes an empty bucket
    idx, val, sc = oracle.compress(g, r, off, 0.05, bits, 512)
    d = oracle.decompress(idx, val, sc, 9000, off, 0.05, bits, 512)
    k_b, K, vb, ns = oracle.layout(off, 0.05, bits, 512)
    assert k_b.tolist() == [5, 0, 195, 250] and K == 450
    mask = np.zeros(9000, bool)
    p = 0
    for b in range(4):
        mask[off[b] + idx[p:p + int(k_b[b])].astype(np.int64)] = True
        p += int(k_b[b])
    assert mask.sum() == K
    assert np.all(d[~mask] == 0) and not np.any(np.signbit(d[~mask]))
