"""nsml_decompress_static, the entry point for callers that cannot allocate, against
nsml_decompress (which is itself checked against the oracle elsewhere): same payload in, the
same dense gradient out, bit for bit, on two calls in a row, the second with a smaller input
(the static tables keep the first call's contents and must not leak into the second)."""
import numpy as np
import pytest
import torch

from paper_2506_16235_amd import binding as nsml
from paper_2506_16235_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _payload(sizes, ratio, bits, chunk, seed):
    off = W.offsets_of(sizes)
    n = int(off[-1])
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    g = torch.randn(n, generator=gen, device=DEV) * 1e-3
    r = torch.zeros_like(g)
    ctx = nsml.Context(n, len(sizes), chunk)
    idx, val, sc = ctx.compress(g, r, off, ratio, bits)
    want = ctx.decompress(idx, val, sc, n, off, ratio, bits)
    torch.cuda.synchronize()
    return off, n, idx, val, sc, want


@pytest.mark.parametrize("bits", [8, 4, 16, 32])
def test_static_decompress_matches_context_decompress_twice(bits):
    big = [300_001, 0, 4_097, 1, 1_200_000, 65_536, 777]
    small = [5_003, 130_000, 3]
    first = _payload(big, 0.02, bits, 2048, 11 + bits)
    second = _payload(small, 0.3, bits, 64, 12 + bits)
    for off, n, idx, val, sc, want in (first, second):
        chunk = 2048 if n > 200_000 else 64
        ratio = 0.02 if n > 200_000 else 0.3
        out = torch.full((n + 64,), 7.0, dtype=torch.float32, device=DEV)      # sentinels after the end
        nsml.decompress_static(idx, val, sc if bits <= 8 else None, n, off, ratio, bits, chunk, out=out[:n])
        torch.cuda.synchronize()
        assert torch.equal(out[:n].view(torch.int32), want.view(torch.int32))
        assert bool((out[n:] == 7.0).all())


def test_static_decompress_rejects_what_it_cannot_hold():
    lib = nsml.raw()
    off = np.array([0, 1 << 29], dtype=np.uint64)             # beyond NSML_STATIC_MAX_N
    dummy = torch.zeros(16, dtype=torch.int32, device=DEV)
    rc = lib.nsml_decompress_static(dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), 1 << 29,
                                    off.ctypes.data, 1, 0.5, 8, 2048, dummy.data_ptr(), None)
    assert rc == nsml.ECAP
    many = np.arange(0, 322, dtype=np.uint64) * 10            # 321 buckets
    rc = lib.nsml_decompress_static(dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), int(many[-1]),
                                    many.ctypes.data, 321, 0.5, 8, 2048, dummy.data_ptr(), None)
    assert rc == nsml.ECAP
    ok = np.array([0, 100], dtype=np.uint64)
    rc = lib.nsml_decompress_static(dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), 100,
                                    ok.ctypes.data, 1, 0.0, 8, 2048, dummy.data_ptr(), None)
    assert rc == nsml.EINVAL
