"""CPU oracle for the NetSenseML gradient data-reduction path -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP package and the
HIP package never imports it.

``nsml_oracle.c`` states Algorithm 2 Step 3 (top-k by magnitude with local
accumulation of what is filtered out, Sec. 4.2 Step 3) as a full sort, plus the
value coding / payload / inverse scatter of the build contract.
``controller.py`` states Algorithm 1 and Eq. (1)-(3) in Python floats.

This module is argument marshalling for the C file (numpy arrays in, numpy
arrays out) and the gcc build line.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

from .controller import CtlParams, CtlState, choose_ratio, ctl_init  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nsml_oracle.c")
_LIB = os.path.join(_HERE, "libnsml_oracle.so")
_lock = threading.Lock()
_lib = None

GCC_FLAGS = ["-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
             "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile nsml_oracle.c with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    with _lock:
        if _lib is None:
            build()
            L = C.CDLL(_LIB)
            u64, u32, i32, dbl, vp = C.c_uint64, C.c_uint32, C.c_int, C.c_double, C.c_void_p
            L.orc_k.restype = u64
            L.orc_k.argtypes = [dbl, u64]
            L.orc_layout.restype = i32
            L.orc_layout.argtypes = [vp, u32, dbl, i32, u32, vp, vp, vp, vp]
            L.orc_compress_bucket.restype = C.c_int64
            L.orc_compress_bucket.argtypes = [vp, vp, u64, dbl, i32, u32, vp, vp, vp]
            L.orc_decompress_bucket.restype = i32
            L.orc_decompress_bucket.argtypes = [vp, vp, vp, u64, u64, i32, u32, vp]
            L.orc_compress.restype = i32
            L.orc_compress.argtypes = [vp, vp, u64, vp, u32, dbl, i32, u32, vp, vp, vp, i32]
            L.orc_decompress.restype = i32
            L.orc_decompress.argtypes = [vp, vp, vp, u64, vp, u32, dbl, i32, u32, vp, i32]
            L.orc_pruned_count.restype = u64
            L.orc_pruned_count.argtypes = [dbl, u64]
            L.orc_keep_mask.restype = i32
            L.orc_keep_mask.argtypes = [vp, u64, dbl, vp]
            L.orc_compress_pruned.restype = i32
            L.orc_compress_pruned.argtypes = [vp, vp, vp, u64, vp, u32, dbl, i32, u32, vp, vp, vp, i32]
            L.orc_decompress_accumulate.restype = i32
            L.orc_decompress_accumulate.argtypes = [vp, vp, vp, u64, vp, u32, dbl, i32, u32, vp]
            L.orc_l2norm.restype = dbl
            L.orc_l2norm.argtypes = [vp, vp, u32, vp]
            L.orc_f32_to_f16.restype = C.c_uint16
            L.orc_f32_to_f16.argtypes = [C.c_float]
            L.orc_f16_to_f32.restype = C.c_float
            L.orc_f16_to_f32.argtypes = [C.c_uint16]
            _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def k_of(ratio: float, n: int) -> int:
    return int(lib().orc_k(float(ratio), int(n)))


def layout(bucket_off, ratio: float, bits: int, chunk: int = 2048):
    """-> (k_b uint64[B], K, val_bytes, n_scales)."""
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    B = len(off) - 1
    k_b = np.zeros(B, dtype=np.uint64)
    K, vb, ns = C.c_uint64(), C.c_uint64(), C.c_uint64()
    rc = lib().orc_layout(_p(off), B, float(ratio), int(bits), int(chunk), _p(k_b),
                          C.addressof(K), C.addressof(vb), C.addressof(ns))
    if rc != 0:
        raise ValueError("orc_layout rc=%d" % rc)
    return k_b, int(K.value), int(vb.value), int(ns.value)


def compress(grad, residual, bucket_off, ratio: float, bits: int, chunk: int = 2048,
             nthreads: int = 1):
    """Compress a bucketed gradient.  ``residual`` (float32, contiguous) is updated in
    place.  -> (idx uint32[K], val uint8[val_bytes], scales float32[n_scales])."""
    g = np.ascontiguousarray(grad, dtype=np.float32)
    if not (isinstance(residual, np.ndarray) and residual.dtype == np.float32
            and residual.flags.c_contiguous and residual.shape == g.shape):
        raise ValueError("residual must be a contiguous float32 array shaped like grad")
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    B = len(off) - 1
    _, K, vb, ns = layout(off, ratio, bits, chunk)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(vb, dtype=np.uint8)
    scales = np.zeros(ns, dtype=np.float32)
    rc = lib().orc_compress(_p(g), _p(residual), g.size, _p(off), B, float(ratio), int(bits),
                            int(chunk), _p(idx), _p(val), _p(scales), int(nthreads))
    if rc != 0:
        raise ValueError("orc_compress rc=%d" % rc)
    return idx, val, scales


def decompress(idx, val, scales, n: int, bucket_off, ratio: float, bits: int, chunk: int = 2048,
               nthreads: int = 1):
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    B = len(off) - 1
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    val = np.ascontiguousarray(val).view(np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    dense = np.empty(int(n), dtype=np.float32)
    rc = lib().orc_decompress(_p(idx), _p(val), _p(scales), int(n), _p(off), B, float(ratio),
                              int(bits), int(chunk), _p(dense), int(nthreads))
    if rc != 0:
        raise ValueError("orc_decompress rc=%d" % rc)
    return dense


def pruned_count(ratio: float, n: int) -> int:
    return int(lib().orc_pruned_count(float(ratio), int(n)))


def keep_mask(weights, ratio: float):
    """One bucket: boolean array, True for the parameters the pruning step keeps."""
    w = np.ascontiguousarray(weights, dtype=np.float32)
    m = np.zeros(w.size, dtype=np.uint8)
    rc = lib().orc_keep_mask(_p(w), w.size, float(ratio), _p(m))
    if rc != 0:
        raise ValueError("orc_keep_mask rc=%d" % rc)
    return m.astype(bool)


def compress_pruned(grad, residual, weights, bucket_off, ratio: float, bits: int,
                    chunk: int = 2048, nthreads: int = 1):
    """As compress, with Algorithm 2 Step 2: only parameters kept by weight-magnitude pruning
    can be selected.  ``residual`` is updated in place."""
    g = np.ascontiguousarray(grad, dtype=np.float32)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    if not (isinstance(residual, np.ndarray) and residual.dtype == np.float32
            and residual.flags.c_contiguous and residual.shape == g.shape and w.shape == g.shape):
        raise ValueError("residual / weights must be contiguous float32 arrays shaped like grad")
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    B = len(off) - 1
    _, K, vb, ns = layout(off, ratio, bits, chunk)
    idx = np.zeros(K, dtype=np.uint32)
    val = np.zeros(vb, dtype=np.uint8)
    scales = np.zeros(ns, dtype=np.float32)
    rc = lib().orc_compress_pruned(_p(g), _p(residual), _p(w), g.size, _p(off), B, float(ratio),
                                   int(bits), int(chunk), _p(idx), _p(val), _p(scales), int(nthreads))
    if rc != 0:
        raise ValueError("orc_compress_pruned rc=%d" % rc)
    return idx, val, scales


def decompress_accumulate(idx, val, scales, dense, bucket_off, ratio: float, bits: int,
                          chunk: int = 2048):
    """dense[off_b + idx[j]] += decoded value j, in place (dense: contiguous float32)."""
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    val = np.ascontiguousarray(val).view(np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    assert dense.dtype == np.float32 and dense.flags.c_contiguous
    rc = lib().orc_decompress_accumulate(_p(idx), _p(val), _p(scales), dense.size, _p(off),
                                         len(off) - 1, float(ratio), int(bits), int(chunk), _p(dense))
    if rc != 0:
        raise ValueError("orc_decompress_accumulate rc=%d" % rc)
    return dense


def l2norm(grad, bucket_off):
    """-> (norm of the whole gradient, per-bucket norms), accumulated in double."""
    g = np.ascontiguousarray(grad, dtype=np.float32)
    off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
    per = np.zeros(len(off) - 1, dtype=np.float64)
    tot = lib().orc_l2norm(_p(g), _p(off), len(off) - 1, _p(per))
    return float(tot), per


def compress_bucket(grad, residual, ratio: float, bits: int, chunk: int = 2048):
    """Single bucket convenience: -> (idx, val, scales); residual updated in place."""
    n = int(np.asarray(grad).size)
    return compress(grad, residual, [0, n], ratio, bits, chunk)


def f32_to_f16_bits(x: float) -> int:
    return int(lib().orc_f32_to_f16(C.c_float(x)))


def f16_bits_to_f32(h: int) -> float:
    return float(lib().orc_f16_to_f32(C.c_uint16(h)))


def unpack_codes(val, k: int, bits: int):
    """Payload value bytes of ONE bucket -> int codes (bits 8/4), float16 (16), float32 (32)."""
    raw = np.ascontiguousarray(val).view(np.uint8)
    if bits == 32:
        return raw[:4 * k].view(np.float32).copy()
    if bits == 16:
        return raw[:2 * k].view(np.float16).copy()
    if bits == 8:
        return raw[:k].view(np.int8).astype(np.int32)
    lo = (raw & 0xF).astype(np.int32)
    hi = (raw >> 4).astype(np.int32)
    q = np.empty(2 * len(raw), dtype=np.int32)
    q[0::2], q[1::2] = lo, hi
    q = np.where(q >= 8, q - 16, q)
    return q[:k]
