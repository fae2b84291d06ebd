"""ctypes binding of libnsml.so -- argument marshalling only.

Same names as the C ABI in include/nsml.h: ``choose_ratio`` (host), ``compress`` and
``decompress`` (GPU, enqueued on torch's current HIP stream), ``payload_layout``.  PyTorch is
used for device memory and streams; every step of the path runs in the library's kernels.
There is no fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnsml.so")

OK, EINVAL, ECAP, EHIP, ENOTIMPL, ENOMEM, EINTERNAL = 0, -1, -2, -3, -4, -5, -6
MAX_KERNELS = 32
CTL_MAX_WIN = 128

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2506_16235_amd.build` "
        "(hipcc, gfx950).  There is no CPU fallback for the GPU path.")

_lib = C.CDLL(LIB_PATH)


class CtlParams(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("alpha", "beta1", "beta2", "floor", "cap", "init", "bdp_frac", "rtt_excess",
                 "tr_q", "tr_q4", "tr_d")] + \
               [(n, C.c_int32) for n in ("startup_max", "win_bw", "win_rt", "quant_mode")]


class CtlState(C.Structure):
    _fields_ = [("p", CtlParams), ("ratio", C.c_double), ("btlbw", C.c_double),
                ("rtprop", C.c_double), ("bdp", C.c_double), ("all_max_ebb", C.c_double),
                ("all_min_rtt", C.c_double), ("ebb", C.c_double * CTL_MAX_WIN),
                ("rtt", C.c_double * CTL_MAX_WIN), ("count", C.c_int64), ("phase", C.c_int32),
                ("startup_steps", C.c_int32)]


_vp, _u64, _u32, _i32, _dbl = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int, C.c_double
_lib.nsml_strerror.restype = C.c_char_p
_lib.nsml_strerror.argtypes = [_i32]
_lib.nsml_ctl_default_params.argtypes = [C.POINTER(CtlParams)]
_lib.nsml_ctl_init.argtypes = [C.POINTER(CtlState), C.POINTER(CtlParams)]
_lib.nsml_choose_ratio.argtypes = [C.POINTER(CtlState), _dbl, _dbl, _dbl, _dbl,
                                   C.POINTER(_dbl), C.POINTER(_i32)]
_lib.nsml_payload_layout.argtypes = [_vp, _u32, _dbl, _i32, _u32, _vp, C.POINTER(_u64),
                                     C.POINTER(_u64), C.POINTER(_u64)]
_lib.nsml_create.argtypes = [C.POINTER(_vp), _i32, _u64, _u32, _u32]
_lib.nsml_create_ex.argtypes = [C.POINTER(_vp), _i32, _u64, _u32, _u32, _dbl]
_lib.nsml_create_ex.restype = _i32
_lib.nsml_set_option.argtypes = [_vp, C.c_char_p, _i32]
_lib.nsml_set_option.restype = _i32
_lib.nsml_decompress_static.argtypes = [_vp, _vp, _vp, _u64, _vp, _u32, _dbl, _i32, _u32, _vp, _vp]
_lib.nsml_decompress_static.restype = _i32
_lib.nsml_calibration_stream.argtypes = [_i32, _vp, _vp, _u64, _i32, _vp]
_lib.nsml_calibration_stream.restype = _i32
_lib.nsml_destroy.argtypes = [_vp]
_lib.nsml_last_hip_error.argtypes = [_vp]
_lib.nsml_workspace_bytes.argtypes = [_vp]
_lib.nsml_workspace_bytes.restype = _u64
_lib.nsml_compress.argtypes = [_vp, _vp, _vp, _u64, _vp, _u32, _dbl, _i32, _vp, _vp, _vp, _vp]
_lib.nsml_compress_pruned.argtypes = [_vp, _vp, _vp, _vp, _u64, _vp, _u32, _dbl, _i32, _vp, _vp, _vp, _vp]
_lib.nsml_compress_pruned.restype = _i32
_lib.nsml_decompress.argtypes = [_vp, _vp, _vp, _vp, _u64, _vp, _u32, _dbl, _i32, _vp, _vp]
_lib.nsml_profile_enable.argtypes = [_vp, _i32]
_lib.nsml_profile_read.argtypes = [_vp, _vp, _vp]
_lib.nsml_path_stats.argtypes = [_vp, C.POINTER(_u32), C.POINTER(_u32)]
_lib.nsml_path_stats.restype = _i32
_lib.nsml_bucket_state.argtypes = [_vp, _u32, C.POINTER(_u32)]
_lib.nsml_bucket_state.restype = _i32
_lib.nsml_prune_stats.argtypes = [_vp, C.POINTER(_u32), C.POINTER(_u32)]
_lib.nsml_prune_stats.restype = _i32
_lib.nsml_decompress_accumulate.argtypes = [_vp, _vp, _vp, _vp, _u64, _vp, _u32, _dbl, _i32, _vp, _vp]
_lib.nsml_decompress_accumulate.restype = _i32
_lib.nsml_last_l2norm.argtypes = [_vp, C.POINTER(_dbl), _vp]
_lib.nsml_last_l2norm.restype = _i32
_lib.nsml_calibration_copy.argtypes = [_vp, _vp, _u64, _vp]
_lib.nsml_calibration_copy.restype = _i32
_lib.nsml_kernel_name.argtypes = [_i32]
_lib.nsml_kernel_name.restype = C.c_char_p
for _f in ("nsml_ctl_default_params", "nsml_ctl_init", "nsml_choose_ratio", "nsml_payload_layout",
           "nsml_create", "nsml_destroy", "nsml_last_hip_error", "nsml_compress",
           "nsml_decompress", "nsml_profile_enable", "nsml_profile_read"):
    getattr(_lib, _f).restype = _i32


class NsmlError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code, self.hip = code, hip
        msg = _lib.nsml_strerror(code).decode()
        super().__init__(f"{where}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))


def _check(rc: int, where: str, ctx=None):
    if rc != OK:
        hip = _lib.nsml_last_hip_error(ctx) if ctx else 0
        raise NsmlError(rc, where, hip)


def raw():
    """The ctypes library handle (for tests of the C ABI itself)."""
    return _lib


# ----------------------------------------------------------------------- controller

def default_params() -> CtlParams:
    p = CtlParams()
    _check(_lib.nsml_ctl_default_params(C.byref(p)), "nsml_ctl_default_params")
    return p


class Controller:
    """Host-side network-sensing controller state (nsml_ctl_state)."""

    def __init__(self, params: Optional[CtlParams] = None, **overrides):
        p = params or default_params()
        for k, v in overrides.items():
            setattr(p, k, v)
        self.state = CtlState()
        _check(_lib.nsml_ctl_init(C.byref(self.state), C.byref(p)), "nsml_ctl_init")

    def choose_ratio(self, last_payload_bytes: float, last_tx_seconds: float,
                     dense_bytes: float = 0.0, last_l2norm: float = -1.0) -> Tuple[float, int]:
        r, b = _dbl(), _i32()
        _check(_lib.nsml_choose_ratio(C.byref(self.state), last_payload_bytes, last_tx_seconds,
                                      dense_bytes, last_l2norm, C.byref(r), C.byref(b)),
               "nsml_choose_ratio")
        return r.value, b.value


def choose_ratio(ctl: Controller, last_payload_bytes: float, last_tx_seconds: float,
                 dense_bytes: float = 0.0, last_l2norm: float = -1.0) -> Tuple[float, int]:
    return ctl.choose_ratio(last_payload_bytes, last_tx_seconds, dense_bytes, last_l2norm)


# ----------------------------------------------------------------------- geometry

def _off(bucket_off) -> np.ndarray:
    return np.ascontiguousarray(bucket_off, dtype=np.uint64)


def payload_layout(bucket_off, ratio: float, bits: int, chunk: int = 2048):
    """-> (k_b uint64[B], K, val_bytes, n_scales)."""
    off = _off(bucket_off)
    B = len(off) - 1
    k_b = np.zeros(max(B, 1), dtype=np.uint64)
    K, vb, ns = _u64(), _u64(), _u64()
    _check(_lib.nsml_payload_layout(off.ctypes.data, B, ratio, bits, chunk, k_b.ctypes.data,
                                    C.byref(K), C.byref(vb), C.byref(ns)), "nsml_payload_layout")
    return k_b[:B], K.value, vb.value, ns.value


# ----------------------------------------------------------------------- GPU path

def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(device) -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def validate_buffers(device, bucket_off, ratio, bits, chunk, *, n=None, grad=None, residual=None,
                     weights=None, idx=None, val=None, scales=None, dense=None):
    """The C ABI carries no capacities, so the sizes, types and placement of every tensor are
    checked here, before a pointer reaches a kernel: a short buffer would be an out-of-bounds
    device write.  Raises ValueError; returns (K, val_bytes, n_scales)."""
    device = torch.device(device)
    off = _off(bucket_off)
    if off.ndim != 1 or len(off) < 2:
        raise ValueError("bucket_off needs at least two entries")
    total = int(off[-1])
    if n is not None and int(n) != total:
        raise ValueError(f"n = {n} but bucket_off ends at {total}")
    _, K, vb, ns = payload_layout(off, ratio, bits, chunk)

    def want(name, t, dtype, numel, exact):
        if t is None:
            return
        if not isinstance(t, torch.Tensor):
            raise ValueError(f"{name} must be a torch tensor")
        if t.device != device:
            raise ValueError(f"{name} is on {t.device}, the context is on {device}")
        if t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
            raise ValueError(f"{name} has dtype {t.dtype}")
        if not t.is_contiguous():
            raise ValueError(f"{name} is not contiguous")
        if (t.numel() != numel) if exact else (t.numel() < numel):
            raise ValueError(f"{name} holds {t.numel()} elements, needs {'exactly' if exact else 'at least'} {numel}")

    want("grad", grad, torch.float32, total, True)
    want("residual", residual, torch.float32, total, True)
    want("weights", weights, torch.float32, total, True)
    want("dense", dense, torch.float32, total, True)
    want("idx", idx, (torch.int32, torch.uint32), K, False)
    want("val", val, (torch.uint8, torch.int8), vb, False)
    if bits <= 8:
        if (idx is not None or val is not None) and scales is None:
            raise ValueError("scales is required for 8- and 4-bit codes")
        want("scales", scales, torch.float32, ns, False)
    return K, vb, ns


class Context:
    """nsml_ctx: device workspace for gradients of up to max_n elements / max_buckets buckets."""

    # nsml_set_option settings applied to every new context (the tests run the path under each)
    default_options: dict = {}

    def __init__(self, max_n: int, max_buckets: int = 1, chunk: int = 2048, device: int = 0,
                 max_ratio: float = 1.0):
        self.device, self.chunk = int(device), int(chunk)
        self._dev = torch.device("cuda", self.device)
        self._h = _vp()
        rc = _lib.nsml_create_ex(C.byref(self._h), self.device, int(max_n), int(max_buckets), self.chunk,
                                 float(max_ratio))
        if rc != OK:
            raise NsmlError(rc, "nsml_create_ex")
        for name, value in self.default_options.items():
            self.set_option(name, value)

    def set_option(self, name: str, value: int):
        _check(_lib.nsml_set_option(self._h, name.encode(), int(value)), f"nsml_set_option({name})", self._h)

    def close(self):
        if getattr(self, "_h", None):
            _lib.nsml_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self) -> int:
        return int(_lib.nsml_workspace_bytes(self._h))

    def alloc_payload(self, bucket_off, ratio: float, bits: int):
        """Device buffers sized by nsml_payload_layout: (idx, val, scales)."""
        _, K, vb, ns = payload_layout(bucket_off, ratio, bits, self.chunk)
        dev = torch.device("cuda", self.device)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        val = torch.empty((vb + 3) // 4 * 4, dtype=torch.uint8, device=dev)
        scales = torch.empty(max(ns, 1), dtype=torch.float32, device=dev)
        return idx, val, scales

    def compress(self, grad: torch.Tensor, residual: torch.Tensor, bucket_off, ratio: float,
                 bits: int, idx: torch.Tensor = None, val: torch.Tensor = None,
                 scales: torch.Tensor = None):
        """nsml_compress on torch's current stream.  residual is updated in place.
        -> (idx int32[K] (bit pattern of uint32), val uint8[...], scales float32[...])."""
        off = _off(bucket_off)
        if idx is None:
            idx, val, scales = self.alloc_payload(off, ratio, bits)
        validate_buffers(self._dev, off, ratio, bits, self.chunk, grad=grad, residual=residual,
                         idx=idx, val=val, scales=scales)
        rc = _lib.nsml_compress(self._h, _ptr(grad), _ptr(residual), grad.numel(), off.ctypes.data,
                                len(off) - 1, float(ratio), int(bits), _ptr(idx), _ptr(val),
                                _ptr(scales), _stream(self.device))
        _check(rc, "nsml_compress", self._h)
        return idx, val, scales

    def compress_pruned(self, grad: torch.Tensor, residual: torch.Tensor, weights: torch.Tensor,
                        bucket_off, ratio: float, bits: int, idx: torch.Tensor = None,
                        val: torch.Tensor = None, scales: torch.Tensor = None):
        """nsml_compress_pruned: as compress, after weight-magnitude pruning of the candidates."""
        off = _off(bucket_off)
        if idx is None:
            idx, val, scales = self.alloc_payload(off, ratio, bits)
        validate_buffers(self._dev, off, ratio, bits, self.chunk, grad=grad, residual=residual,
                         weights=weights, idx=idx, val=val, scales=scales)
        rc = _lib.nsml_compress_pruned(self._h, _ptr(grad), _ptr(residual), _ptr(weights), grad.numel(),
                                       off.ctypes.data, len(off) - 1, float(ratio), int(bits),
                                       _ptr(idx), _ptr(val), _ptr(scales), _stream(self.device))
        _check(rc, "nsml_compress_pruned", self._h)
        return idx, val, scales

    def decompress(self, idx: torch.Tensor, val: torch.Tensor, scales: torch.Tensor, n: int,
                   bucket_off, ratio: float, bits: int, out: torch.Tensor = None) -> torch.Tensor:
        off = _off(bucket_off)
        if out is None:
            out = torch.empty(int(n), dtype=torch.float32, device=self._dev)
        validate_buffers(self._dev, off, ratio, bits, self.chunk, n=n, idx=idx, val=val, scales=scales,
                         dense=out)
        rc = _lib.nsml_decompress(self._h, _ptr(idx), _ptr(val), _ptr(scales), int(n),
                                  off.ctypes.data, len(off) - 1, float(ratio), int(bits),
                                  _ptr(out), _stream(self.device))
        _check(rc, "nsml_decompress", self._h)
        return out

    def decompress_accumulate(self, idx, val, scales, bucket_off, ratio: float, bits: int,
                              dense: torch.Tensor) -> torch.Tensor:
        """dense[bucket_off[b] + idx[j]] += decoded value j, in place."""
        off = _off(bucket_off)
        validate_buffers(self._dev, off, ratio, bits, self.chunk, idx=idx, val=val, scales=scales,
                         dense=dense)
        rc = _lib.nsml_decompress_accumulate(self._h, _ptr(idx), _ptr(val), _ptr(scales),
                                             dense.numel(), off.ctypes.data, len(off) - 1,
                                             float(ratio), int(bits), _ptr(dense), _stream(self.device))
        _check(rc, "nsml_decompress_accumulate", self._h)
        return dense

    def last_l2norm(self, n_buckets: int = 0):
        """-> (norm of the last compressed gradient, per-bucket norms or None).  Synchronises."""
        tot = _dbl()
        per = np.zeros(n_buckets, dtype=np.float64) if n_buckets else None
        _check(_lib.nsml_last_l2norm(self._h, C.byref(tot), per.ctypes.data if n_buckets else None),
               "nsml_last_l2norm", self._h)
        return tot.value, per

    def path_stats(self):
        """-> (fast buckets, fallback buckets) of the last compress call (synchronises)."""
        a, b = _u32(), _u32()
        _check(_lib.nsml_path_stats(self._h, C.byref(a), C.byref(b)), "nsml_path_stats", self._h)
        return a.value, b.value

    def bucket_state(self, b: int):
        """-> dict with the selection state of bucket b after the last compress call (synchronises)."""
        out = (_u32 * 8)()
        _check(_lib.nsml_bucket_state(self._h, b, out), "nsml_bucket_state", self._h)
        names = ("path", "why", "L", "H", "T", "need", "sh", "k")
        return dict(zip(names, (int(x) for x in out)))

    def prune_stats(self):
        """-> (band buckets, dense buckets) of the weight stage of the last compress_pruned (synchronises)."""
        a, b = _u32(), _u32()
        _check(_lib.nsml_prune_stats(self._h, C.byref(a), C.byref(b)), "nsml_prune_stats", self._h)
        return a.value, b.value

    def profile_enable(self, on: bool = True):
        _check(_lib.nsml_profile_enable(self._h, 1 if on else 0), "nsml_profile_enable", self._h)

    def profile_read(self):
        """-> {kernel name: (launches, total ms)} since the last read."""
        n = (C.c_uint32 * MAX_KERNELS)()
        ms = (C.c_double * MAX_KERNELS)()
        _check(_lib.nsml_profile_read(self._h, n, ms), "nsml_profile_read", self._h)
        out = {}
        for i in range(MAX_KERNELS):
            name = _lib.nsml_kernel_name(i)
            if name is not None and n[i]:
                out[name.decode()] = (int(n[i]), float(ms[i]))
        return out


def decompress_accumulate(ctx: Context, idx, val, scales, bucket_off, ratio, bits, dense):
    return ctx.decompress_accumulate(idx, val, scales, bucket_off, ratio, bits, dense)


def decompress_static(idx: torch.Tensor, val: torch.Tensor, scales: Optional[torch.Tensor], n: int, bucket_off,
                      ratio: float, bits: int, chunk: int = 2048, out: torch.Tensor = None) -> torch.Tensor:
    """nsml_decompress_static: decompress without a context and without any allocation inside
    the library (the output tensor is the caller's), on the tensors' device."""
    off = _off(bucket_off)
    dev = idx.device
    if out is None:
        out = torch.empty(int(n), dtype=torch.float32, device=dev)
    validate_buffers(dev, off, ratio, bits, chunk, n=n, idx=idx, val=val, scales=scales, dense=out)
    with torch.cuda.device(dev):
        rc = _lib.nsml_decompress_static(_ptr(idx), _ptr(val), _ptr(scales), int(n), off.ctypes.data,
                                         len(off) - 1, float(ratio), int(bits), int(chunk), _ptr(out), _stream(dev))
    _check(rc, "nsml_decompress_static")
    return out


CALIB_MODES = {"read": 0, "fill": 1, "add": 2, "copy": 3}


def calibration_stream(mode: str, a: torch.Tensor, b: torch.Tensor, nontemporal: bool = False):
    """Plain streaming kernel of the given access pattern over a and b (same byte size)."""
    nbytes = a.numel() * a.element_size()
    assert nbytes == b.numel() * b.element_size()
    _check(_lib.nsml_calibration_stream(CALIB_MODES[mode], _ptr(a), _ptr(b), nbytes, 1 if nontemporal else 0,
                                        _stream(a.device)), "nsml_calibration_stream")


def calibration_copy(src: torch.Tensor, dst: torch.Tensor):
    """Plain copy kernel of known size (src -> dst, same byte size, a multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(_lib.nsml_calibration_copy(_ptr(src), _ptr(dst), nbytes, _stream(src.device)),
           "nsml_calibration_copy")


def compress(ctx: Context, grad, residual, bucket_off, ratio, bits, idx=None, val=None, scales=None):
    return ctx.compress(grad, residual, bucket_off, ratio, bits, idx, val, scales)


def compress_pruned(ctx: Context, grad, residual, weights, bucket_off, ratio, bits,
                    idx=None, val=None, scales=None):
    return ctx.compress_pruned(grad, residual, weights, bucket_off, ratio, bits, idx, val, scales)


def decompress(ctx: Context, idx, val, scales, n, bucket_off, ratio, bits, out=None):
    return ctx.decompress(idx, val, scales, n, bucket_off, ratio, bits, out)
