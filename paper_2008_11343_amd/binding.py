"""Thin ctypes binding of libapms.so: same names as the C ABI (include/apms.h), argument marshalling only.

Array arguments are torch tensors on the GPU (their data_ptr() is passed) or plain integer device
addresses; `stream` is a torch.cuda.Stream, a raw hipStream_t integer or None (= torch's current
stream).  Every step of the method runs in the library's HIP kernels; there is no fallback: if the
shared library is missing it is built with hipcc, and if that is impossible the import fails.
"""
from __future__ import annotations

import ctypes
import os

import torch  # first: libapms must bind to the HIP runtime torch has already loaded

from . import build as _build

APMS_OK = 0
APMS_EINVAL, APMS_EALIGN, APMS_ESHAPE, APMS_ENOMEM, APMS_EHIP, APMS_ENODEV, APMS_EALIAS, APMS_ESTATE, APMS_ELIMIT = (
    -1, -2, -3, -4, -5, -6, -7, -8, -9)
APMS_DEVICE_NONE = -1
APMS_STATIC_SCRATCH_BYTES = 1 << 20
APMS_GRAD_F16 = 1
APMS_GRAD_BF16 = 2
APMS_DEFER_ERRORS = 1
APMS_DEFER_GATHER = 2
APMS_IMPLICIT_MOMENTUM = 4
APMS_KERNEL_COMPRESS, APMS_KERNEL_SERVER, APMS_KERNEL_APPLY, APMS_KERNEL_FINALIZE, APMS_KERNEL_WARMUP = 0, 1, 2, 3, 4
APMS_KERNEL_COUNT = 5
APMS_PAD_AUTO = -1
APMS_GATHER_SPLIT, APMS_GATHER_FUSED, APMS_GATHER_AUTO = 0, 1, 2

EXPORTS = (
    "apms_create", "apms_destroy", "apms_strerror", "apms_last_hip_error", "apms_get_plan",
    "apms_set_tiles_per_block", "apms_set_occupancy_pad", "apms_set_gather_mode", "apms_set_deferral", "apms_finalize", "apms_warmup_step",
    "apms_warmup_step_g16", "apms_freeze", "apms_compress", "apms_compress_g16", "apms_server_reduce", "apms_apply",
    "apms_compress_gradient", "apms_apply_gradient",
    "apms_topk_reserve", "apms_topk_compress", "apms_topk_server_reduce", "apms_topk_apply",
    "apms_server_reduce_static",
)


class apms_plan(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int64), ("n", ctypes.c_int32), ("chunk_elems", ctypes.c_int64),
        ("chunks", ctypes.c_int64),
        ("compress_tile_elems", ctypes.c_int32), ("compress_tiles_per_block", ctypes.c_int32),
        ("compress_blocks_per_chunk", ctypes.c_int32), ("compress_grid", ctypes.c_int64),
        ("server_tile_elems", ctypes.c_int32), ("server_tiles_per_block", ctypes.c_int32),
        ("server_blocks_per_chunk", ctypes.c_int32), ("server_grid", ctypes.c_int64),
        ("apply_tile_elems", ctypes.c_int32), ("apply_grid", ctypes.c_int64),
        ("scratch_bytes", ctypes.c_int64), ("occupancy_pad", ctypes.c_int32 * 8), ("topk_scratch_bytes", ctypes.c_int64),
        ("gather_mode", ctypes.c_int32), ("gather_choice", ctypes.c_int32), ("gather_uncapped", ctypes.c_int32),
        ("gather_ms", ctypes.c_float * 3),
    ]

    def as_dict(self):
        out = {name: getattr(self, name) for name, _ in self._fields_}
        out["occupancy_pad"] = list(self.occupancy_pad)[:APMS_KERNEL_COUNT]
        out["gather_ms"] = list(self.gather_ms)
        return out


class ApmsError(RuntimeError):
    def __init__(self, status, where, hip=0):
        self.status = status
        self.hip = hip
        msg = "%s: %s (status %d)" % (where, apms_strerror(status), status)
        if hip:
            msg += " [hipError_t %d]" % hip
        super().__init__(msg)


_lib = None


def library_path() -> str:
    return _build.LIB


def _stale() -> bool:
    """True if libapms.so is missing or older than any of its sources."""
    if not os.path.exists(_build.LIB):
        return True
    built = os.path.getmtime(_build.LIB)
    return any(os.path.getmtime(src) > built for src in _build.source_files() if os.path.exists(src))


def load():
    """Load libapms.so, building it first if it is missing or older than a source it is built from."""
    global _lib
    if _lib is not None:
        return _lib
    if _stale():
        _build.build()
    lib = ctypes.CDLL(_build.LIB)
    vp, i32, i64, f32, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_int
    sig = {
        "apms_create": (ci, [ctypes.POINTER(vp), i64, i32, i64, ci]),
        "apms_destroy": (ci, [vp]),
        "apms_strerror": (ctypes.c_char_p, [ci]),
        "apms_last_hip_error": (ci, [vp]),
        "apms_get_plan": (ci, [vp, ctypes.POINTER(apms_plan)]),
        "apms_set_tiles_per_block": (ci, [vp, i32, i32]),
        "apms_set_occupancy_pad": (ci, [vp, ci, i32]),
        "apms_set_deferral": (ci, [vp, ci]),
        "apms_set_gather_mode": (ci, [vp, ci]),
        "apms_finalize": (ci, [vp, vp, vp, vp, vp]),
        "apms_warmup_step": (ci, [vp, vp, vp, vp, vp, f32, f32, f32, f32, i64, vp]),
        "apms_warmup_step_g16": (ci, [vp, vp, vp, vp, vp, ci, f32, f32, f32, f32, i64, vp]),
        "apms_compress_g16": (ci, [vp, vp, vp, ci, vp, vp, vp, f32, vp]),
        "apms_compress_gradient": (ci, [vp, vp, ci, vp, vp, vp, vp]),
        "apms_apply_gradient": (ci, [vp, vp, vp, vp, vp, vp, f32, f32, f32, vp]),
        "apms_topk_reserve": (ci, [vp, i64]),
        "apms_server_reduce_static": (ci, [i64, i32, i64, vp, vp, vp, vp, vp, vp]),
        "apms_topk_compress": (ci, [vp, vp, vp, vp, vp, vp, i64, f32, vp]),
        "apms_topk_server_reduce": (ci, [vp, vp, vp, i64, vp, vp, vp, vp]),
        "apms_topk_apply": (ci, [vp, vp, vp, i64, vp, vp, vp, f32, f32, vp]),
        "apms_freeze": (ci, [vp, vp, vp, vp, vp]),
        "apms_compress": (ci, [vp, vp, vp, vp, vp, vp, f32, vp]),
        "apms_server_reduce": (ci, [vp, vp, vp, vp, vp, vp, vp]),
        "apms_apply": (ci, [vp, vp, vp, vp, vp, vp, f32, f32, vp]),
    }
    for name in EXPORTS:
        fn = getattr(lib, name)          # AttributeError if the library does not export it
        fn.restype, fn.argtypes = sig[name]
    _lib = lib
    return lib


def _ptr(a):
    if a is None:
        return None
    if isinstance(a, int):
        return a
    if isinstance(a, torch.Tensor):
        if not a.is_contiguous():
            raise ValueError("tensor arguments must be contiguous")
        return a.data_ptr() or None
    raise TypeError("expected a torch tensor, an integer device address or None")


def _stream(s):
    if s is None:
        return torch.cuda.current_stream().cuda_stream or None if torch.cuda.is_available() else None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def _check(ctx, status, where):
    if status != APMS_OK:
        hip = load().apms_last_hip_error(ctx) if (ctx and status == APMS_EHIP) else 0
        raise ApmsError(status, where, hip)


def apms_strerror(status: int) -> str:
    return load().apms_strerror(status).decode()


def apms_create(d: int, n: int, chunk_elems: int, device: int = 0):
    """Returns the opaque context handle."""
    out = ctypes.c_void_p()
    _check(None, load().apms_create(ctypes.byref(out), d, n, chunk_elems, device), "apms_create")
    return out


def apms_destroy(ctx):
    _check(None, load().apms_destroy(ctx), "apms_destroy")


def apms_last_hip_error(ctx) -> int:
    return load().apms_last_hip_error(ctx)


def apms_get_plan(ctx) -> dict:
    plan = apms_plan()
    _check(ctx, load().apms_get_plan(ctx, ctypes.byref(plan)), "apms_get_plan")
    return plan.as_dict()


def apms_set_tiles_per_block(ctx, compress_tiles: int = 0, server_tiles: int = 0):
    _check(ctx, load().apms_set_tiles_per_block(ctx, compress_tiles, server_tiles), "apms_set_tiles_per_block")


def apms_set_occupancy_pad(ctx, kernel: int, lds_bytes: int):
    _check(ctx, load().apms_set_occupancy_pad(ctx, kernel, lds_bytes), "apms_set_occupancy_pad")


def apms_set_gather_mode(ctx, mode: int):
    _check(ctx, load().apms_set_gather_mode(ctx, mode), "apms_set_gather_mode")


def apms_set_deferral(ctx, flags: int):
    _check(ctx, load().apms_set_deferral(ctx, flags), "apms_set_deferral")


def apms_finalize(ctx, worker_err=None, server_err=None, m=None, stream=None):
    _check(ctx, load().apms_finalize(ctx, _ptr(worker_err), _ptr(server_err), _ptr(m), _stream(stream)),
           "apms_finalize")


def apms_warmup_step(ctx, x, m, v, g, lr, beta1, beta2, eps, t, stream=None):
    _check(ctx, load().apms_warmup_step(ctx, _ptr(x), _ptr(m), _ptr(v), _ptr(g), lr, beta1, beta2, eps, t,
                                        _stream(stream)), "apms_warmup_step")


def apms_warmup_step_g16(ctx, x, m, v, g, grad_format, lr, beta1, beta2, eps, t, stream=None):
    _check(ctx, load().apms_warmup_step_g16(ctx, _ptr(x), _ptr(m), _ptr(v), _ptr(g), grad_format, lr, beta1, beta2,
                                            eps, t, _stream(stream)), "apms_warmup_step_g16")


def apms_compress_g16(ctx, m, g, grad_format, worker_err, packed, scales, beta, stream=None):
    _check(ctx, load().apms_compress_g16(ctx, _ptr(m), _ptr(g), grad_format, _ptr(worker_err), _ptr(packed),
                                         _ptr(scales), beta, _stream(stream)), "apms_compress_g16")


def apms_freeze(ctx, m, worker_err, server_err, stream=None):
    _check(ctx, load().apms_freeze(ctx, _ptr(m), _ptr(worker_err), _ptr(server_err), _stream(stream)),
           "apms_freeze")


def apms_compress(ctx, m, g, worker_err, packed, scales, beta, stream=None):
    _check(ctx, load().apms_compress(ctx, _ptr(m), _ptr(g), _ptr(worker_err), _ptr(packed), _ptr(scales), beta,
                                     _stream(stream)), "apms_compress")


def apms_server_reduce(ctx, packed, scales, server_err, spacked, sscales, stream=None):
    _check(ctx, load().apms_server_reduce(ctx, _ptr(packed), _ptr(scales), _ptr(server_err), _ptr(spacked),
                                          _ptr(sscales), _stream(stream)), "apms_server_reduce")


def apms_apply(ctx, spacked, sscales, v, x, m, lr, eps, stream=None):
    _check(ctx, load().apms_apply(ctx, _ptr(spacked), _ptr(sscales), _ptr(v), _ptr(x), _ptr(m), lr, eps,
                                  _stream(stream)), "apms_apply")


def apms_compress_gradient(ctx, g, grad_format, worker_err, packed, scales, stream=None):
    _check(ctx, load().apms_compress_gradient(ctx, _ptr(g), grad_format, _ptr(worker_err), _ptr(packed),
                                              _ptr(scales), _stream(stream)), "apms_compress_gradient")


def apms_apply_gradient(ctx, spacked, sscales, v, x, m, lr, beta, eps, stream=None):
    _check(ctx, load().apms_apply_gradient(ctx, _ptr(spacked), _ptr(sscales), _ptr(v), _ptr(x), _ptr(m), lr, beta,
                                           eps, _stream(stream)), "apms_apply_gradient")


def apms_topk_reserve(ctx, K_max):
    _check(ctx, load().apms_topk_reserve(ctx, K_max), "apms_topk_reserve")


def apms_server_reduce_static(d, n, chunk_elems, packed, scales, server_err, spacked, sscales, stream=None):
    _check(None, load().apms_server_reduce_static(d, n, chunk_elems, _ptr(packed), _ptr(scales), _ptr(server_err),
                                                  _ptr(spacked), _ptr(sscales), _stream(stream)),
           "apms_server_reduce_static")


def apms_topk_compress(ctx, m, g, worker_err, idx, val, K, beta, stream=None):
    _check(ctx, load().apms_topk_compress(ctx, _ptr(m), _ptr(g), _ptr(worker_err), _ptr(idx), _ptr(val), K, beta,
                                          _stream(stream)), "apms_topk_compress")


def apms_topk_server_reduce(ctx, idx, val, K, server_err, sidx, sval, stream=None):
    _check(ctx, load().apms_topk_server_reduce(ctx, _ptr(idx), _ptr(val), K, _ptr(server_err), _ptr(sidx),
                                               _ptr(sval), _stream(stream)), "apms_topk_server_reduce")


def apms_topk_apply(ctx, sidx, sval, K, v, x, m, lr, eps, stream=None):
    _check(ctx, load().apms_topk_apply(ctx, _ptr(sidx), _ptr(sval), K, _ptr(v), _ptr(x), _ptr(m), lr, eps,
                                       _stream(stream)), "apms_topk_apply")
