"""ctypes front end of the plain-C APMSqueeze oracle (test infrastructure only).

The arithmetic lives in ``apms_oracle.c``; this module only compiles it with
gcc, loads it and marshals numpy arrays.  Nothing here imports or is imported
by the HIP library or its Python binding.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.

Compression stage: Algorithm 1 lines 3-12 / supplement "Proof to the Updating
Form" steps 1-3; 1-bit operator: Section 5.1; warm-up: Section 3.2.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

ONEBIT = 0
IDENTITY = 1
GRAD_F16 = 1
GRAD_BF16 = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "apms_oracle.c")
_LIB = os.path.join(_HERE, "libapms_oracle.so")
_lib = None

# No FMA contraction, no fast-math: every fp32 operation rounds once, in order.
CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i32, i64, f32, ptr = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
        lib.apms_oracle_compress.argtypes = [ctypes.c_int, i64, i32, i64, ptr, ptr, ptr, ptr, ptr, ptr, f32]
        lib.apms_oracle_server_reduce.argtypes = [ctypes.c_int, i64, i32, i64, ptr, ptr, ptr, ptr, ptr, ptr, ptr]
        lib.apms_oracle_apply.argtypes = [ctypes.c_int, i64, i32, i64, ptr, ptr, ptr, ptr, ptr, ptr, f32, f32]
        lib.apms_oracle_apply_gradient.argtypes = [ctypes.c_int, i64, i32, i64, ptr, ptr, ptr, ptr, ptr, ptr, f32, f32, f32]
        lib.apms_oracle_apply_gradient.restype = ctypes.c_int
        lib.apms_oracle_warmup_step.argtypes = [i64, i32, ptr, ptr, ptr, ptr, f32, f32, f32, f32, i64]
        lib.apms_oracle_freeze.argtypes = [i64, i32, ptr, ptr, ptr, ptr]
        lib.apms_oracle_topk_compress.argtypes = [i64, i32, i64, i64, ptr, ptr, ptr, ptr, ptr, f32]
        lib.apms_oracle_topk_server_reduce.argtypes = [i64, i32, i64, i64, ptr, ptr, ptr, ptr, ptr]
        lib.apms_oracle_topk_apply.argtypes = [i64, i32, i64, i64, ptr, ptr, ptr, ptr, ptr, f32, f32]
        for fn in (lib.apms_oracle_topk_compress, lib.apms_oracle_topk_server_reduce, lib.apms_oracle_topk_apply):
            fn.restype = ctypes.c_int
        lib.apms_oracle_widen_g16.argtypes = [ctypes.c_int, i64, ptr, ptr]
        lib.apms_oracle_widen_g16.restype = ctypes.c_int
        lib.apms_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.apms_oracle_set_threads.restype = None
        for fn in (lib.apms_oracle_compress, lib.apms_oracle_server_reduce, lib.apms_oracle_apply,
                   lib.apms_oracle_warmup_step, lib.apms_oracle_freeze):
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def set_threads(threads: int) -> None:
    """Threads the oracle may spread INDEPENDENT work over ((worker, chunk) problems, chunks, elements of a
    loop without a carried value); 1, the default, is serial.  The results do not depend on it."""
    _load().apms_oracle_set_threads(int(threads))


def host_cores() -> int:
    """Cores this process may run on."""
    return len(os.sched_getaffinity(0))


def _p(a, dtype, size):
    """Pointer to a C-contiguous numpy array of the given dtype and element count (None -> NULL)."""
    if a is None:
        return None
    if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"]):
        raise TypeError("expected a C-contiguous %s array" % np.dtype(dtype).name)
    if a.size != size:
        raise ValueError("expected %d elements, got %d" % (size, a.size))
    return a.ctypes.data_as(ctypes.c_void_p)


def _check_shape(d, n, L):
    if n < 1 or d < 0 or L < 32 or L % 32 or d % L:
        raise ValueError("need n >= 1, L a positive multiple of 32, d a multiple of L")


def compress(d, n, L, m, g, werr, packed, scales, beta, compressor=ONEBIT, dense=None):
    """Worker step for all n workers and all chunks; werr, packed, scales (, dense) written in place.
    m=None selects the APGSqueeze variant (the gradient itself is compensated and compressed)."""
    _check_shape(d, n, L)
    C = d // L
    f, u = np.float32, np.uint32
    rc = _load().apms_oracle_compress(
        compressor, d, n, L, _p(m, f, n * d), _p(g, f, n * d), _p(werr, f, n * d),
        _p(packed, u, n * d // 32), _p(scales, f, n * C), _p(dense, f, n * d), np.float32(beta))
    if rc:
        raise MemoryError("oracle compress")


def server_reduce(d, n, L, packed, scales, serr, spacked, sscales, compressor=ONEBIT,
                  dense=None, sdense=None):
    """Server step for all chunks; serr, spacked, sscales (, sdense) written in place."""
    _check_shape(d, n, L)
    C = d // L
    f, u = np.float32, np.uint32
    rc = _load().apms_oracle_server_reduce(
        compressor, d, n, L, _p(packed, u, n * d // 32), _p(scales, f, n * C), _p(dense, f, n * d),
        _p(serr, f, d), _p(spacked, u, d // 32), _p(sscales, f, C), _p(sdense, f, d))
    if rc:
        raise MemoryError("oracle server_reduce")


def apply(d, n, L, spacked, sscales, v, x, m, lr, eps, compressor=ONEBIT, sdense=None):
    """Gather + frozen-variance model update; x and all n slices of m written in place."""
    _check_shape(d, n, L)
    C = d // L
    f, u = np.float32, np.uint32
    _load().apms_oracle_apply(
        compressor, d, n, L, _p(spacked, u, d // 32), _p(sscales, f, C), _p(sdense, f, d),
        _p(v, f, d), _p(x, f, d), _p(m, f, n * d), np.float32(lr), np.float32(eps))


def apply_gradient(d, n, L, spacked, sscales, v, x, m, lr, beta, eps, compressor=ONEBIT, sdense=None):
    """APGSqueeze: momentum step on the decoded averaged gradient + frozen-variance model update; x, m in place."""
    _check_shape(d, n, L)
    C = d // L
    f, u = np.float32, np.uint32
    _load().apms_oracle_apply_gradient(
        compressor, d, n, L, _p(spacked, u, d // 32), _p(sscales, f, C), _p(sdense, f, d),
        _p(v, f, d), _p(x, f, d), _p(m, f, n * d), np.float32(lr), np.float32(beta), np.float32(eps))


def warmup_step(d, n, x, m, v, g, lr, beta1, beta2, eps, t):
    """One Adam warm-up step on the average of the n gradients; x, m, v ([d]) in place; t is 1-based."""
    if n < 1 or d < 0 or t < 1:
        raise ValueError("need n >= 1, d >= 0, t >= 1")
    f = np.float32
    _load().apms_oracle_warmup_step(
        d, n, _p(x, f, d), _p(m, f, d), _p(v, f, d), _p(g, f, n * d),
        np.float32(lr), np.float32(beta1), np.float32(beta2), np.float32(eps), t)


def freeze(d, n, m_warm, m, werr, serr):
    """Warm-up -> compression stage hand-over: replicate m, zero both errors."""
    f = np.float32
    _load().apms_oracle_freeze(d, n, _p(m_warm, f, d), _p(m, f, n * d), _p(werr, f, n * d), _p(serr, f, d))


def widen_g16(g16, fmt):
    """binary16 (GRAD_F16) or bfloat16 (GRAD_BF16) bit patterns (uint16 array) -> float32 array, same shape."""
    if not (isinstance(g16, np.ndarray) and g16.dtype == np.uint16 and g16.flags["C_CONTIGUOUS"]):
        raise TypeError("expected a C-contiguous uint16 array")
    out = np.empty(g16.shape, np.float32)
    rc = _load().apms_oracle_widen_g16(fmt, g16.size, g16.ctypes.data_as(ctypes.c_void_p),
                                       out.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ValueError("unknown 16-bit gradient format %r" % (fmt,))
    return out


def _check_topk(d, n, L, K):
    _check_shape(d, n, L)
    if not 1 <= K <= L:
        raise ValueError("need 1 <= K <= L")


def topk_compress(d, n, L, K, m, g, werr, idx, val, beta):
    """Worker step with the top-k compressor; werr, idx, val ([n][C][K]) written in place."""
    _check_topk(d, n, L, K)
    C = d // L
    f, u = np.float32, np.uint32
    rc = _load().apms_oracle_topk_compress(d, n, L, K, _p(m, f, n * d), _p(g, f, n * d), _p(werr, f, n * d),
                                           _p(idx, u, n * C * K), _p(val, f, n * C * K), np.float32(beta))
    if rc:
        raise MemoryError("oracle topk_compress")


def topk_server_reduce(d, n, L, K, idx, val, serr, sidx, sval):
    """Server step with the top-k compressor; serr, sidx, sval ([C][K]) written in place."""
    _check_topk(d, n, L, K)
    C = d // L
    f, u = np.float32, np.uint32
    rc = _load().apms_oracle_topk_server_reduce(d, n, L, K, _p(idx, u, n * C * K), _p(val, f, n * C * K),
                                                _p(serr, f, d), _p(sidx, u, C * K), _p(sval, f, C * K))
    if rc:
        raise MemoryError("oracle topk_server_reduce")


def topk_apply(d, n, L, K, sidx, sval, v, x, m, lr, eps):
    """Gather + model update with the top-k compressor; x and all n slices of m written in place."""
    _check_topk(d, n, L, K)
    C = d // L
    f, u = np.float32, np.uint32
    _load().apms_oracle_topk_apply(d, n, L, K, _p(sidx, u, C * K), _p(sval, f, C * K), _p(v, f, d), _p(x, f, d),
                                   _p(m, f, n * d), np.float32(lr), np.float32(eps))


class State:
    """Host-side state of the compression stage for n simulated workers (numpy arrays)."""

    def __init__(self, d, n, L, x, m, v, werr=None, serr=None):
        _check_shape(d, n, L)
        self.d, self.n, self.L, self.C = d, n, L, d // L
        f = np.float32
        self.x = np.ascontiguousarray(x, dtype=f).copy()
        self.m = np.ascontiguousarray(m, dtype=f).reshape(n, d).copy()
        self.v = np.ascontiguousarray(v, dtype=f).copy()
        self.werr = np.zeros((n, d), f) if werr is None else np.ascontiguousarray(werr, dtype=f).reshape(n, d).copy()
        self.serr = np.zeros(d, f) if serr is None else np.ascontiguousarray(serr, dtype=f).copy()
        self.packed = np.zeros((n, d // 32), np.uint32)
        self.scales = np.zeros((n, self.C), f)
        self.spacked = np.zeros(d // 32, np.uint32)
        self.sscales = np.zeros(self.C, f)
        self.dense = None
        self.sdense = None

    def step(self, g, beta, lr, eps, compressor=ONEBIT):
        """One full compressed step (compress -> server_reduce -> apply) on gradients g [n][d]."""
        d, n, L = self.d, self.n, self.L
        g = np.ascontiguousarray(g, dtype=np.float32).reshape(n, d)
        if compressor == IDENTITY and self.dense is None:
            self.dense = np.zeros((n, d), np.float32)
            self.sdense = np.zeros(d, np.float32)
        compress(d, n, L, self.m, g, self.werr, self.packed, self.scales, beta, compressor, self.dense)
        server_reduce(d, n, L, self.packed, self.scales, self.serr, self.spacked, self.sscales,
                      compressor, self.dense, self.sdense)
        apply(d, n, L, self.spacked, self.sscales, self.v, self.x, self.m, lr, eps, compressor, self.sdense)

    def step_topk(self, g, K, beta, lr, eps):
        """One compressed step with the top-k compressor (K kept elements per chunk)."""
        d, n, L, C = self.d, self.n, self.L, self.C
        g = np.ascontiguousarray(g, dtype=np.float32).reshape(n, d)
        if getattr(self, "idx", None) is None or self.idx.shape[-1] != K:
            self.idx = np.zeros((n, C, K), np.uint32)
            self.val = np.zeros((n, C, K), np.float32)
            self.sidx = np.zeros((C, K), np.uint32)
            self.sval = np.zeros((C, K), np.float32)
        topk_compress(d, n, L, K, self.m, g, self.werr, self.idx, self.val, beta)
        topk_server_reduce(d, n, L, K, self.idx, self.val, self.serr, self.sidx, self.sval)
        topk_apply(d, n, L, K, self.sidx, self.sval, self.v, self.x, self.m, lr, eps)

    def step_gradient(self, g, beta, lr, eps, compressor=ONEBIT):
        """One APGSqueeze step: compress g + delta, server reduce, momentum + model update."""
        d, n, L = self.d, self.n, self.L
        g = np.ascontiguousarray(g, dtype=np.float32).reshape(n, d)
        if compressor == IDENTITY and self.dense is None:
            self.dense = np.zeros((n, d), np.float32)
            self.sdense = np.zeros(d, np.float32)
        compress(d, n, L, None, g, self.werr, self.packed, self.scales, 0.0, compressor, self.dense)
        server_reduce(d, n, L, self.packed, self.scales, self.serr, self.spacked, self.sscales,
                      compressor, self.dense, self.sdense)
        apply_gradient(d, n, L, self.spacked, self.sscales, self.v, self.x, self.m, lr, beta, eps, compressor,
                       self.sdense)
