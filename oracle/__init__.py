"""CPU oracle for direct sparse convolution -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It wraps ``escoin_oracle.c`` (plain C, fp64 accumulation; see that
file's header for what each function computes and which passage of the paper defines it)
through ctypes and shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "escoin_oracle.c")
_LIB = os.path.join(_HERE, "libescoin_oracle.so")

F_BIAS = 1
F_RELU = 2

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over (n, m) only, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", _LIB,
               _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def threads() -> int:
    return int(_load().oracle_threads())


def csr_to_dense(M, C, R, S, rowptr, colidx, value) -> np.ndarray:
    rowptr, colidx, value = _i32(rowptr), _i32(colidx), _f32(value)
    Wd = np.empty((M, C, R, S), dtype=np.float64)
    rc = _load().oracle_csr_to_dense(M, C, R, S, _p(rowptr, ctypes.c_int32),
                                     _p(colidx, ctypes.c_int32), _p(value, ctypes.c_float),
                                     _p(Wd, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_csr_to_dense: column index out of range")
    return Wd


def _shape_args(x, Wd, stride, pad):
    N, C, H, W = x.shape
    M, C2, R, S = Wd.shape
    assert C == C2
    return [ctypes.c_int(v) for v in (N, C, H, W, M, R, S, stride, pad)]


def conv(x, Wd, stride=1, pad=0, bias=None, flags=0):
    """Eq. (1) with zero padding and stride.  Returns (out fp32, bound fp64) as (N,M,E,F)."""
    x = _f32(x)
    Wd = np.ascontiguousarray(Wd, dtype=np.float64)
    N, C, H, W = x.shape
    M, _, R, S = Wd.shape
    E = (H + 2 * pad - R) // stride + 1
    F = (W + 2 * pad - S) // stride + 1
    out = np.empty((N, M, E, F), dtype=np.float32)
    bound = np.empty((N, M, E, F), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    rc = _load().oracle_conv(*_shape_args(x, Wd, stride, pad), _p(x, ctypes.c_float),
                             _p(Wd, ctypes.c_double), _p(b, ctypes.c_float),
                             ctypes.c_uint(flags), _p(out, ctypes.c_float),
                             _p(bound, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_conv: bad shape")
    return out, bound


def conv_points(x, Wd, pts, stride=1, pad=0, bias=None, flags=0):
    """Sampled outputs; ``pts`` is (npts, 4) int32 rows of (n, m, h, w)."""
    x = _f32(x)
    Wd = np.ascontiguousarray(Wd, dtype=np.float64)
    pts = _i32(pts).reshape(-1, 4)
    out = np.empty(len(pts), dtype=np.float32)
    bound = np.empty(len(pts), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    rc = _load().oracle_conv_points(*_shape_args(x, Wd, stride, pad), _p(x, ctypes.c_float),
                                    _p(Wd, ctypes.c_double), _p(b, ctypes.c_float),
                                    ctypes.c_uint(flags), ctypes.c_int64(len(pts)),
                                    _p(pts, ctypes.c_int32), _p(out, ctypes.c_float),
                                    _p(bound, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_conv_points: bad shape")
    return out, bound


def stretch(C, H, W, R, S, pad, colidx) -> np.ndarray:
    colidx = _i32(colidx)
    out = np.empty_like(colidx)
    rc = _load().oracle_stretch(C, H, W, R, S, pad, ctypes.c_int64(len(colidx)),
                                _p(colidx, ctypes.c_int32), _p(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_stretch: column index out of range")
    return out


def pad_input(x, pad) -> np.ndarray:
    x = _f32(x)
    N, C, H, W = x.shape
    out = np.empty((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float32)
    _load().oracle_pad(N, C, H, W, pad, _p(x, ctypes.c_float), _p(out, ctypes.c_float))
    return out


def sconv_alg2(shape, rowptr, stretched, value, padded):
    """Algorithm 2 on the stretched CSR and the padded input.  ``shape`` is
    (N, C, H, W, M, R, S, stride, pad) with H, W the unpadded dims."""
    N, C, H, W, M, R, S, stride, pad = shape
    rowptr, stretched, value = _i32(rowptr), _i32(stretched), _f32(value)
    padded = _f32(padded)
    E = (H + 2 * pad - R) // stride + 1
    F = (W + 2 * pad - S) // stride + 1
    out = np.empty((N, M, E, F), dtype=np.float32)
    _load().oracle_sconv_alg2(*[ctypes.c_int(v) for v in shape], _p(rowptr, ctypes.c_int32),
                              _p(stretched, ctypes.c_int32), _p(value, ctypes.c_float),
                              _p(padded, ctypes.c_float), _p(out, ctypes.c_float))
    return out
