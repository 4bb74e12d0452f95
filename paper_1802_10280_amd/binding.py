"""ctypes binding of libescoin.so: the same names as the C ABI, argument marshalling only.

Host arguments are numpy arrays, device arguments are torch CUDA tensors (PyTorch supplies
device memory and streams, nothing else); every step of the path runs inside the library.
There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libescoin.so")

OK, EINVAL, ERANGE, EHIP, ESIZE = 0, -1, -2, -3, -4
F_BIAS, F_RELU = 1, 2


class escoin_conv_desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("N", "C", "H", "W", "M", "R", "S", "stride", "pad")]


class escoin_sconv_tuning(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("K", "Q", "B", "WM", "CC", "NB", "TH", "CS", "WS", "CC0")]


class EscoinError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1802_10280_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        D = ctypes.POINTER(escoin_conv_desc)
        vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        L.escoin_strerror.restype = ctypes.c_char_p
        L.escoin_strerror.argtypes = [ctypes.c_int]
        L.escoin_check_desc.argtypes = [D]
        L.escoin_output_dims.argtypes = [D, i32p, i32p]
        L.escoin_padded_elems.restype = ctypes.c_size_t
        L.escoin_padded_elems.argtypes = [D]
        L.escoin_output_elems.restype = ctypes.c_size_t
        L.escoin_output_elems.argtypes = [D]
        L.escoin_sconv_pack.argtypes = [D, vp, vp, vp]
        L.escoin_pad_in.argtypes = [D, vp, vp, vp]
        L.escoin_sconv_forward.argtypes = [D, vp, vp, vp, vp, vp, vp, ctypes.c_uint32, vp]
        T = ctypes.POINTER(escoin_sconv_tuning)
        L.escoin_sconv_plan_size.argtypes = [D, vp, vp, T, ctypes.POINTER(ctypes.c_size_t)]
        L.escoin_sconv_plan_build.argtypes = [D, vp, vp, vp, T, vp, ctypes.c_size_t]
        L.escoin_sconv_forward_tiled.argtypes = [D, vp, vp, vp, vp, vp, ctypes.c_uint32, vp]
        _lib = L
    return _lib


def make_desc(N, C, H, W, M, R, S, stride, pad) -> escoin_conv_desc:
    return escoin_conv_desc(N, C, H, W, M, R, S, stride, pad)


def desc_of(spec) -> escoin_conv_desc:
    """Descriptor from any object with the Table-1 attribute names."""
    return make_desc(spec.N, spec.C, spec.H, spec.W, spec.M, spec.R, spec.S, spec.stride, spec.pad)


def _check(rc: int, where: str):
    if rc != OK:
        raise EscoinError(rc, where)


def _hptr(a, dtype=None):
    """Pointer to a host numpy array (C-contiguous, expected dtype) or None."""
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("host arguments must be C-contiguous numpy arrays")
    if dtype is not None and a.dtype != dtype:
        raise TypeError(f"host array has dtype {a.dtype}, expected {dtype}")
    return a.ctypes.data


def _dptr(t, dtype=None):
    """Pointer to a contiguous torch CUDA tensor or None."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise TypeError("device arguments must be contiguous CUDA tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"device tensor has dtype {t.dtype}, expected {dtype}")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def strerror(code: int) -> str:
    return lib().escoin_strerror(code).decode()


def escoin_check_desc(desc) -> int:
    return lib().escoin_check_desc(ctypes.byref(desc))


def escoin_output_dims(desc):
    E, F = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().escoin_output_dims(ctypes.byref(desc), ctypes.byref(E), ctypes.byref(F)),
           "escoin_output_dims")
    return E.value, F.value


def escoin_padded_elems(desc) -> int:
    return lib().escoin_padded_elems(ctypes.byref(desc))


def escoin_output_elems(desc) -> int:
    return lib().escoin_output_elems(ctypes.byref(desc))


def escoin_sconv_pack(desc, rowptr: np.ndarray, colidx: np.ndarray,
                      colidx_stretched: np.ndarray | None = None) -> np.ndarray:
    if colidx_stretched is None:
        colidx_stretched = np.empty_like(colidx)
    _check(lib().escoin_sconv_pack(ctypes.byref(desc), _hptr(rowptr, np.int32),
                                   _hptr(colidx, np.int32), _hptr(colidx_stretched, np.int32)),
           "escoin_sconv_pack")
    return colidx_stretched


def escoin_pad_in(desc, d_in, d_padded, stream=None):
    import torch
    _check(lib().escoin_pad_in(ctypes.byref(desc), _dptr(d_in, torch.float32),
                               _dptr(d_padded, torch.float32), _stream(stream)), "escoin_pad_in")


def escoin_sconv_forward(desc, d_rowptr, d_colidx_stretched, d_value, d_padded, d_out,
                         d_bias=None, flags=0, stream=None):
    import torch
    _check(lib().escoin_sconv_forward(ctypes.byref(desc), _dptr(d_rowptr, torch.int32),
                                      _dptr(d_colidx_stretched, torch.int32),
                                      _dptr(d_value, torch.float32),
                                      _dptr(d_padded, torch.float32),
                                      _dptr(d_out, torch.float32), _dptr(d_bias, torch.float32),
                                      flags, _stream(stream)), "escoin_sconv_forward")


def make_tuning(**kw):
    """Tiling knobs for the plan (K, Q, B, WM, CC, NB, TH, CS, WS, CC0); omitted fields are chosen by the
    library.  Returns None when nothing is given."""
    if not kw:
        return None
    return escoin_sconv_tuning(**{k: int(v) for k, v in kw.items()})


def _tref(tuning):
    return ctypes.byref(tuning) if tuning is not None else None


def escoin_sconv_plan_size(desc, rowptr: np.ndarray, colidx_stretched: np.ndarray, tuning=None) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().escoin_sconv_plan_size(ctypes.byref(desc), _hptr(rowptr, np.int32),
                                        _hptr(colidx_stretched, np.int32), _tref(tuning),
                                        ctypes.byref(n)), "escoin_sconv_plan_size")
    return n.value


def escoin_sconv_plan_build(desc, rowptr: np.ndarray, colidx_stretched: np.ndarray,
                            value: np.ndarray, tuning=None, plan: np.ndarray | None = None) -> np.ndarray:
    """Returns the plan blob as a uint8 numpy array (host)."""
    if plan is None:
        plan = np.empty(escoin_sconv_plan_size(desc, rowptr, colidx_stretched, tuning), dtype=np.uint8)
    _check(lib().escoin_sconv_plan_build(ctypes.byref(desc), _hptr(rowptr, np.int32),
                                         _hptr(colidx_stretched, np.int32), _hptr(value, np.float32),
                                         _tref(tuning), _hptr(plan, np.uint8), plan.nbytes),
           "escoin_sconv_plan_build")
    return plan


def escoin_sconv_forward_tiled(desc, plan_host: np.ndarray, d_plan, d_in, d_out, d_bias=None,
                               flags=0, stream=None):
    import torch
    _check(lib().escoin_sconv_forward_tiled(ctypes.byref(desc), _hptr(plan_host, np.uint8),
                                            _dptr(d_plan, torch.uint8), _dptr(d_in, torch.float32),
                                            _dptr(d_out, torch.float32), _dptr(d_bias, torch.float32),
                                            flags, _stream(stream)), "escoin_sconv_forward_tiled")


class _PlanHeader(ctypes.Structure):
    """Mirror of the plan blob's header (csrc/plan.h), for diagnostics, tests and the bench."""
    _fields_ = ([("magic", ctypes.c_uint32), ("version", ctypes.c_uint32)]
                + [(k, ctypes.c_int32) for k in (
                    "C", "H", "W", "M", "R", "S", "stride", "pad", "E", "F", "K", "Q", "B", "WM", "WQ",
                    "CC", "NB", "TH", "n_tiles", "n_mgroups", "n_chunks", "n_phases", "pitch", "front",
                    "rows_in", "plane_stride", "P4", "n_items", "buf_floats", "tail_floats",
                    "rec_buf_bytes", "lds_bytes", "nnz", "n_records")]
                + [(k, ctypes.c_uint64) for k in (
                    "off_items", "off_lanes", "off_dst_lut", "off_perm", "off_blk", "off_seg", "off_rec",
                    "total_bytes")]
                + [(k, ctypes.c_int32) for k in (
                    "CS", "pitch1", "VW", "WW", "WS", "CC0", "zero_floats", "max_regions", "MB", "n_dma")]
                + [("off_dma", ctypes.c_uint64), ("off_zero", ctypes.c_uint64)])


def plan_header(plan: np.ndarray) -> dict:
    """Decodes the (opaque) plan header for diagnostics, tests and the bench's reporting."""
    h = _PlanHeader.from_buffer_copy(plan[:ctypes.sizeof(_PlanHeader)].tobytes())
    return {k: int(getattr(h, k)) for k, _ in _PlanHeader._fields_}
