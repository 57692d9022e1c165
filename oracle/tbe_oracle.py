"""ctypes wrapper around the CPU oracle (oracle/tbe_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU-baseline leg
may import this module; the HIP library and its Python binding never do, and this
module imports nothing from them.  Arrays are numpy, host memory, C-contiguous.

The functions mirror the C entry points one to one; see the C file for the passages of
the paper (Sections 2, 5.1, 5.2, 7.1) each one follows and for the data layout.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tbe_oracle.c")
_LIB = os.path.join(_HERE, "libtbe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no intrinsics, single thread)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.oracle_tbe_forward.argtypes = [i32, vp, vp, i32, vp, vp, vp, i32, vp, vp]
        lib.oracle_tbe_forward.restype = ctypes.c_int
        lib.oracle_tbe_sort_artifacts.argtypes = [i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_tbe_sort_artifacts.restype = ctypes.c_int
        lib.oracle_tbe_backward_rowwise_adagrad.argtypes = [
            i32, vp, vp, i32, vp, vp, vp, vp, i32, vp, dbl, dbl, vp, vp, vp, vp]
        lib.oracle_tbe_backward_rowwise_adagrad.restype = ctypes.c_int
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_half_to_double.restype = dbl
        lib.oracle_double_to_half.argtypes = [dbl]
        lib.oracle_double_to_half.restype = ctypes.c_uint16
        _ = i64
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, name):
    a = np.ascontiguousarray(a, dtype=dtype)
    if a.dtype != np.dtype(dtype):
        raise TypeError(name)
    return a


def _wdtype(dtype: int):
    return np.float32 if dtype == 0 else np.float16


def half_to_double(bits: int) -> float:
    return _load().oracle_half_to_double(int(bits))


def double_to_half(x: float) -> int:
    return _load().oracle_double_to_half(float(x))


def forward(rows, dims, dtype, weights, indices, offsets, B, want_absref=False):
    """Sum-pooled forward.  Returns out[B, sumD] float32 (and absref float64 if asked)."""
    lib = _load()
    rows = _chk(rows, np.int64, "rows")
    dims = _chk(dims, np.int32, "dims")
    T = len(rows)
    weights = _chk(weights, _wdtype(dtype), "weights")
    indices = _chk(indices, np.int32, "indices")
    offsets = _chk(offsets, np.int64, "offsets")
    assert len(offsets) == T * B + 1
    assert weights.size == int((rows * dims.astype(np.int64)).sum())
    sumD = int(dims.sum())
    out = np.empty((B, sumD), dtype=np.float32)
    absref = np.empty((B, sumD), dtype=np.float64) if want_absref else None
    rc = lib.oracle_tbe_forward(T, _p(rows), _p(dims), dtype, _p(weights), _p(indices), _p(offsets),
                                B, _p(out), _p(absref))
    if rc:
        raise ValueError(f"oracle_tbe_forward rc={rc}")
    return (out, absref) if want_absref else out


@dataclass
class SortArtifacts:
    sorted_keys: np.ndarray   # uint32[N]
    sorted_vals: np.ndarray   # int32[N]
    unique_keys: np.ndarray   # uint32[U]
    seg_offsets: np.ndarray   # int64[U+1]
    num_unique: int


def sort_artifacts(rows, B, indices, offsets) -> SortArtifacts:
    lib = _load()
    rows = _chk(rows, np.int64, "rows")
    T = len(rows)
    indices = _chk(indices, np.int32, "indices")
    offsets = _chk(offsets, np.int64, "offsets")
    assert len(offsets) == T * B + 1
    N = int(offsets[-1])
    sk = np.empty(N, np.uint32)
    sv = np.empty(N, np.int32)
    uk = np.empty(N, np.uint32)
    so = np.empty(N + 1, np.int64)
    nu = np.zeros(1, np.int64)
    rc = lib.oracle_tbe_sort_artifacts(T, _p(rows), B, _p(indices), _p(offsets), _p(sk), _p(sv), _p(uk),
                                       _p(so), _p(nu))
    if rc:
        raise ValueError(f"oracle_tbe_sort_artifacts rc={rc}")
    U = int(nu[0])
    return SortArtifacts(sk, sv, uk[:U].copy(), so[:U + 1].copy(), U)


@dataclass
class BackwardDetail:
    G: np.ndarray          # float64, concatenated per touched row (ascending key)
    Gabs: np.ndarray       # float64, sum of |terms|
    g_offsets: np.ndarray  # int64[U+1]
    m_new: np.ndarray      # float64[U], unrounded updated moment


def backward_rowwise_adagrad(rows, dims, dtype, weights, moments, indices, offsets, B, grad_out,
                             lr, eps, want_detail=False):
    """In-place update of `weights` and `moments` (numpy arrays owned by the caller)."""
    lib = _load()
    rows = _chk(rows, np.int64, "rows")
    dims = _chk(dims, np.int32, "dims")
    T = len(rows)
    if weights.dtype != np.dtype(_wdtype(dtype)) or not weights.flags.c_contiguous:
        raise TypeError("weights must be a contiguous array of the table storage type")
    if moments.dtype != np.float32 or not moments.flags.c_contiguous:
        raise TypeError("moments must be contiguous float32")
    indices = _chk(indices, np.int32, "indices")
    offsets = _chk(offsets, np.int64, "offsets")
    grad_out = _chk(grad_out, np.float32, "grad_out")
    sumD = int(dims.sum())
    assert len(offsets) == T * B + 1
    assert grad_out.size == B * sumD
    assert weights.size == int((rows * dims.astype(np.int64)).sum())
    assert moments.size == int(rows.sum())
    N = int(offsets[-1])
    G = Gabs = goff = mnew = None
    if want_detail:
        cap = N * int(dims.max()) if N else 1
        G = np.zeros(cap, np.float64)
        Gabs = np.zeros(cap, np.float64)
        goff = np.zeros(N + 1, np.int64)
        mnew = np.zeros(max(N, 1), np.float64)
    # lr/eps arrive at the GPU library as float32: hand the oracle the same values
    lr = float(np.float32(lr))
    eps = float(np.float32(eps))
    rc = lib.oracle_tbe_backward_rowwise_adagrad(T, _p(rows), _p(dims), dtype, _p(weights), _p(moments),
                                                 _p(indices), _p(offsets), B, _p(grad_out), lr, eps,
                                                 _p(G), _p(Gabs), _p(goff), _p(mnew))
    if rc:
        raise ValueError(f"oracle_tbe_backward_rowwise_adagrad rc={rc}")
    if not want_detail:
        return None
    # number of touched rows = first u>0 with g_offsets[u]==total and monotone; recompute from sort
    U = sort_artifacts(rows, B, indices, offsets).num_unique
    tot = int(goff[U])
    return BackwardDetail(G[:tot].copy(), Gabs[:tot].copy(), goff[:U + 1].copy(), mnew[:U].copy())
