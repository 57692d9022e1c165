"""ctypes wrapper of oracle/inputs_oracle.c (input-side kernels: lengths->offsets, (W,T,B)->(T,W,B)
permute, row-wise bucketize; Sections 4 and 7.1).  TEST INFRASTRUCTURE ONLY; numpy host arrays."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "inputs_oracle.c")
_LIB = os.path.join(_HERE, "libinputs_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.oracle_lengths_to_offsets.argtypes = [vp, i64, vp]
        L.oracle_permute_wtb_to_twb.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
        L.oracle_bucketize_rowwise.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def lengths_to_offsets(lengths) -> np.ndarray:
    lengths = np.ascontiguousarray(lengths, np.int32)
    off = np.empty(len(lengths) + 1, np.int64)
    if _load().oracle_lengths_to_offsets(_p(lengths), len(lengths), _p(off)):
        raise ValueError("negative length")
    return off


def permute_wtb_to_twb(W, T, B, lengths_in, indices_in):
    lengths_in = np.ascontiguousarray(lengths_in, np.int32)
    indices_in = np.ascontiguousarray(indices_in, np.int32)
    n = W * T * B
    assert len(lengths_in) == n and len(indices_in) == int(lengths_in.sum())
    lo = np.empty(n, np.int32)
    oo = np.empty(n + 1, np.int64)
    io = np.empty(max(len(indices_in), 1), np.int32)
    if _load().oracle_permute_wtb_to_twb(W, T, B, _p(lengths_in), _p(indices_in), _p(lo), _p(oo), _p(io)):
        raise ValueError("bad lengths")
    return lo, oo, io[:len(indices_in)]


def bucketize_rowwise(rows, B, W, indices, offsets):
    rows = np.ascontiguousarray(rows, np.int64)
    indices = np.ascontiguousarray(indices, np.int32)
    offsets = np.ascontiguousarray(offsets, np.int64)
    T = len(rows)
    assert len(offsets) == T * B + 1 and int(offsets[-1]) == len(indices)
    n = W * T * B
    lo = np.empty(n, np.int32)
    oo = np.empty(n + 1, np.int64)
    io = np.empty(max(len(indices), 1), np.int32)
    rc = _load().oracle_bucketize_rowwise(T, B, W, _p(rows), _p(indices), _p(offsets), _p(lo), _p(oo), _p(io))
    if rc:
        raise ValueError(f"oracle_bucketize_rowwise rc={rc}")
    return lo, oo, io[:len(indices)]
