"""Thin ctypes binding of libtbe.so: argument marshalling only, same names as include/tbe.h.

Every step of the operator runs in the HIP kernels of the library; torch is used here only to
hold device memory and to name the stream.  There is no CPU fallback: if the library has not been
built (python -m paper_2104_05158_amd.build) loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtbe.so")

TBE_OK = 0
TBE_ERR_INVALID_ARG = 1
TBE_ERR_UNSUPPORTED = 2
TBE_ERR_NOT_BOUND = 3
TBE_ERR_WORKSPACE_TOO_SMALL = 4
TBE_ERR_INDEX_OUT_OF_RANGE = 5
TBE_ERR_HIP = 6
TBE_DTYPE_FP32 = 0
TBE_DTYPE_FP16 = 1
TBE_DTYPE_BF16 = 2
TBE_POOLING_SUM = 0
TBE_OPT_ROWWISE_ADAGRAD = 0
TBE_OPT_ADAGRAD = 1
TBE_OPT_ADAM = 2
TBE_LAYOUT_BATCH_MAJOR = 0
TBE_LAYOUT_TABLE_MAJOR = 1
_TORCH_DTYPE = {TBE_DTYPE_FP32: torch.float32, TBE_DTYPE_FP16: torch.float16, TBE_DTYPE_BF16: torch.bfloat16}

EXPORTED = [
    "tbe_create", "tbe_destroy", "tbe_query_sizes", "tbe_bind", "tbe_forward",
    "tbe_backward_rowwise_adagrad", "tbe_backward_adagrad", "tbe_backward_adam", "tbe_backward_sort",
    "tbe_backward_update_rowwise_adagrad", "tbe_backward_update_adagrad", "tbe_backward_update_adam",
    "tbe_backward_artifacts", "tbe_check_inputs",
    "tbe_profile_enable", "tbe_profile_read", "tbe_probe_read", "tbe_status_string", "tbe_last_hip_error",
]
# include/tbe_inputs.h
EXPORTED_INPUTS = [
    "tbe_inputs_scratch_bytes", "tbe_lengths_to_offsets", "tbe_permute_wtb_to_twb", "tbe_bucketize_rowwise",
    "tbe_lengths_to_offsets_noalloc", "tbe_lengths_to_offsets_noalloc_max_bags",
]


class TbeError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)}) {detail}".strip())


class tbe_config_t(ctypes.Structure):
    _fields_ = [
        ("num_tables", ctypes.c_int32),
        ("rows", ctypes.POINTER(ctypes.c_int64)),
        ("dims", ctypes.POINTER(ctypes.c_int32)),
        ("weight_dtype", ctypes.c_int32),
        ("pooling", ctypes.c_int32),
        ("max_batch", ctypes.c_int32),
        ("max_indices", ctypes.c_int64),
        ("optimizer", ctypes.c_int32),
        ("output_dtype", ctypes.c_int32),
        ("grad_dtype", ctypes.c_int32),
        ("layout", ctypes.c_int32),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libtbe.so; raises if it was not built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2104_05158_amd.build)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        L.tbe_create.argtypes = [ctypes.POINTER(tbe_config_t), ctypes.POINTER(vp)]
        L.tbe_destroy.argtypes = [vp]
        L.tbe_query_sizes.argtypes = [vp] + [ctypes.POINTER(ctypes.c_size_t)] * 3 + [vp, vp, vp]
        L.tbe_bind.argtypes = [vp, vp, vp, vp, ctypes.c_size_t]
        L.tbe_forward.argtypes = [vp, vp, vp, i64, i32, vp, vp]
        L.tbe_backward_rowwise_adagrad.argtypes = [vp, vp, vp, i64, i32, vp, f32, f32, vp]
        L.tbe_backward_adagrad.argtypes = [vp, vp, vp, i64, i32, vp, f32, f32, vp]
        L.tbe_backward_adam.argtypes = [vp, vp, vp, i64, i32, vp, f32, f32, f32, f32, i64, vp]
        L.tbe_backward_sort.argtypes = [vp, vp, vp, i64, i32, vp]
        L.tbe_backward_update_rowwise_adagrad.argtypes = [vp, vp, f32, f32, vp]
        L.tbe_backward_update_adagrad.argtypes = [vp, vp, f32, f32, vp]
        L.tbe_backward_update_adam.argtypes = [vp, vp, f32, f32, f32, f32, i64, vp]
        L.tbe_backward_artifacts.argtypes = [vp] + [ctypes.POINTER(vp)] * 5
        L.tbe_check_inputs.argtypes = [vp, vp, vp, i64, i32, vp]
        L.tbe_profile_enable.argtypes = [vp, i32]
        L.tbe_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i64),
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        sz = ctypes.c_size_t
        L.tbe_probe_read.argtypes = [vp, sz, i32, vp, vp]
        L.tbe_inputs_scratch_bytes.argtypes = [i64]
        L.tbe_lengths_to_offsets.argtypes = [vp, i64, vp, vp, sz, vp]
        L.tbe_lengths_to_offsets_noalloc.argtypes = [vp, i64, vp, vp]
        L.tbe_lengths_to_offsets_noalloc_max_bags.argtypes = []
        L.tbe_permute_wtb_to_twb.argtypes = [i32, i32, i32, vp, vp, i64, vp, vp, vp, vp, sz, vp]
        L.tbe_bucketize_rowwise.argtypes = [i32, i32, i32, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
        for name in EXPORTED + EXPORTED_INPUTS:
            getattr(L, name).restype = ctypes.c_int
        L.tbe_inputs_scratch_bytes.restype = sz
        L.tbe_lengths_to_offsets_noalloc_max_bags.restype = i64
        L.tbe_status_string.argtypes = [ctypes.c_int]
        L.tbe_status_string.restype = ctypes.c_char_p
        L.tbe_last_hip_error.argtypes = [vp]
        L.tbe_last_hip_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().tbe_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


# ---- raw calls, one per C entry point (return the status; raise nothing) ----

def tbe_create(rows, dims, weight_dtype: int, max_batch: int, max_indices: int,
               pooling: int = TBE_POOLING_SUM, optimizer: int = TBE_OPT_ROWWISE_ADAGRAD,
               output_dtype: int = TBE_DTYPE_FP32, grad_dtype: int = TBE_DTYPE_FP32,
               layout: int = 0) -> Tuple[int, Optional[int]]:
    rows = np.ascontiguousarray(rows, np.int64)
    dims = np.ascontiguousarray(dims, np.int32)
    cfg = tbe_config_t(len(rows), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                       dims.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), weight_dtype, pooling,
                       max_batch, max_indices, optimizer, output_dtype, grad_dtype, layout)
    h = ctypes.c_void_p()
    rc = lib().tbe_create(ctypes.byref(cfg), ctypes.byref(h))
    return rc, (h.value if rc == TBE_OK else None)


def tbe_destroy(h) -> int:
    return lib().tbe_destroy(ctypes.c_void_p(h))


def tbe_query_sizes(h, T: int):
    wb, sb, ws = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    woff = np.zeros(T + 1, np.int64)
    soff = np.zeros(T + 1, np.int64)
    coff = np.zeros(T + 1, np.int32)
    rc = lib().tbe_query_sizes(ctypes.c_void_p(h), ctypes.byref(wb), ctypes.byref(sb), ctypes.byref(ws),
                               woff.ctypes.data_as(ctypes.c_void_p), soff.ctypes.data_as(ctypes.c_void_p),
                               coff.ctypes.data_as(ctypes.c_void_p))
    return rc, dict(weight_bytes=wb.value, state_bytes=sb.value, workspace_bytes=ws.value,
                    weight_offsets=woff, state_offsets=soff, out_col_offsets=coff)


def tbe_bind(h, weights: torch.Tensor, state: torch.Tensor, workspace: torch.Tensor) -> int:
    return lib().tbe_bind(ctypes.c_void_p(h), _ptr(weights), _ptr(state), _ptr(workspace),
                          workspace.numel() * workspace.element_size())


def tbe_forward(h, indices, offsets, num_indices: int, batch: int, out, stream=None) -> int:
    return lib().tbe_forward(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices, batch, _ptr(out),
                             _stream_ptr(stream))


def tbe_backward_rowwise_adagrad(h, indices, offsets, num_indices: int, batch: int, grad_out, lr: float,
                                 eps: float, stream=None) -> int:
    return lib().tbe_backward_rowwise_adagrad(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices,
                                              batch, _ptr(grad_out), lr, eps, _stream_ptr(stream))


def tbe_backward_adagrad(h, indices, offsets, num_indices: int, batch: int, grad_out, lr: float, eps: float,
                         stream=None) -> int:
    return lib().tbe_backward_adagrad(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices, batch,
                                      _ptr(grad_out), lr, eps, _stream_ptr(stream))


def tbe_backward_adam(h, indices, offsets, num_indices: int, batch: int, grad_out, lr: float, beta1: float,
                      beta2: float, eps: float, step: int, stream=None) -> int:
    return lib().tbe_backward_adam(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices, batch,
                                   _ptr(grad_out), lr, beta1, beta2, eps, step, _stream_ptr(stream))


def tbe_backward_update_adagrad(h, grad_out, lr: float, eps: float, stream=None) -> int:
    return lib().tbe_backward_update_adagrad(ctypes.c_void_p(h), _ptr(grad_out), lr, eps, _stream_ptr(stream))


def tbe_backward_update_adam(h, grad_out, lr: float, beta1: float, beta2: float, eps: float, step: int,
                             stream=None) -> int:
    return lib().tbe_backward_update_adam(ctypes.c_void_p(h), _ptr(grad_out), lr, beta1, beta2, eps, step,
                                          _stream_ptr(stream))


def tbe_backward_sort(h, indices, offsets, num_indices: int, batch: int, stream=None) -> int:
    return lib().tbe_backward_sort(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices, batch,
                                   _stream_ptr(stream))


def tbe_backward_update_rowwise_adagrad(h, grad_out, lr: float, eps: float, stream=None) -> int:
    return lib().tbe_backward_update_rowwise_adagrad(ctypes.c_void_p(h), _ptr(grad_out), lr, eps,
                                                     _stream_ptr(stream))


def tbe_backward_artifacts(h):
    ps = [ctypes.c_void_p() for _ in range(5)]
    rc = lib().tbe_backward_artifacts(ctypes.c_void_p(h), *[ctypes.byref(p) for p in ps])
    return rc, [p.value for p in ps]


def tbe_check_inputs(h, indices, offsets, num_indices: int, batch: int, stream=None) -> int:
    return lib().tbe_check_inputs(ctypes.c_void_p(h), _ptr(indices), _ptr(offsets), num_indices, batch,
                                  _stream_ptr(stream))


def tbe_profile_enable(h, max_calls: int) -> int:
    return lib().tbe_profile_enable(ctypes.c_void_p(h), max_calls)


def tbe_profile_read(h) -> Tuple[int, Dict[str, Tuple[int, float]]]:
    cap = 32
    names = (ctypes.c_char_p * cap)()
    launches = (ctypes.c_int64 * cap)()
    ms = (ctypes.c_double * cap)()
    n = ctypes.c_int32()
    rc = lib().tbe_profile_read(ctypes.c_void_p(h), cap, names, launches, ms, ctypes.byref(n))
    out = {}
    if rc == TBE_OK:
        for i in range(n.value):
            out[names[i].decode()] = (int(launches[i]), float(ms[i]))
    return rc, out


def tbe_probe_read(src: torch.Tensor, nbytes: int, passes: int, sink: torch.Tensor, stream=None) -> int:
    return lib().tbe_probe_read(_ptr(src), ctypes.c_size_t(nbytes), int(passes), _ptr(sink), _stream_ptr(stream))


def tbe_last_hip_error(h) -> str:
    return lib().tbe_last_hip_error(ctypes.c_void_p(h)).decode()


# ---- input-side entry points (include/tbe_inputs.h); the caller provides every buffer ----

def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def tbe_inputs_scratch_bytes(num_bags: int) -> int:
    return int(lib().tbe_inputs_scratch_bytes(num_bags))


def tbe_lengths_to_offsets(lengths, num_bags: int, offsets, scratch, stream=None) -> int:
    return lib().tbe_lengths_to_offsets(_ptr(lengths), num_bags, _ptr(offsets), _ptr(scratch), _nbytes(scratch),
                                        _stream_ptr(stream))


def tbe_lengths_to_offsets_noalloc(lengths, num_bags: int, offsets, stream=None) -> int:
    return lib().tbe_lengths_to_offsets_noalloc(_ptr(lengths), num_bags, _ptr(offsets), _stream_ptr(stream))


def tbe_lengths_to_offsets_noalloc_max_bags() -> int:
    return int(lib().tbe_lengths_to_offsets_noalloc_max_bags())


def tbe_permute_wtb_to_twb(W: int, T: int, B: int, lengths_in, indices_in, num_indices: int, lengths_out,
                           offsets_out, indices_out, scratch, stream=None) -> int:
    return lib().tbe_permute_wtb_to_twb(W, T, B, _ptr(lengths_in), _ptr(indices_in), num_indices,
                                        _ptr(lengths_out), _ptr(offsets_out), _ptr(indices_out), _ptr(scratch),
                                        _nbytes(scratch), _stream_ptr(stream))


def tbe_bucketize_rowwise(T: int, B: int, W: int, rows, indices, offsets, num_indices: int, lengths_out,
                          offsets_out, indices_out, scratch, stream=None) -> int:
    return lib().tbe_bucketize_rowwise(T, B, W, _ptr(rows), _ptr(indices), _ptr(offsets), num_indices,
                                       _ptr(lengths_out), _ptr(offsets_out), _ptr(indices_out), _ptr(scratch),
                                       _nbytes(scratch), _stream_ptr(stream))


def _view_device(ptr: int, nbytes: int, dtype: torch.dtype, owner: torch.Tensor) -> torch.Tensor:
    """A tensor view of `nbytes` at device address `ptr`, which must lie inside `owner` (uint8)."""
    base = owner.data_ptr()
    off = ptr - base
    assert 0 <= off and off + nbytes <= owner.numel(), "pointer outside the workspace"
    return owner[off:off + nbytes].view(dtype)


class TableBatchedEmbeddingBags:
    """Convenience owner of one handle and its device buffers (allocation is torch's, compute is the library's)."""

    def __init__(self, rows, dims, weight_dtype: int, max_batch: int, max_indices: int, device="cuda:0",
                 weights: Optional[torch.Tensor] = None, optimizer: int = TBE_OPT_ROWWISE_ADAGRAD,
                 output_dtype: int = TBE_DTYPE_FP32, grad_dtype: int = TBE_DTYPE_FP32,
                 layout: int = TBE_LAYOUT_BATCH_MAJOR):
        self.rows = np.ascontiguousarray(rows, np.int64)
        self.dims = np.ascontiguousarray(dims, np.int32)
        self.T = len(self.rows)
        self.weight_dtype = weight_dtype
        self.optimizer = optimizer
        self.out_torch_dtype = _TORCH_DTYPE[output_dtype]
        self.grad_torch_dtype = _TORCH_DTYPE[grad_dtype]
        self.device = torch.device(device)
        rc, h = tbe_create(self.rows, self.dims, weight_dtype, max_batch, max_indices, optimizer=optimizer,
                           output_dtype=output_dtype, grad_dtype=grad_dtype, layout=layout)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_create")
        self.h = h
        rc, q = tbe_query_sizes(h, self.T)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_query_sizes")
        self.sizes = q
        self.sumD = int(q["out_col_offsets"][-1])
        wdt = torch.float32 if weight_dtype == TBE_DTYPE_FP32 else torch.float16
        n_w = q["weight_bytes"] // (4 if weight_dtype == TBE_DTYPE_FP32 else 2)
        if weights is None:
            weights = torch.zeros(n_w, dtype=wdt, device=self.device)
        assert weights.dtype == wdt and weights.numel() == n_w and weights.is_contiguous()
        self.weights = weights
        self.state = torch.zeros(q["state_bytes"] // 4, dtype=torch.float32, device=self.device)
        self.workspace = torch.empty(q["workspace_bytes"], dtype=torch.uint8, device=self.device)
        rc = tbe_bind(h, self.weights, self.state, self.workspace)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_bind", tbe_last_hip_error(h))

    def close(self):
        if getattr(self, "h", None):
            tbe_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def forward(self, indices, offsets, batch: int, out: Optional[torch.Tensor] = None, stream=None,
                num_indices: Optional[int] = None):
        n = indices.numel() if num_indices is None else num_indices
        if out is None:
            out = torch.empty(batch, self.sumD, dtype=self.out_torch_dtype, device=self.device)
        assert out.dtype == self.out_torch_dtype and out.is_contiguous()
        rc = tbe_forward(self.h, indices, offsets, n, batch, out, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_forward", tbe_last_hip_error(self.h))
        return out

    def backward_rowwise_adagrad(self, indices, offsets, batch: int, grad_out, lr: float, eps: float,
                                 stream=None, num_indices: Optional[int] = None):
        n = indices.numel() if num_indices is None else num_indices
        self._last_n = n
        assert grad_out.dtype == self.grad_torch_dtype and grad_out.is_contiguous()
        rc = tbe_backward_rowwise_adagrad(self.h, indices, offsets, n, batch, grad_out, lr, eps, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_rowwise_adagrad", tbe_last_hip_error(self.h))

    def backward_adagrad(self, indices, offsets, batch: int, grad_out, lr: float, eps: float, stream=None,
                         num_indices: Optional[int] = None):
        n = indices.numel() if num_indices is None else num_indices
        self._last_n = n
        assert grad_out.dtype == self.grad_torch_dtype and grad_out.is_contiguous()
        rc = tbe_backward_adagrad(self.h, indices, offsets, n, batch, grad_out, lr, eps, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_adagrad", tbe_last_hip_error(self.h))

    def backward_adam(self, indices, offsets, batch: int, grad_out, lr: float, beta1: float, beta2: float,
                      eps: float, step: int, stream=None, num_indices: Optional[int] = None):
        n = indices.numel() if num_indices is None else num_indices
        self._last_n = n
        assert grad_out.dtype == self.grad_torch_dtype and grad_out.is_contiguous()
        rc = tbe_backward_adam(self.h, indices, offsets, n, batch, grad_out, lr, beta1, beta2, eps, step, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_adam", tbe_last_hip_error(self.h))

    def backward_sort(self, indices, offsets, batch: int, stream=None, num_indices: Optional[int] = None):
        n = indices.numel() if num_indices is None else num_indices
        self._last_n = n
        rc = tbe_backward_sort(self.h, indices, offsets, n, batch, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_sort", tbe_last_hip_error(self.h))

    def backward_update_rowwise_adagrad(self, grad_out, lr: float, eps: float, stream=None):
        rc = tbe_backward_update_rowwise_adagrad(self.h, grad_out, lr, eps, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_update_rowwise_adagrad", tbe_last_hip_error(self.h))

    def backward_update_adagrad(self, grad_out, lr: float, eps: float, stream=None):
        rc = tbe_backward_update_adagrad(self.h, grad_out, lr, eps, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_update_adagrad", tbe_last_hip_error(self.h))

    def backward_update_adam(self, grad_out, lr: float, beta1: float, beta2: float, eps: float, step: int,
                             stream=None):
        rc = tbe_backward_update_adam(self.h, grad_out, lr, beta1, beta2, eps, step, stream)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_update_adam", tbe_last_hip_error(self.h))

    def check_inputs(self, indices, offsets, batch: int, num_indices: Optional[int] = None) -> int:
        n = indices.numel() if num_indices is None else num_indices
        return tbe_check_inputs(self.h, indices, offsets, n, batch)

    def artifacts(self):
        """Views (no copies) of the last backward's integer artefacts; synchronises to read U."""
        rc, ptrs = tbe_backward_artifacts(self.h)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_backward_artifacts")
        torch.cuda.synchronize(self.device)
        n = self._last_n
        nu = int(_view_device(ptrs[4], 8, torch.int64, self.workspace)[0].item())
        if n == 0:
            z = lambda dt: torch.zeros(0, dtype=dt, device=self.device)
            return dict(sorted_keys=z(torch.int32), sorted_vals=z(torch.int32), unique_keys=z(torch.int32),
                        seg_offsets=torch.zeros(1, dtype=torch.int32, device=self.device), num_unique=0)
        return dict(
            sorted_keys=_view_device(ptrs[0], 4 * n, torch.int32, self.workspace),   # uint32 bit patterns
            sorted_vals=_view_device(ptrs[1], 4 * n, torch.int32, self.workspace),
            unique_keys=_view_device(ptrs[2], 4 * nu, torch.int32, self.workspace),  # uint32 bit patterns
            seg_offsets=_view_device(ptrs[3], 4 * (nu + 1), torch.int32, self.workspace),
            num_unique=nu,
        )

    def profile_enable(self, max_calls: int):
        rc = tbe_profile_enable(self.h, max_calls)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_profile_enable", tbe_last_hip_error(self.h))

    def profile_read(self):
        rc, d = tbe_profile_read(self.h)
        if rc != TBE_OK:
            raise TbeError(rc, "tbe_profile_read", tbe_last_hip_error(self.h))
        return d
