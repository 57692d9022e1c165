"""Shared helpers of the GPU parity tests: run one step through the C-ABI library and through the
CPU oracle on the same seeded inputs, and compare with the stated tolerances.

Tolerances (relative, measured against the condition-aware scale sum|terms|, because a plain |ref|
denominator is meaningless when a sum of N(0,1) terms cancels):
    fp32 tables:          1e-5
    fp16-stored tables:   2e-3  (fp32 accumulation; the write-back rounds to fp16)
The forward pass converts fp16 exactly to fp32, so it is held to 1e-5 for both storage types.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import tbe_oracle as orc
from paper_2104_05158_amd import tbe

RTOL_FP32 = 1e-5
RTOL_FP16 = 2e-3


def rtol_for(dtype: int) -> float:
    return RTOL_FP32 if dtype == 0 else RTOL_FP16


def make_op(spec, device, max_batch=None, max_indices=None, weights=None, layout=0):
    return tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, spec.dtype,
                                         spec.batch if max_batch is None else max_batch,
                                         max_indices, device=device, weights=weights, layout=layout)


def to_table_major(x: np.ndarray, dims) -> np.ndarray:
    """[B, sumD] rows -> the flat array that holds one contiguous [B, D_t] block per table, in table order."""
    cols = np.concatenate([[0], np.cumsum(dims)]).astype(np.int64)
    return np.concatenate([np.ascontiguousarray(x[:, cols[t]:cols[t + 1]]).ravel() for t in range(len(dims))])


def from_table_major(flat: np.ndarray, batch: int, dims) -> np.ndarray:
    cols = np.concatenate([[0], np.cumsum(dims)]).astype(np.int64)
    out = np.empty((batch, int(cols[-1])), flat.dtype)
    for t in range(len(dims)):
        out[:, cols[t]:cols[t + 1]] = flat[batch * cols[t]:batch * cols[t + 1]].reshape(batch, int(dims[t]))
    return out


def assert_forward_close(gpu_out: np.ndarray, ref_out: np.ndarray, absref: np.ndarray, what=""):
    err = np.abs(gpu_out.astype(np.float64) - ref_out.astype(np.float64))
    scale = np.maximum(np.abs(ref_out.astype(np.float64)), absref)
    bad = err > RTOL_FP32 * scale + 1e-30
    assert not bad.any(), f"forward mismatch {what}: {bad.sum()} elements, max rel {np.max(err / (scale + 1e-30)):.3e}"
    return float(np.max(err / (scale + 1e-300)))


def assert_artifacts_equal(gpu_art: dict, ref: orc.SortArtifacts, what=""):
    assert gpu_art["num_unique"] == ref.num_unique, f"num_unique {what}"
    sk = gpu_art["sorted_keys"].cpu().numpy().view(np.uint32)
    sv = gpu_art["sorted_vals"].cpu().numpy()
    uk = gpu_art["unique_keys"].cpu().numpy().view(np.uint32)
    so = gpu_art["seg_offsets"].cpu().numpy()
    assert np.array_equal(sk, ref.sorted_keys), f"sorted_keys {what}"
    assert np.array_equal(sv, ref.sorted_vals), f"sorted_vals {what}"
    assert np.array_equal(uk, ref.unique_keys), f"unique_keys {what}"
    assert np.array_equal(so.astype(np.int64), ref.seg_offsets), f"seg_offsets {what}"
    counts = np.diff(so.astype(np.int64))
    assert np.array_equal(counts, np.diff(ref.seg_offsets)), f"counts {what}"


def oracle_step(spec, indices, offsets, w0: np.ndarray, m0: np.ndarray, grad: np.ndarray, lr, eps):
    """Forward on w0, then backward in place on copies.  Returns a dict of everything to compare."""
    B = spec.batch
    out, absref = orc.forward(spec.rows, spec.dims, spec.dtype, w0, indices, offsets, B, want_absref=True)
    w1, m1 = w0.copy(), m0.copy()
    det = orc.backward_rowwise_adagrad(spec.rows, spec.dims, spec.dtype, w1, m1, indices, offsets, B, grad,
                                       lr, eps, want_detail=True)
    art = orc.sort_artifacts(spec.rows, B, indices, offsets)
    return dict(out=out, absref=absref, w1=w1, m1=m1, det=det, art=art)


def assert_update_close(spec, ref: dict, w0: np.ndarray, m0: np.ndarray, gpu_w: np.ndarray, gpu_m: np.ndarray,
                        lr: float, eps: float, what=""):
    """Touched rows within tolerance, untouched rows bit-identical."""
    det, art = ref["det"], ref["art"]
    rtol = rtol_for(spec.dtype)
    R = np.concatenate([[0], np.cumsum(spec.rows)])
    woffs = np.concatenate([[0], np.cumsum(spec.rows * spec.dims.astype(np.int64))])
    lr = float(np.float32(lr))
    eps = float(np.float32(eps))
    keys = art.unique_keys.astype(np.int64)
    tab = np.searchsorted(R, keys, side="right") - 1
    worst_w = worst_m = 0.0
    gpu_w_masked = gpu_w.copy()
    for t in np.unique(tab):
        t = int(t)
        sel = np.flatnonzero(tab == t)          # contiguous: keys ascend
        u0, u1 = int(sel[0]), int(sel[-1]) + 1
        D, H = int(spec.dims[t]), int(spec.rows[t])
        r = keys[u0:u1] - R[t]
        gabs = det.Gabs[det.g_offsets[u0]:det.g_offsets[u1]].reshape(-1, D)
        m_new = det.m_new[u0:u1]
        W0 = w0[woffs[t]:woffs[t + 1]].reshape(H, D)
        Wg = gpu_w[woffs[t]:woffs[t + 1]].reshape(H, D)
        Wr = ref["w1"][woffs[t]:woffs[t + 1]].reshape(H, D)
        scale_w = np.abs(W0[r].astype(np.float64)) + lr * gabs / (np.sqrt(m_new)[:, None] + eps)
        err_w = np.abs(Wg[r].astype(np.float64) - Wr[r].astype(np.float64))
        # a result on a rounding boundary of the storage type may differ by one unit in the last
        # place; the tolerance class covers it (fp16 ulp 4.9e-4 relative, fp32 1.2e-7)
        rel = err_w / (scale_w + 1e-300)
        i = np.unravel_index(np.argmax(rel), rel.shape)
        assert rel[i] <= rtol, f"weights {what}: table {t} row {r[i[0]]} col {i[1]} rel err {rel[i]:.3e}"
        worst_w = max(worst_w, float(rel[i]))
        scale_m = m0[keys[u0:u1]].astype(np.float64) + (gabs ** 2).mean(1)
        rel_m = np.abs(gpu_m[keys[u0:u1]].astype(np.float64) - ref["m1"][keys[u0:u1]].astype(np.float64)) / (scale_m + 1e-300)
        j = int(np.argmax(rel_m))
        assert rel_m[j] <= RTOL_FP32, f"moment {what}: table {t} row {r[j]} rel err {rel_m[j]:.3e}"
        worst_m = max(worst_m, float(rel_m[j]))
        # put the original bits back into the touched rows so that one whole-array comparison
        # below proves that nothing else was written
        gpu_w_masked[woffs[t]:woffs[t + 1]].reshape(H, D)[r] = W0[r]
    assert np.array_equal(gpu_w_masked.view(np.uint8), w0.view(np.uint8)), f"untouched weights changed {what}"
    tm = np.zeros(m0.size, bool)
    tm[keys] = True
    assert np.array_equal(gpu_m[~tm], m0[~tm]), f"untouched moments changed {what}"
    return worst_w, worst_m


def full_parity_step(spec, indices: np.ndarray, offsets: np.ndarray, w0: np.ndarray, grad: np.ndarray, device,
                     lr=0.01, eps=1e-8, m0=None, what="", check_inputs=True, layout=0):
    """One forward + one backward through the C ABI, every output compared with the oracle.
    With layout=1 the library writes its output and reads the gradient table-major; the oracle
    always works on [B, sumD] rows and the conversion happens here, on the host."""
    B = spec.batch
    N = int(offsets[-1])
    if m0 is None:
        m0 = np.zeros(spec.total_rows, np.float32)
    ref = oracle_step(spec, indices, offsets, w0, m0, grad, lr, eps)
    op = make_op(spec, device, max_indices=max(N, 1), weights=torch.from_numpy(w0.copy()).to(device), layout=layout)
    op.state.copy_(torch.from_numpy(m0))
    d_idx = torch.from_numpy(indices).to(device)
    d_off = torch.from_numpy(offsets).to(device)
    d_grad = torch.from_numpy(to_table_major(grad, spec.dims) if layout else grad).to(device)
    if check_inputs:
        assert op.check_inputs(d_idx, d_off, B, num_indices=N) == tbe.TBE_OK
    out = op.forward(d_idx, d_off, B, num_indices=N)
    torch.cuda.synchronize()
    h_out = out.cpu().numpy()
    if layout:
        h_out = from_table_major(h_out.ravel(), B, spec.dims)
    fwd_err = assert_forward_close(h_out, ref["out"], ref["absref"], what)
    op.backward_rowwise_adagrad(d_idx, d_off, B, d_grad, lr, eps, num_indices=N)
    art = op.artifacts()
    assert_artifacts_equal(art, ref["art"], what)
    gw = op.weights.cpu().numpy()
    gm = op.state.cpu().numpy()
    ww, wm = assert_update_close(spec, ref, w0, m0, gw, gm, lr, eps, what)
    op.close()
    return dict(fwd_err=fwd_err, w_err=ww, m_err=wm, num_unique=ref["art"].num_unique, N=N)
