"""CPU oracle for the other fused sparse optimizers the paper names next to row-wise AdaGrad.

TEST INFRASTRUCTURE, NOT THE PRODUCT (numpy, float64, one Python loop over the touched rows); only
tests may call it, and it shares no code with the HIP library.

arxiv 2104.05158, Section 5.1: the backward pass is fused with the sparse optimizer, and because
"advanced optimizers like AdaGrad, LAMB and Adam" are non-linear, all gradients that reach one
embedding row are aggregated first and the optimizer runs ONCE per touched row.  The aggregation is
the same as for row-wise AdaGrad (Section 5.2) and is taken from the pinned C oracle; this file
only applies the textbook update rules to the aggregated gradient G of each touched row:

  element-wise AdaGrad   S   += G*G                      (state: one float32 per weight element)
                         w   -= lr * G / (sqrt(S) + eps)
  Adam (lazy / sparse)   m    = beta1*m + (1-beta1)*G    (state: two float32 per weight element)
                         v    = beta2*v + (1-beta2)*G*G
                         w   -= lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)

Readings where the paper is silent: states start at 0; the updated state scales the step; epsilon
sits outside the square root (as in the row-wise form); Adam is the lazy sparse variant -- rows that
are not looked up in a batch keep weights AND moments untouched -- with the global step count
`step` >= 1 supplied by the caller; no weight decay, no amsgrad.  States are stored as float32,
weights in the table's storage type, each rounded once (to nearest even) from the float64 result.
"""
from __future__ import annotations

import numpy as np

from . import tbe_oracle as orc


def aggregated_gradients(rows, dims, dtype, weights, indices, offsets, B, grad_out):
    """Per touched row (ascending linear row id): its key, and the float64 sum / sum of |terms| of the
    gradient rows of all its lookups.  Uses the pinned aggregation of oracle/tbe_oracle.c on scratch copies."""
    rows = np.asarray(rows, np.int64)
    w = np.array(weights, copy=True)
    m = np.zeros(int(rows.sum()), np.float32)
    det = orc.backward_rowwise_adagrad(rows, dims, dtype, w, m, indices, offsets, B, grad_out, 0.0, 1.0,
                                       want_detail=True)
    art = orc.sort_artifacts(rows, B, indices, offsets)
    return art.unique_keys.astype(np.int64), det.g_offsets, det.G, det.Gabs


def _row_slices(rows, dims, keys):
    rows = np.asarray(rows, np.int64)
    dims = np.asarray(dims, np.int64)
    R = np.concatenate([[0], np.cumsum(rows)])
    W = np.concatenate([[0], np.cumsum(rows * dims)])
    t = np.searchsorted(R, keys, side="right") - 1
    start = W[t] + (keys - R[t]) * dims[t]
    return start, dims[t]


def backward_adagrad(rows, dims, dtype, weights, state, indices, offsets, B, grad_out, lr, eps):
    """Element-wise AdaGrad, in place on `weights` (storage type) and `state` (float32, one per element)."""
    assert state.dtype == np.float32 and state.size == weights.size
    lr, eps = float(np.float32(lr)), float(np.float32(eps))   # the library receives them as float32
    keys, goff, G, _ = aggregated_gradients(rows, dims, dtype, weights, indices, offsets, B, grad_out)
    start, D = _row_slices(rows, dims, keys)
    for u in range(len(keys)):
        sl = slice(int(start[u]), int(start[u] + D[u]))
        g = G[goff[u]:goff[u + 1]]
        s_new = state[sl].astype(np.float64) + g * g
        w_new = weights[sl].astype(np.float64) - lr * g / (np.sqrt(s_new) + eps)
        state[sl] = s_new.astype(np.float32)
        weights[sl] = w_new.astype(weights.dtype)


def backward_adam(rows, dims, dtype, weights, m, v, indices, offsets, B, grad_out, lr, beta1, beta2, eps, step):
    """Lazy sparse Adam with bias correction, in place on `weights`, `m`, `v` (float32, one per element each)."""
    assert m.dtype == np.float32 and v.dtype == np.float32 and m.size == weights.size == v.size and step >= 1
    lr, eps = float(np.float32(lr)), float(np.float32(eps))
    beta1, beta2 = float(np.float32(beta1)), float(np.float32(beta2))
    bc1 = 1.0 - beta1 ** int(step)
    bc2 = 1.0 - beta2 ** int(step)
    keys, goff, G, _ = aggregated_gradients(rows, dims, dtype, weights, indices, offsets, B, grad_out)
    start, D = _row_slices(rows, dims, keys)
    for u in range(len(keys)):
        sl = slice(int(start[u]), int(start[u] + D[u]))
        g = G[goff[u]:goff[u + 1]]
        m_new = beta1 * m[sl].astype(np.float64) + (1.0 - beta1) * g
        v_new = beta2 * v[sl].astype(np.float64) + (1.0 - beta2) * g * g
        w_new = weights[sl].astype(np.float64) - lr * (m_new / bc1) / (np.sqrt(v_new / bc2) + eps)
        m[sl] = m_new.astype(np.float32)
        v[sl] = v_new.astype(np.float32)
        weights[sl] = w_new.astype(weights.dtype)
