"""Pins for the CPU oracle: each test checks oracle/tbe_oracle.c against something that is
NOT the oracle -- a hand-worked example, a dense count-matrix formulation, torch's CPU
embedding_bag + autograd, closed forms of one AdaGrad step, and invariants -- chosen so that a
plausible mistake (mean vs sum of squares, epsilon inside the root, old vs new moment,
sequential instead of aggregated updates, wrong table offsets, unstable sort) fails one of them.

Citations: Section 2 "Embedding operators" (forward), Section 5.1 (aggregation before the
optimizer, gradient sorting), Section 5.2 (row-wise AdaGrad), Section 7.1 (jagged input layout).
"""
import os

import numpy as np
import pytest
import torch

from oracle import tbe_oracle as orc
from paper_2104_05158_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_rowwise_adagrad.txt")


# ---------------------------------------------------------------- fp16 conversion helpers

def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.half_to_double(int(b)) for b in bits])
    both_nan = np.isnan(ref) & np.isnan(got)
    assert np.all((ref == got) | both_nan)
    assert np.all(np.signbit(ref[~both_nan]) == np.signbit(got[~both_nan]))


def test_double_to_half_matches_ieee_rounding():
    rng = np.random.default_rng(5)
    xs = np.concatenate([
        rng.uniform(-0.02, 0.02, 4000), rng.normal(size=2000), rng.uniform(-70000, 70000, 500),
        rng.uniform(-1e-4, 1e-4, 2000), rng.uniform(-1e-7, 1e-7, 500),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                  2.0 ** -14, 2.0 ** -14 - 2.0 ** -25]),
    ])
    # exact ties between neighbouring halves must go to the even mantissa
    h = rng.integers(0, 0x7BFF, 3000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    xs = np.concatenate([xs, (lo + hi) / 2, -(lo + hi) / 2])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([orc.double_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(ref, got)


# ---------------------------------------------------------------- hand-worked golden example

def _read_golden():
    d = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        d[k] = np.array([float(x) for x in v])
    return d


def test_handworked_example():
    g = _read_golden()
    rows = np.array([int(g["rows"][0])], np.int64)
    dims = np.array([int(g["dim"][0])], np.int32)
    B = 2
    w = g["weights"].astype(np.float32)
    m = np.zeros(3, np.float32)
    idx = g["indices"].astype(np.int32)
    off = g["offsets"].astype(np.int64)
    grad = g["grad"].astype(np.float32).reshape(B, 4)
    out = orc.forward(rows, dims, 0, w, idx, off, B)
    assert np.array_equal(out.ravel(), g["out"].astype(np.float32))
    art = orc.sort_artifacts(rows, B, idx, off)
    assert np.array_equal(art.sorted_keys, g["sorted_keys"].astype(np.uint32))
    assert np.array_equal(art.sorted_vals, g["sorted_vals"].astype(np.int32))
    assert np.array_equal(art.unique_keys, g["unique_keys"].astype(np.uint32))
    assert np.array_equal(art.seg_offsets, g["seg_offsets"].astype(np.int64))
    orc.backward_rowwise_adagrad(rows, dims, 0, w, m, idx, off, B, grad, g["lr"][0], g["eps"][0])
    np.testing.assert_allclose(m, g["moments_after"], rtol=1e-7)
    np.testing.assert_allclose(w, g["weights_after"], rtol=2e-7)
    assert np.array_equal(w[4:8], g["weights"][4:8].astype(np.float32))  # untouched row: bit-identical
    orc.backward_rowwise_adagrad(rows, dims, 0, w, m, idx, off, B, grad, g["lr"][0], g["eps"][0])
    np.testing.assert_allclose(m, g["moments_after2"], rtol=1e-7)
    np.testing.assert_allclose(w[8:12], g["weights_after2_row2"], rtol=3e-7)


# ---------------------------------------------------------------- P1 dense brute force

def _dense_reference(spec, indices, offsets, weights, grad, moments0, lr, eps):
    """Count-matrix formulation: out_t = C_t W_t, G_t = C_t^T grad_t, C_t[b,r] = multiplicity."""
    T, B = spec.T, spec.batch
    outs, new_w, new_m, absrefs, Gs, Gabss = [], [], [], [], [], []
    woff = col = R = 0
    for t in range(T):
        H, D = int(spec.rows[t]), int(spec.dims[t])
        W = weights[woff:woff + H * D].astype(np.float64).reshape(H, D)
        C = np.zeros((B, H))
        for b in range(B):
            for p in range(offsets[t * B + b], offsets[t * B + b + 1]):
                C[b, indices[p]] += 1.0
        outs.append(C @ W)
        absrefs.append(C @ np.abs(W))                 # sum of |terms| of every pooled value
        G = C.T @ grad[:, col:col + D].astype(np.float64)
        touched = C.sum(0) > 0
        Gs.append(G[touched].ravel())                 # touched rows ascend, tables in order = unique-key order
        Gabss.append((C.T @ np.abs(grad[:, col:col + D].astype(np.float64)))[touched].ravel())
        m = moments0[R:R + H].astype(np.float64).copy()
        m[touched] += (G[touched] ** 2).mean(1)
        Wn = W.copy()
        Wn[touched] -= lr * G[touched] / (np.sqrt(m[touched])[:, None] + eps)
        new_w.append(Wn.ravel())
        new_m.append(m)
        woff += H * D
        col += D
        R += H
    extra = dict(absref=np.concatenate(absrefs, 1), G=np.concatenate(Gs), Gabs=np.concatenate(Gabss))
    return np.concatenate(outs, 1), np.concatenate(new_w), np.concatenate(new_m), extra


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("dtype", [0, 1])
def test_dense_brute_force(seed, dtype):
    spec, idx, off, w, grad = wl.tiny_random(100 + seed, T=1 + seed % 3, dtype=dtype, dup_heavy=seed % 2 == 0)
    rng = np.random.default_rng(seed)
    m0 = rng.uniform(0, 2, spec.total_rows).astype(np.float32) * (seed % 3 != 0)
    lr, eps = float(np.float32(0.05)), float(np.float32(1e-8))
    ref_out, ref_w, ref_m, extra = _dense_reference(spec, idx, off, w, grad, m0, lr, eps)
    out, absref = orc.forward(spec.rows, spec.dims, dtype, w, idx, off, spec.batch, want_absref=True)
    np.testing.assert_allclose(out, ref_out.astype(np.float32), rtol=0, atol=0)
    assert np.all(absref + 1e-12 >= np.abs(ref_out))
    # the scale every GPU forward comparison divides by is exactly |C| . |W| (sums of a few fp64 terms:
    # equal up to the order of the additions)
    np.testing.assert_allclose(absref, extra["absref"], rtol=1e-14, atol=0)
    w2, m2 = w.copy(), m0.copy()
    det = orc.backward_rowwise_adagrad(spec.rows, spec.dims, dtype, w2, m2, idx, off, spec.batch, grad, lr, eps,
                                       want_detail=True)
    assert np.array_equal(m2, ref_m.astype(np.float32))
    wdt = np.float32 if dtype == 0 else np.float16
    assert np.array_equal(w2, ref_w.astype(wdt))
    # detail outputs are consistent with the update that was applied
    assert det.g_offsets[-1] == det.G.size and np.all(det.Gabs + 1e-12 >= np.abs(det.G))
    # the per-row aggregated gradient and the scale of every GPU update comparison are exactly
    # C^T . grad and C^T . |grad|, in unique-key order
    assert det.G.size == extra["G"].size
    np.testing.assert_allclose(det.G, extra["G"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(det.Gabs, extra["Gabs"], rtol=1e-14, atol=0)


# ---------------------------------------------------------------- P2 torch embedding_bag + autograd

@pytest.mark.parametrize("seed", range(4))
def test_against_torch_embedding_bag(seed):
    rng = np.random.default_rng(seed)
    H, D, B = 37, 12, 9
    lens = rng.integers(0, 7, B)
    off = np.zeros(B + 1, np.int64)
    off[1:] = np.cumsum(lens)
    idx = rng.integers(0, H, off[-1]).astype(np.int32)
    w = rng.normal(size=(H, D)).astype(np.float32)
    grad = rng.normal(size=(B, D)).astype(np.float32)
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    tout = torch.nn.functional.embedding_bag(torch.tensor(idx, dtype=torch.int64), tw,
                                             torch.tensor(off[:-1]), mode="sum")
    tout.backward(torch.tensor(grad, dtype=torch.float64))
    rows, dims = np.array([H], np.int64), np.array([D], np.int32)
    out = orc.forward(rows, dims, 0, w.ravel(), idx, off, B)
    assert np.array_equal(out, tout.detach().numpy().astype(np.float32))
    w2, m2 = w.ravel().copy(), np.zeros(H, np.float32)
    det = orc.backward_rowwise_adagrad(rows, dims, 0, w2, m2, idx, off, B, grad, 0.1, 1e-8, want_detail=True)
    dense = tw.grad.numpy()
    art = orc.sort_artifacts(rows, B, idx, off)
    assert np.array_equal(np.flatnonzero(np.abs(dense).sum(1) > 0), art.unique_keys[np.abs(det.G.reshape(-1, D)).sum(1) > 0])
    np.testing.assert_allclose(det.G.reshape(-1, D), dense[art.unique_keys], rtol=1e-14, atol=1e-14)


# ---------------------------------------------------------------- P3 pure gather

@pytest.mark.parametrize("dtype", [0, 1])
def test_pooling_one_unique_is_pure_gather(dtype):
    rng = np.random.default_rng(3)
    spec = wl.custom([50, 20], [8, 4], dtype, 16, 1.0)
    wdt = np.float32 if dtype == 0 else np.float16
    w = rng.normal(size=spec.weight_elems).astype(wdt)
    idx = np.concatenate([rng.permutation(50)[:16], rng.permutation(20)[:16]]).astype(np.int32)
    off = np.arange(2 * 16 + 1, dtype=np.int64)
    out = orc.forward(spec.rows, spec.dims, dtype, w, idx, off, 16)
    w0 = w[:400].reshape(50, 8)
    w1 = w[400:].reshape(20, 4)
    assert np.array_equal(out[:, :8], w0[idx[:16]].astype(np.float32))
    assert np.array_equal(out[:, 8:], w1[idx[16:]].astype(np.float32))


# ---------------------------------------------------------------- P4 closed forms of one step

def _single_row_step(g, lr, eps, steps=1, D=None, m0=0.0, w0=None):
    D = len(g)
    rows, dims = np.array([1], np.int64), np.array([D], np.int32)
    w = np.zeros(D, np.float32) if w0 is None else np.asarray(w0, np.float32).copy()
    m = np.array([m0], np.float32)
    for _ in range(steps):
        orc.backward_rowwise_adagrad(rows, dims, 0, w, m, np.zeros(1, np.int32), np.array([0, 1], np.int64), 1,
                                     np.asarray(g, np.float32).reshape(1, D), lr, eps)
    return w, m


def test_closed_form_one_step_mean_of_squares():
    g = np.array([0.5, -1.0, 2.0, 0.25, 0.0, 3.0, -0.125, 1.0], np.float32)
    lr, eps = 0.01, 1e-8
    w, m = _single_row_step(g, lr, eps, w0=np.ones(8))
    ms = float((g.astype(np.float64) ** 2).mean())
    assert m[0] == np.float32(ms)                                   # mean, not sum, of squares
    assert abs(m[0] - float((g.astype(np.float64) ** 2).sum())) > 1
    np.testing.assert_allclose(w, 1.0 - lr * g / (np.sqrt(ms) + float(np.float32(eps))), rtol=1e-7)


def test_closed_form_constant_gradient_is_sign_step():
    for c in (3.0, -0.2):
        w, m = _single_row_step(np.full(16, c), 0.01, 1e-8)
        np.testing.assert_allclose(w, -0.01 * np.sign(c), rtol=1e-6)  # lr*c/(|c|+eps)
        np.testing.assert_allclose(m[0], c * c, rtol=1e-6)


def test_closed_form_two_steps_moment_doubles():
    g = np.array([1.0, 2.0, 3.0, 4.0])
    w1, m1 = _single_row_step(g, 0.1, 0.0, steps=1)
    w2, m2 = _single_row_step(g, 0.1, 0.0, steps=2)
    np.testing.assert_allclose(m2, 2 * m1, rtol=1e-7)
    # second step is 1/sqrt(2) of the first: the UPDATED moment scales the step
    np.testing.assert_allclose(w2 - w1, w1 / np.sqrt(2.0), rtol=1e-6)


def test_epsilon_sits_outside_the_square_root():
    # |g| = 1e-5 and eps = 1e-8: sqrt(m)+eps = 1.001e-5, whereas sqrt(m+eps) ~ 1.005e-4 (10x smaller step)
    c = 1e-5
    w, _ = _single_row_step(np.full(4, c), 0.01, 1e-8)
    expect = -0.01 * c / (c + 1e-8)
    np.testing.assert_allclose(w, expect, rtol=1e-4)
    assert abs(w[0] - (-0.01 * c / np.sqrt(c * c + 1e-8))) > 0.5 * abs(expect)


def test_nonzero_initial_moment_is_used():
    g = np.array([2.0, 0.0, 0.0, 0.0])
    w, m = _single_row_step(g, 1.0, 0.0, m0=3.0)
    assert m[0] == 4.0 and w[0] == -1.0


# ---------------------------------------------------------------- P5 aggregate, then one step

def test_duplicates_aggregate_before_the_optimizer():
    D, k = 8, 5
    rng = np.random.default_rng(0)
    g = rng.normal(size=D).astype(np.float32)
    rows, dims = np.array([4], np.int64), np.array([D], np.int32)
    # row 2 appears in k different bags, each bag receiving the same upstream gradient g
    idx = np.full(k, 2, np.int32)
    off = np.arange(k + 1, dtype=np.int64)
    grad = np.tile(g, (k, 1))
    w, m = np.zeros(4 * D, np.float32), np.zeros(4, np.float32)
    orc.backward_rowwise_adagrad(rows, dims, 0, w, m, idx, off, k, grad, 0.01, 0.0)
    ms = float((g.astype(np.float64) ** 2).mean())
    np.testing.assert_allclose(m[2], k * k * ms, rtol=1e-6)          # (k g)^2, not k g^2
    one = -0.01 * g / np.sqrt(ms)
    np.testing.assert_allclose(w[2 * D:3 * D], one, rtol=1e-6)       # k g / (k sqrt(ms)) == single step
    seq = sum(1.0 / np.sqrt(i) for i in range(1, k + 1))              # what k sequential steps would give
    assert np.all(np.abs(w[2 * D:3 * D] - seq * one) > 0.5 * np.abs(one))
    assert not w[:2 * D].any() and not w[3 * D:].any() and m[0] == m[1] == m[3] == 0


def test_same_row_twice_in_one_bag_counts_twice():
    rows, dims = np.array([3], np.int64), np.array([4], np.int32)
    w = np.arange(12, dtype=np.float32)
    idx, off = np.array([1, 1, 1], np.int32), np.array([0, 3], np.int64)
    out = orc.forward(rows, dims, 0, w, idx, off, 1)
    assert np.array_equal(out[0], 3 * w[4:8])
    grad = np.array([[1, -1, 2, 0]], np.float32)
    w2, m = w.copy(), np.zeros(3, np.float32)
    det = orc.backward_rowwise_adagrad(rows, dims, 0, w2, m, idx, off, 1, grad, 0.1, 0.0, want_detail=True)
    assert np.array_equal(det.G, 3.0 * grad[0])


# ---------------------------------------------------------------- sort artefacts vs a library stable sort

@pytest.mark.parametrize("seed", range(6))
def test_sort_artifacts_against_numpy_stable_sort(seed):
    spec, idx, off, _, _ = wl.tiny_random(seed, T=4, max_rows=9, B=7, max_len=6)
    T, B = spec.T, spec.batch
    R = np.concatenate([[0], np.cumsum(spec.rows)])
    lens = np.diff(off)
    bag = np.repeat(np.arange(T * B), lens)
    keys = (R[bag // B] + idx).astype(np.uint32)
    order = np.argsort(keys, kind="stable")
    art = orc.sort_artifacts(spec.rows, B, idx, off)
    assert np.array_equal(art.sorted_keys, keys[order])
    assert np.array_equal(art.sorted_vals, (bag % B)[order].astype(np.int32))
    uk, first, counts = np.unique(keys[order], return_index=True, return_counts=True)
    assert art.num_unique == len(uk)
    assert np.array_equal(art.unique_keys, uk)
    assert np.array_equal(art.seg_offsets[:-1], first) and art.seg_offsets[-1] == len(keys)
    assert np.array_equal(np.diff(art.seg_offsets), counts)


# ---------------------------------------------------------------- P6 invariants, P7 independence

def _cfg_small(seed, dtype):
    spec = wl.custom([300, 41, 1000], [8, 16, 4], dtype, 24, [3.0, 6.0, 1.0], index_dist="zipf", name="inv")
    batch = wl.make_batch(spec, "cpu", seed=seed)
    w = wl.make_weights(spec, "cpu", seed=seed + 1).numpy()
    grad = wl.make_grad(spec, "cpu", seed=seed + 2).numpy()
    return spec, batch.indices.numpy(), batch.offsets.numpy(), w, grad


@pytest.mark.parametrize("dtype", [0, 1])
def test_invariants(dtype):
    spec, idx, off, w, grad = _cfg_small(11, dtype)
    B, T = spec.batch, spec.T
    out = orc.forward(spec.rows, spec.dims, dtype, w, idx, off, B)
    # permuting the indices inside every bag leaves the output unchanged up to fp64 summation order
    rng = np.random.default_rng(0)
    idx_p = idx.copy()
    for j in range(T * B):
        idx_p[off[j]:off[j + 1]] = rng.permutation(idx[off[j]:off[j + 1]])
    np.testing.assert_allclose(orc.forward(spec.rows, spec.dims, dtype, w, idx_p, off, B), out, rtol=1e-6, atol=1e-9)
    # column sums: sum_b out[b] == sum_r count_r W[r]
    woff = col = 0
    for t in range(T):
        H, D = int(spec.rows[t]), int(spec.dims[t])
        cnt = np.bincount(idx[off[t * B]:off[(t + 1) * B]], minlength=H).astype(np.float64)
        W = w[woff:woff + H * D].astype(np.float64).reshape(H, D)
        np.testing.assert_allclose(out[:, col:col + D].astype(np.float64).sum(0), cnt @ W, rtol=1e-5, atol=1e-6)
        woff += H * D
        col += D
    # linearity (exact for a power of two)
    np.testing.assert_array_equal(orc.forward(spec.rows, spec.dims, dtype, (w * 2).astype(w.dtype), idx, off, B), 2 * out)
    # backward: moments never decrease, untouched rows are bit-identical, counts add up
    w2, m = w.copy(), np.zeros(spec.total_rows, np.float32)
    orc.backward_rowwise_adagrad(spec.rows, spec.dims, dtype, w2, m, idx, off, B, grad, 0.01, 1e-8)
    art = orc.sort_artifacts(spec.rows, B, idx, off)
    assert np.all(m >= 0) and np.count_nonzero(m) <= art.num_unique
    touched_rows = np.zeros(spec.total_rows, bool)
    touched_rows[art.unique_keys] = True
    assert not m[~touched_rows].any()
    rowid = np.concatenate([np.repeat(np.arange(int(h)), int(d)) + r0 for h, d, r0 in
                            zip(spec.rows, spec.dims, np.concatenate([[0], np.cumsum(spec.rows)[:-1]]))])
    assert np.array_equal(w2[~touched_rows[rowid]].view(np.uint8), w[~touched_rows[rowid]].view(np.uint8))
    assert np.all(np.diff(art.seg_offsets) > 0) and np.all(np.diff(art.unique_keys.astype(np.int64)) > 0)
    assert art.seg_offsets[-1] == len(idx) == off[-1]


def test_empty_bags_and_empty_batch():
    rows, dims = np.array([5, 7], np.int64), np.array([4, 8], np.int32)
    w = np.ones(5 * 4 + 7 * 8, np.float32)
    B = 3
    off = np.array([0, 0, 2, 2, 2, 2, 3], np.int64)  # table0: [], [a,b], []; table1: [], [], [c]
    idx = np.array([1, 4, 6], np.int32)
    out = orc.forward(rows, dims, 0, w, idx, off, B)
    assert np.array_equal(out[:, :4], np.array([[0] * 4, [2] * 4, [0] * 4], np.float32))
    assert np.array_equal(out[:, 4:], np.array([[0] * 8, [0] * 8, [1] * 8], np.float32))
    art = orc.sort_artifacts(rows, B, idx, off)
    assert art.sorted_keys.tolist() == [1, 4, 11] and art.sorted_vals.tolist() == [1, 1, 2]
    off0 = np.zeros(2 * B + 1, np.int64)
    out0 = orc.forward(rows, dims, 0, w, np.zeros(0, np.int32), off0, B)
    assert not out0.any()
    w2, m = w.copy(), np.zeros(12, np.float32)
    orc.backward_rowwise_adagrad(rows, dims, 0, w2, m, np.zeros(0, np.int32), off0, B, np.ones((B, 12), np.float32), 0.1, 1e-8)
    assert np.array_equal(w2, w) and not m.any()
    assert orc.sort_artifacts(rows, B, np.zeros(0, np.int32), off0).num_unique == 0


@pytest.mark.parametrize("dtype", [0, 1])
def test_tables_are_independent(dtype):
    spec, idx, off, w, grad = _cfg_small(23, dtype)
    B = spec.batch
    out = orc.forward(spec.rows, spec.dims, dtype, w, idx, off, B)
    w_all, m_all = w.copy(), np.zeros(spec.total_rows, np.float32)
    orc.backward_rowwise_adagrad(spec.rows, spec.dims, dtype, w_all, m_all, idx, off, B, grad, 0.01, 1e-8)
    t = 1
    lo, hi = off[t * B], off[(t + 1) * B]
    wlo = int(spec.rows[0]) * int(spec.dims[0])
    whi = wlo + int(spec.rows[1]) * int(spec.dims[1])
    c0, c1 = int(spec.dims[0]), int(spec.dims[0] + spec.dims[1])
    sub_rows, sub_dims = spec.rows[1:2], spec.dims[1:2]
    sub_off = (off[t * B:(t + 1) * B + 1] - lo).astype(np.int64)
    out1 = orc.forward(sub_rows, sub_dims, dtype, w[wlo:whi].copy(), idx[lo:hi].copy(), sub_off, B)
    assert np.array_equal(out1, out[:, c0:c1])
    w1, m1 = w[wlo:whi].copy(), np.zeros(int(spec.rows[1]), np.float32)
    orc.backward_rowwise_adagrad(sub_rows, sub_dims, dtype, w1, m1, idx[lo:hi].copy(), sub_off, B,
                                 np.ascontiguousarray(grad[:, c0:c1]), 0.01, 1e-8)
    assert np.array_equal(w1, w_all[wlo:whi])
    assert np.array_equal(m1, m_all[int(spec.rows[0]):int(spec.rows[0] + spec.rows[1])])


def test_bad_inputs_are_rejected():
    rows, dims = np.array([4], np.int64), np.array([4], np.int32)
    w = np.zeros(16, np.float32)
    with pytest.raises(ValueError):
        orc.forward(rows, dims, 0, w, np.array([4], np.int32), np.array([0, 1], np.int64), 1)
    with pytest.raises(ValueError):
        orc.forward(rows, dims, 0, w, np.array([-1], np.int32), np.array([0, 1], np.int64), 1)
