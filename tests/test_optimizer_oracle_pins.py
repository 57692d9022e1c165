"""Pins of oracle/optimizers_oracle.py (element-wise AdaGrad, lazy sparse Adam; Section 5.1 names
them as the non-linear optimizers the fused backward must serve) against things that are not the
oracle: torch.optim on dense autograd gradients, closed forms, and the sparse-update invariants."""
import numpy as np
import pytest
import torch

from oracle import optimizers_oracle as oo
from paper_2104_05158_amd import workloads as wl


def _dense_reference(spec, idx, off, w, grad, make_opt, steps=1):
    """torch CPU float64: embedding_bag(sum) per table + autograd gives the dense weight gradient (duplicates
    aggregated by definition); torch.optim applies the update.  Valid as a reference for the SPARSE rule only
    on rows whose gradient is non-zero in every step -- the tests use cases where every row is looked up."""
    B = spec.batch
    params, outs = [], []
    woff = 0
    for t in range(spec.T):
        H, D = int(spec.rows[t]), int(spec.dims[t])
        params.append(torch.tensor(w[woff:woff + H * D].astype(np.float64).reshape(H, D), requires_grad=True))
        woff += H * D
    opt = make_opt(params)
    for _ in range(steps):
        opt.zero_grad()
        col = 0
        loss = 0.0
        for t in range(spec.T):
            D = int(spec.dims[t])
            lo, hi = int(off[t * B]), int(off[(t + 1) * B])
            o = torch.nn.functional.embedding_bag(torch.tensor(idx[lo:hi].astype(np.int64)), params[t],
                                                  torch.tensor(off[t * B:(t + 1) * B] - lo), mode="sum")
            loss = loss + (o * torch.tensor(grad[:, col:col + D].astype(np.float64))).sum()
            col += D
        loss.backward()
        opt.step()
    return np.concatenate([p.detach().numpy().ravel() for p in params])


def _all_rows_case(seed):
    """Every row of every (tiny) table is looked up, several times, also twice inside one bag."""
    rng = np.random.default_rng(seed)
    rows, dims, B = [5, 3], [8, 4], 6
    spec = wl.custom(rows, dims, 0, B, 0.0, name="allrows")
    idx, lens = [], []
    for t, H in enumerate(rows):
        for b in range(B):
            n = int(rng.integers(2, 6))
            bag = list(rng.integers(0, H, n))
            bag.append(bag[0])                      # a duplicate inside the bag
            idx += bag
            lens.append(len(bag))
        idx[-H:] = list(range(H))                   # make sure every row occurs
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.array(idx, np.int32)
    w = rng.uniform(-1, 1, spec.weight_elems).astype(np.float32)
    g = rng.normal(size=(B, spec.sumD)).astype(np.float32)
    return spec, idx, off, w, g


@pytest.mark.parametrize("seed", range(3))
def test_adagrad_matches_torch_optim_when_every_row_is_touched(seed):
    spec, idx, off, w, g = _all_rows_case(seed)
    lr, eps = 0.05, 1e-8
    ref = _dense_reference(spec, idx, off, w, g, lambda p: torch.optim.Adagrad(p, lr=lr, eps=eps), steps=2)
    w2 = w.astype(np.float64).astype(np.float32)
    st = np.zeros_like(w2)
    for _ in range(2):
        oo.backward_adagrad(spec.rows, spec.dims, 0, w2, st, idx, off, spec.batch, g, lr, eps)
    np.testing.assert_allclose(w2, ref, rtol=2e-6, atol=2e-7)


@pytest.mark.parametrize("seed", range(3))
def test_adam_matches_torch_optim_when_every_row_is_touched(seed):
    spec, idx, off, w, g = _all_rows_case(seed)
    lr, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    b1f, b2f = float(np.float32(b1)), float(np.float32(b2))   # the oracle takes the float32 values the library gets
    ref = _dense_reference(spec, idx, off, w, g,
                           lambda p: torch.optim.Adam(p, lr=float(np.float32(lr)), betas=(b1f, b2f),
                                                      eps=float(np.float32(eps))), steps=3)
    w2 = w.copy()
    m, v = np.zeros_like(w2), np.zeros_like(w2)
    for step in (1, 2, 3):
        oo.backward_adam(spec.rows, spec.dims, 0, w2, m, v, idx, off, spec.batch, g, lr, b1, b2, eps, step)
    np.testing.assert_allclose(w2, ref, rtol=3e-6, atol=3e-7)


def _one_row_case(g_row, k=1):
    """One table, row 2 looked up by k bags that all carry the gradient g_row."""
    D = len(g_row)
    spec = wl.custom([4], [D], 0, k, 0.0, name="onerow")
    idx = np.full(k, 2, np.int32)
    off = np.arange(k + 1, dtype=np.int64)
    grad = np.tile(np.asarray(g_row, np.float32), (k, 1))
    w = np.linspace(-1, 1, 4 * D).astype(np.float32)
    return spec, idx, off, w, grad


def test_adagrad_closed_forms():
    g = np.array([0.5, -2.0, 1e-5, 3.0], np.float32)
    spec, idx, off, w, grad = _one_row_case(g)
    lr, eps = 0.1, 1e-8
    w1, st = w.copy(), np.zeros_like(w)
    oo.backward_adagrad(spec.rows, spec.dims, 0, w1, st, idx, off, 1, grad, lr, eps)
    sl = slice(8, 12)
    # first step from a zero state: per ELEMENT  S = g^2, step = lr * g / (|g| + eps) ~ lr * sign(g)
    np.testing.assert_allclose(st[sl], g.astype(np.float64) ** 2, rtol=1e-7)
    np.testing.assert_allclose(w1[sl], w[sl] - 0.1 * np.sign(g), rtol=0, atol=2e-4)
    # eps outside the root matters for the 1e-5 element: 1e-5/(1e-5+1e-8) vs 1e-5/sqrt(1e-10+1e-8)
    assert abs((w[sl][2] - w1[sl][2]) / 0.1 - 1e-5 / (1e-5 + 1e-8)) < 1e-4
    # second step, same gradient: S = 2 g^2 and the step shrinks by sqrt(2)
    w2 = w1.copy()
    oo.backward_adagrad(spec.rows, spec.dims, 0, w2, st, idx, off, 1, grad, lr, eps)
    np.testing.assert_allclose(st[sl], 2 * g.astype(np.float64) ** 2, rtol=1e-6)
    np.testing.assert_allclose((w1[sl] - w2[sl])[[0, 1, 3]], (w[sl] - w1[sl])[[0, 1, 3]] / np.sqrt(2), rtol=1e-4)
    # the rule is per element, not per row: elements with different |g| take the SAME first step size
    assert np.allclose(np.abs(w[sl] - w1[sl])[[0, 1, 3]], 0.1, atol=1e-6)
    # untouched rows and their state are bit-identical
    mask = np.ones(w.size, bool)
    mask[sl] = False
    assert np.array_equal(w2[mask], w[mask]) and not st[mask].any()


def test_adam_closed_forms():
    g = np.array([0.5, -2.0, 3.0, -0.25], np.float32)
    spec, idx, off, w, grad = _one_row_case(g)
    lr, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    sl = slice(8, 12)
    w1 = w.copy()
    m, v = np.zeros_like(w), np.zeros_like(w)
    oo.backward_adam(spec.rows, spec.dims, 0, w1, m, v, idx, off, 1, grad, lr, b1, b2, eps, 1)
    # step 1 from zero moments: m_hat = g, v_hat = g^2  =>  step = lr * sign(g)
    b1f, b2f = float(np.float32(b1)), float(np.float32(b2))
    np.testing.assert_allclose(m[sl], (1 - b1f) * g, rtol=1e-6)
    np.testing.assert_allclose(v[sl], (1 - b2f) * g.astype(np.float64) ** 2, rtol=1e-6)
    np.testing.assert_allclose(w1[sl], w[sl] - 0.01 * np.sign(g), atol=1e-6)
    # a constant gradient keeps m_hat = g and v_hat = g^2: every later step is again lr * sign(g)
    w2 = w1.copy()
    oo.backward_adam(spec.rows, spec.dims, 0, w2, m, v, idx, off, 1, grad, lr, b1, b2, eps, 2)
    np.testing.assert_allclose(w2[sl], w[sl] - 0.02 * np.sign(g), atol=2e-6)
    # lazy: untouched rows keep weights and both moments
    mask = np.ones(w.size, bool)
    mask[sl] = False
    assert np.array_equal(w2[mask], w[mask]) and not m[mask].any() and not v[mask].any()
    # without bias correction the first step would be (1-b1)/sqrt(1-b2) ~ 3.16 times larger: it is not
    assert np.all(np.abs(w[sl] - w1[sl]) < 0.0101)


@pytest.mark.parametrize("which", ["adagrad", "adam"])
def test_duplicates_are_aggregated_before_the_single_step(which):
    """Section 5.1: k bags that hit the same row give ONE step with G = k*g, not k sequential steps."""
    g = np.array([1.0, -0.5, 2.0, 0.25], np.float32)
    k = 3
    spec, idx, off, w, grad = _one_row_case(g, k)
    sl = slice(8, 12)
    agg = w.copy()
    seq = w.copy()
    if which == "adagrad":
        st = np.zeros_like(w)
        oo.backward_adagrad(spec.rows, spec.dims, 0, agg, st, idx, off, k, grad, 0.1, 1e-8)
        np.testing.assert_allclose(st[sl], (k * g.astype(np.float64)) ** 2, rtol=1e-6)
        st2 = np.zeros_like(w)
        for i in range(k):
            oo.backward_adagrad(spec.rows, spec.dims, 0, seq, st2, idx[:1], off[:2], 1, grad[:1], 0.1, 1e-8)
        # one aggregated step moves by lr*sign(g); three sequential ones by lr*(1 + 1/sqrt2 + 1/sqrt3)
        np.testing.assert_allclose(np.abs(w[sl] - agg[sl]), 0.1, atol=1e-6)
        np.testing.assert_allclose(np.abs(w[sl] - seq[sl]), 0.1 * (1 + 2 ** -0.5 + 3 ** -0.5), atol=1e-5)
    else:
        m, v = np.zeros_like(w), np.zeros_like(w)
        oo.backward_adam(spec.rows, spec.dims, 0, agg, m, v, idx, off, k, grad, 0.01, 0.9, 0.999, 1e-8, 1)
        np.testing.assert_allclose(m[sl], (1 - float(np.float32(0.9))) * k * g, rtol=1e-6)
        np.testing.assert_allclose(np.abs(w[sl] - agg[sl]), 0.01, atol=1e-6)


def test_fp16_tables_round_once_to_nearest_even():
    rng = np.random.default_rng(5)
    spec = wl.custom([6], [8], 1, 4, 0.0, name="half")
    idx = np.array([0, 1, 1, 5], np.int32)
    off = np.arange(5, dtype=np.int64)
    w = rng.uniform(-1, 1, 48).astype(np.float16)
    g = rng.normal(size=(4, 8)).astype(np.float32)
    w1, st = w.copy(), np.zeros(48, np.float32)
    oo.backward_adagrad(spec.rows, spec.dims, 1, w1, st, idx, off, 4, g, 0.05, 1e-8)
    G = np.zeros((6, 8))
    for p, r in enumerate(idx):
        G[r] += g[p].astype(np.float64)
    touched = [0, 1, 5]
    for r in range(6):
        row = slice(8 * r, 8 * r + 8)
        if r in touched:
            exact = w[row].astype(np.float64) - 0.05 * G[r] / (np.abs(G[r]) + float(np.float32(1e-8)))
            assert np.array_equal(w1[row], exact.astype(np.float16))
        else:
            assert np.array_equal(w1[row], w[row])
