"""GPU parity of the configurations the benchmark times but the single-step tests do not reach:

  * ONE handle created for a larger batch and more lookups than any call passes, fed several batches of
    different batch size and lookup count one after another (the rotation bench.py runs), both layouts;
  * float16 output + bfloat16 gradient + table-major layout together;
  * the two-call backward (tbe_backward_sort + tbe_backward_update_<optimizer>) against the one-call
    form for all three optimizers, an update repeated after one sort, and tbe_check_inputs between the two;
  * a well-conditioned case (positive weights and gradients, nothing cancels) held to the PLAIN relative
    tolerance 1e-5 / 2e-3, where the condition-aware scale of the other tests cannot hide lost low-order bits.

Every float comparison is against the CPU oracle on the same seeded inputs, through the C ABI; integer
artefacts are compared bit-exactly.
"""
import dataclasses

import numpy as np
import pytest
import torch

import tbe_testlib as tl
from oracle import tbe_oracle as orc
from paper_2104_05158_amd import tbe
from paper_2104_05158_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _base_spec(dtype):
    return wl.custom([5000, 300, 20000, 64], [128, 32, 64, 256], dtype, 700, [20.0, 4.0, 30.0, 3.0],
                     index_dist="zipf", zipf_s=1.1, name="variants")


def _step_and_check(op, spec, b, w_prev, m_prev, grad32, dev, layout=0, out16=False, grad_dtype=tbe.TBE_DTYPE_FP32,
                    lr=0.02, eps=1e-8, what=""):
    """One forward + backward of `spec`'s batch `b` on an existing handle, everything compared with the oracle
    started from (w_prev, m_prev).  grad32: float32 [B, sumD] holding exactly the values the library is given."""
    idx, off = b.indices.numpy(), b.offsets.numpy()
    B, N = spec.batch, b.num_indices
    ref = tl.oracle_step(spec, idx, off, w_prev, m_prev, grad32, lr, eps)
    d_idx = torch.from_numpy(idx).to(dev) if N else torch.zeros(1, dtype=torch.int32, device=dev)
    d_off = torch.from_numpy(off).to(dev)
    g = tl.to_table_major(grad32, spec.dims) if layout else grad32
    d_grad = torch.from_numpy(np.ascontiguousarray(g)).to(dev).to(tbe._TORCH_DTYPE[grad_dtype])
    assert op.check_inputs(d_idx, d_off, B, num_indices=N) == tbe.TBE_OK
    out = torch.full((B * spec.sumD,), float("nan"), dtype=op.out_torch_dtype, device=dev).view(B, spec.sumD)
    op.forward(d_idx, d_off, B, out=out, num_indices=N)
    torch.cuda.synchronize()
    h_out = out.float().cpu().numpy()
    if layout:
        h_out = tl.from_table_major(h_out.ravel(), B, spec.dims)
    if out16:
        r64 = ref["out"].astype(np.float64)
        tol = tl.RTOL_FP32 * np.maximum(np.abs(r64), ref["absref"]) + 2.0 ** -11 * np.abs(r64) + 2.0 ** -25
        assert (np.abs(h_out.astype(np.float64) - r64) <= tol).all(), f"fp16 output {what}"
    else:
        tl.assert_forward_close(h_out, ref["out"], ref["absref"], what)
    op.backward_rowwise_adagrad(d_idx, d_off, B, d_grad, lr, eps, num_indices=N)
    tl.assert_artifacts_equal(op.artifacts(), ref["art"], what)
    gw, gm = op.weights.cpu().numpy(), op.state.cpu().numpy()
    tl.assert_update_close(spec, ref, w_prev, m_prev, gw, gm, lr, eps, what)
    return gw, gm


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("dtype", [0, 1])
def test_one_handle_many_batches(gpu_device, dtype, layout):
    """max_batch > batch and max_indices > N in every call; N and B go down, up, to one bag, to an empty
    batch of lookups and back up, so stale tile plans, histograms and artefacts of a larger earlier call sit
    in the workspace behind every later one."""
    dev = gpu_device
    base = _base_spec(dtype)
    plan = [(700, 1.0), (333, 0.4), (512, 2.2), (1, 1.0), (64, 0.0), (700, 1.3)]     # (batch, pooling scale)
    specs = [dataclasses.replace(base, batch=B, pooling_mean=base.pooling_mean * s, name=f"reuse{i}")
             for i, (B, s) in enumerate(plan)]
    batches = [wl.make_batch(s, "cpu", seed=40 + i) for i, s in enumerate(specs)]
    n_max = max(b.num_indices for b in batches)
    assert batches[4].num_indices == 0
    w = wl.make_weights(base, "cpu", seed=2).numpy()
    m = np.zeros(base.total_rows, np.float32)
    op = tbe.TableBatchedEmbeddingBags(base.rows, base.dims, dtype, 1024, 2 * n_max + 12345, device=dev,
                                       weights=torch.from_numpy(w.copy()).to(dev), layout=layout)
    for i, (s, b) in enumerate(zip(specs, batches)):
        print(f"reuse step {i}: B={s.batch} N={b.num_indices} layout={layout} dtype={dtype}", flush=True)
        g = wl.make_grad(s, "cpu", seed=70 + i).numpy()
        w, m = _step_and_check(op, s, b, w, m, g, dev, layout=layout, what=f"reuse step {i}")
    op.close()


@pytest.mark.parametrize("dtype", [0, 1])
def test_fp16_output_bf16_gradient_table_major_together(gpu_device, dtype):
    dev = gpu_device
    spec = _base_spec(dtype)
    b = wl.make_batch(spec, "cpu", seed=5)
    w = wl.make_weights(spec, "cpu", seed=6).numpy()
    m = np.zeros(spec.total_rows, np.float32)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, dtype, spec.batch + 100, b.num_indices + 999, device=dev,
                                       weights=torch.from_numpy(w.copy()).to(dev), output_dtype=tbe.TBE_DTYPE_FP16,
                                       grad_dtype=tbe.TBE_DTYPE_BF16, layout=tbe.TBE_LAYOUT_TABLE_MAJOR)
    for step in range(2):
        # the oracle gets the float32 values of exactly the bfloat16 numbers the library reads
        g = torch.from_numpy(wl.make_grad(spec, "cpu", seed=7 + step).numpy()).to(torch.bfloat16).float().numpy()
        w, m = _step_and_check(op, spec, b, w, m, g, dev, layout=1, out16=True, grad_dtype=tbe.TBE_DTYPE_BF16,
                               what=f"all three, step {step}")
    op.close()


def _make_op(spec, w0, dev, optimizer, N):
    return tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, spec.dtype, spec.batch, N, device=dev,
                                         weights=torch.from_numpy(w0.copy()).to(dev), optimizer=optimizer)


@pytest.mark.parametrize("optimizer", [tbe.TBE_OPT_ROWWISE_ADAGRAD, tbe.TBE_OPT_ADAGRAD, tbe.TBE_OPT_ADAM])
@pytest.mark.parametrize("dtype", [0, 1])
def test_two_call_backward_equals_one_call(gpu_device, optimizer, dtype):
    """tbe_backward_sort + tbe_backward_update_<optimizer> run the same kernels as tbe_backward_<optimizer>
    (itself checked against the oracle elsewhere): weights, states and artefacts must be bit-identical, also
    with tbe_check_inputs called between the two halves."""
    dev = gpu_device
    spec = _base_spec(dtype)
    b = wl.make_batch(spec, "cpu", seed=11)
    w0 = wl.make_weights(spec, "cpu", seed=12).numpy()
    N, B = b.num_indices, spec.batch
    d_idx, d_off = b.indices.to(dev), b.offsets.to(dev)
    one, two = _make_op(spec, w0, dev, optimizer, N), _make_op(spec, w0, dev, optimizer, N)
    for step in (1, 2):
        g = wl.make_grad(spec, "cpu", seed=20 + step).to(dev)
        if optimizer == tbe.TBE_OPT_ROWWISE_ADAGRAD:
            one.backward_rowwise_adagrad(d_idx, d_off, B, g, 0.03, 1e-8, num_indices=N)
        elif optimizer == tbe.TBE_OPT_ADAGRAD:
            one.backward_adagrad(d_idx, d_off, B, g, 0.03, 1e-8, num_indices=N)
        else:
            one.backward_adam(d_idx, d_off, B, g, 0.03, 0.9, 0.999, 1e-8, step, num_indices=N)
        two.backward_sort(d_idx, d_off, B, num_indices=N)
        assert two.check_inputs(d_idx, d_off, B, num_indices=N) == tbe.TBE_OK
        if optimizer == tbe.TBE_OPT_ROWWISE_ADAGRAD:
            two.backward_update_rowwise_adagrad(g, 0.03, 1e-8)
        elif optimizer == tbe.TBE_OPT_ADAGRAD:
            two.backward_update_adagrad(g, 0.03, 1e-8)
        else:
            two.backward_update_adam(g, 0.03, 0.9, 0.999, 1e-8, step)
        a1, a2 = one.artifacts(), two.artifacts()
        assert a1["num_unique"] == a2["num_unique"] > 0
        for k in ("sorted_keys", "sorted_vals", "unique_keys", "seg_offsets"):
            assert torch.equal(a1[k], a2[k]), k
        assert torch.equal(one.weights.view(torch.uint8), two.weights.view(torch.uint8)), f"weights, step {step}"
        assert torch.equal(one.state.view(torch.uint8), two.state.view(torch.uint8)), f"state, step {step}"
    one.close()
    two.close()


@pytest.mark.parametrize("dtype", [0, 1])
def test_sort_once_update_twice(gpu_device, dtype):
    """A second update after ONE sort applies a second step for the same batch: checked against the oracle
    stepping twice (the long-run queue of the first update must not leak into the second), with a
    tbe_check_inputs of ANOTHER batch in between that must leave the sort's artefacts alone."""
    dev = gpu_device
    spec = _base_spec(dtype)
    b = wl.make_batch(spec, "cpu", seed=31)
    other = wl.make_batch(spec, "cpu", seed=32)
    idx, off = b.indices.numpy(), b.offsets.numpy()
    N, B = b.num_indices, spec.batch
    assert np.bincount(idx[off[0]:off[B]]).max() > 1024, "the case must contain runs that are split over chunks"
    w = wl.make_weights(spec, "cpu", seed=33).numpy()
    m = np.zeros(spec.total_rows, np.float32)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, dtype, B, max(N, other.num_indices), device=dev,
                                       weights=torch.from_numpy(w.copy()).to(dev))
    d_idx, d_off = b.indices.to(dev), b.offsets.to(dev)
    op.backward_sort(d_idx, d_off, B, num_indices=N)
    for step in range(2):
        g = wl.make_grad(spec, "cpu", seed=34 + step).numpy()
        ref = tl.oracle_step(spec, idx, off, w, m, g, 0.02, 1e-8)
        if step == 1:
            assert op.check_inputs(other.indices.to(dev), other.offsets.to(dev), B,
                                   num_indices=other.num_indices) == tbe.TBE_OK
        op.backward_update_rowwise_adagrad(torch.from_numpy(g).to(dev), 0.02, 1e-8)
        tl.assert_artifacts_equal(op.artifacts(), ref["art"], f"update {step}")
        gw, gm = op.weights.cpu().numpy(), op.state.cpu().numpy()
        tl.assert_update_close(spec, ref, w, m, gw, gm, 0.02, 1e-8, f"update {step}")
        w, m = gw, gm
    op.close()


@pytest.mark.parametrize("dtype", [0, 1])
def test_well_conditioned_case_meets_plain_relative_tolerance(gpu_device, dtype):
    """Weights in [0.5, 1.5) and gradients in [0.1, 1.1): every sum has only positive terms, so the plain
    relative error |gpu - ref| / |ref| must stay within 1e-5 (fp32 tables; forward and moments for both
    storage types) and 2e-3 (fp16-stored weights after the update)."""
    dev = gpu_device
    spec = _base_spec(dtype)
    rng = np.random.default_rng(5)
    b = wl.make_batch(spec, "cpu", seed=51)
    idx, off = b.indices.numpy(), b.offsets.numpy()
    N, B = b.num_indices, spec.batch
    wdt = np.float32 if dtype == 0 else np.float16
    w0 = rng.uniform(0.5, 1.5, spec.weight_elems).astype(wdt)
    g = rng.uniform(0.1, 1.1, (B, spec.sumD)).astype(np.float32)
    m0 = rng.uniform(0.0, 2.0, spec.total_rows).astype(np.float32)
    lr, eps = 0.01, 1e-8
    ref = tl.oracle_step(spec, idx, off, w0, m0, g, lr, eps)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, dtype, B, N, device=dev,
                                       weights=torch.from_numpy(w0.copy()).to(dev))
    op.state.copy_(torch.from_numpy(m0))
    d_idx, d_off = b.indices.to(dev), b.offsets.to(dev)
    out = op.forward(d_idx, d_off, B, num_indices=N).cpu().numpy().astype(np.float64)
    r = ref["out"].astype(np.float64)
    nz = r != 0                                      # empty bags pool to exactly 0 on both sides
    assert np.array_equal(out[~nz], r[~nz])
    rel_f = np.abs(out[nz] - r[nz]) / r[nz]
    op.backward_rowwise_adagrad(d_idx, d_off, B, torch.from_numpy(g).to(dev), lr, eps, num_indices=N)
    torch.cuda.synchronize()
    gw, gm = op.weights.cpu().numpy().astype(np.float64), op.state.cpu().numpy().astype(np.float64)
    rel_w = np.abs(gw - ref["w1"].astype(np.float64)) / np.abs(ref["w1"].astype(np.float64))
    keys = ref["art"].unique_keys.astype(np.int64)
    rel_m = np.abs(gm[keys] - ref["m1"][keys].astype(np.float64)) / ref["m1"][keys].astype(np.float64)
    print(f"plain relative error: forward {rel_f.max():.2e}, weights {rel_w.max():.2e}, moments {rel_m.max():.2e}",
          flush=True)
    assert rel_f.max() <= tl.RTOL_FP32
    assert rel_w.max() <= tl.rtol_for(dtype)
    assert rel_m.max() <= tl.RTOL_FP32
    op.close()


def test_read_probe_runs_and_touches_nothing(gpu_device):
    """The read-rate probe of the C-ABI: enqueues on the given stream, reads only, and leaves source and sink as
    they were (the sink is written for one xor value in 2^32 only; this buffer's xor is not that value)."""
    import torch

    n = (8 << 20) // 4 + 12                      # a ragged tail beyond the last 16-byte word
    src = torch.arange(n, dtype=torch.int32, device=gpu_device)
    before = src.clone()
    sink = torch.full((1,), 77, dtype=torch.int32, device=gpu_device)
    for passes in (1, 3):
        assert tbe.tbe_probe_read(src, 4 * n, passes, sink) == tbe.TBE_OK
    s2 = torch.cuda.Stream()
    with torch.cuda.stream(s2):
        assert tbe.tbe_probe_read(src, 4 * n, 2, sink, stream=s2) == tbe.TBE_OK
    torch.cuda.synchronize()
    assert torch.equal(src, before) and int(sink.item()) == 77
    assert tbe.tbe_probe_read(src, 16, 1, sink) == tbe.TBE_OK      # a single word
    torch.cuda.synchronize()
