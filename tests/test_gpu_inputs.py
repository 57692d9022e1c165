"""GPU parity of the input-side kernels (include/tbe_inputs.h) against oracle/inputs_oracle.c:
lengths -> offsets, (W,T,B) -> (T,W,B) permute, row-wise bucketize.  Integer work: every output is
compared bit-exactly, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import inputs_oracle as io
from paper_2104_05158_amd import tbe
from paper_2104_05158_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _scratch(n, dev):
    return torch.empty(tbe.tbe_inputs_scratch_bytes(n), dtype=torch.uint8, device=dev)


def _gpu_lengths_to_offsets(lens_np, dev):
    n = len(lens_np)
    lens = torch.from_numpy(np.ascontiguousarray(lens_np, np.int32)).to(dev)
    off = torch.full((n + 1,), -7, dtype=torch.int64, device=dev)
    rc = tbe.tbe_lengths_to_offsets(lens, n, off, _scratch(n, dev))
    assert rc == tbe.TBE_OK
    torch.cuda.synchronize()
    return off.cpu().numpy()


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 12289, 1_000_003])
def test_lengths_to_offsets(gpu_device, n):
    rng = np.random.default_rng(n)
    lens = rng.poisson(20.0, n).astype(np.int32)
    print(f"lengths_to_offsets n={n}", flush=True)
    got = _gpu_lengths_to_offsets(lens, gpu_device)
    assert np.array_equal(got, io.lengths_to_offsets(lens))


def test_lengths_to_offsets_sums_past_32_bits(gpu_device):
    lens = np.full(9001, 2 ** 30, np.int32)
    lens[::7] = 0
    got = _gpu_lengths_to_offsets(lens, gpu_device)
    ref = io.lengths_to_offsets(lens)
    assert ref[-1] > 2 ** 42 and np.array_equal(got, ref)


def _gpu_permute(W, T, B, lens, idx, dev):
    n = W * T * B
    N = int(idx.numel())
    lo = torch.full((max(n, 1),), -7, dtype=torch.int32, device=dev)
    oo = torch.full((n + 1,), -7, dtype=torch.int64, device=dev)
    ix = torch.full((max(N, 1),), -7, dtype=torch.int32, device=dev)
    rc = tbe.tbe_permute_wtb_to_twb(W, T, B, lens, idx, N, lo, oo, ix, _scratch(n, dev))
    assert rc == tbe.TBE_OK
    torch.cuda.synchronize()
    return lo[:n].cpu().numpy(), oo.cpu().numpy(), ix[:N].cpu().numpy()


@pytest.mark.parametrize("W,T,B,mean,max_len", [
    (1, 1, 1, 3.0, None), (2, 2, 2, 0.0, 3), (1, 5, 7, 4.0, None), (5, 1, 7, 4.0, None), (3, 4, 1, 2.0, None),
    (4, 3, 300, 20.0, None), (8, 13, 257, 0.5, None), (2, 3, 1000, 0.0, 0), (7, 5, 64, 0.0, 400),
    (8, 26, 2048, 20.0, None),
])
def test_permute_wtb_to_twb(gpu_device, W, T, B, mean, max_len):
    rows = 1000 + 37 * np.arange(T)
    lens, idx = wl.make_wtb_input(W, T, B, rows, mean, "cpu", seed=W * 100 + T, max_len=max_len)
    print(f"permute W={W} T={T} B={B} N={idx.numel()}", flush=True)
    ref = io.permute_wtb_to_twb(W, T, B, lens.numpy(), idx.numpy())
    got = _gpu_permute(W, T, B, lens.to(gpu_device), idx.to(gpu_device), gpu_device)
    for g, r, name in zip(got, ref, ("lengths", "offsets", "indices")):
        assert np.array_equal(g, r), name


def _gpu_bucketize(rows, B, W, idx, off, dev):
    T = len(rows)
    n = W * T * B
    N = int(idx.numel())
    lo = torch.full((max(n, 1),), -7, dtype=torch.int32, device=dev)
    oo = torch.full((n + 1,), -7, dtype=torch.int64, device=dev)
    ix = torch.full((max(N, 1),), -7, dtype=torch.int32, device=dev)
    d_rows = torch.from_numpy(np.ascontiguousarray(rows, np.int64)).to(dev)
    rc = tbe.tbe_bucketize_rowwise(T, B, W, d_rows, idx, off, N, lo, oo, ix, _scratch(n, dev))
    assert rc == tbe.TBE_OK
    torch.cuda.synchronize()
    return lo[:n].cpu().numpy(), oo.cpu().numpy(), ix[:N].cpu().numpy()


def _check_bucketize(spec, W, dev, seed=1):
    b = wl.make_batch(spec, "cpu", seed=seed)
    print(f"bucketize {spec.name} T={spec.T} B={spec.batch} W={W} N={b.num_indices}", flush=True)
    ref = io.bucketize_rowwise(spec.rows, spec.batch, W, b.indices.numpy(), b.offsets.numpy())
    got = _gpu_bucketize(spec.rows, spec.batch, W, b.indices.to(dev), b.offsets.to(dev), dev)
    for g, r, name in zip(got, ref, ("lengths", "offsets", "indices")):
        assert np.array_equal(g, r), name
    return got


@pytest.mark.parametrize("W", [1, 2, 3, 8, 64, 1000, 1024])
def test_bucketize_rowwise_small(gpu_device, W):
    spec = wl.custom([1000, 17, 5003], [8, 8, 8], 0, 37, [20.0, 3.0, 0.7], name="buck_small")
    _check_bucketize(spec, W, gpu_device)


def test_bucketize_long_bags_span_many_wavefront_steps(gpu_device):
    # bags of ~500 lookups: the per-shard running counts are carried across 8 steps of 64 positions
    spec = wl.custom([100_000, 999], [8, 8], 0, 50, [500.0, 300.0], name="buck_long")
    for W in (4, 7, 128):
        _check_bucketize(spec, W, gpu_device, seed=W)


def test_bucketize_skew_and_empty(gpu_device):
    spec = wl.custom([1 << 20, 50], [8, 8], 0, 4096, [30.0, 0.2], index_dist="zipf", zipf_s=1.1, name="buck_zipf")
    _check_bucketize(spec, 8, gpu_device)
    spec0 = wl.custom([1000], [8], 0, 300, [0.0], pooling_kind="fixed", name="buck_empty")
    _check_bucketize(spec0, 4, gpu_device)


def test_bucketize_full_size_shard_table_then_permute(gpu_device):
    """The row-wise sharded table of configuration 3 at its real shape (50M rows, batch 32768,
    pooling 30) split over 8 shards; the (W,T,B) result is then permuted to (T,W,B) on the GPU and
    both steps are compared with the oracle."""
    spec = wl.custom([50_000_000], [256], 1, 32768, [30.0], index_dist="zipf", zipf_s=1.1, name="cfg3_shard")
    W = 8
    lo, oo, ix = _check_bucketize(spec, W, gpu_device)
    ref = io.permute_wtb_to_twb(W, 1, spec.batch, lo, ix)
    dev = gpu_device
    got = _gpu_permute(W, 1, spec.batch, torch.from_numpy(lo).to(dev), torch.from_numpy(ix).to(dev), dev)
    for g, r, name in zip(got, ref, ("lengths", "offsets", "indices")):
        assert np.array_equal(g, r), name


def test_input_kernels_are_deterministic(gpu_device):
    spec = wl.custom([30_000, 777], [8, 8], 0, 2048, [25.0, 5.0], name="buck_det")
    b = wl.make_batch(spec, "cpu", seed=3)
    idx, off = b.indices.to(gpu_device), b.offsets.to(gpu_device)
    a = _gpu_bucketize(spec.rows, spec.batch, 16, idx, off, gpu_device)
    c = _gpu_bucketize(spec.rows, spec.batch, 16, idx, off, gpu_device)
    assert all(np.array_equal(x, y) for x, y in zip(a, c))
