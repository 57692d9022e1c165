"""GPU test of the entry point that allocates nothing: tbe_lengths_to_offsets_noalloc keeps the
scan's block sums in a fixed array inside the library instead of a caller-provided scratch buffer.
Its offsets must equal those of tbe_lengths_to_offsets (and of the CPU oracle) bit for bit, on two
calls in a row that share the array, the second with a smaller input, and it must reject sizes
beyond its stated maximum before touching the device."""
import numpy as np
import pytest
import torch

from oracle import inputs_oracle as io
from paper_2104_05158_amd import tbe

pytestmark = pytest.mark.gpu


def _with_scratch(lens, dev):
    n = lens.numel()
    off = torch.full((n + 1,), -7, dtype=torch.int64, device=dev)
    scratch = torch.empty(tbe.tbe_inputs_scratch_bytes(n), dtype=torch.uint8, device=dev)
    assert tbe.tbe_lengths_to_offsets(lens, n, off, scratch) == tbe.TBE_OK
    return off


def _noalloc(lens, dev):
    n = lens.numel()
    off = torch.full((n + 1,), -9, dtype=torch.int64, device=dev)
    assert tbe.tbe_lengths_to_offsets_noalloc(lens, n, off) == tbe.TBE_OK
    return off


def test_noalloc_matches_scratch_variant_twice_second_smaller(gpu_device):
    dev = gpu_device
    rng = np.random.default_rng(77)
    # 3,000,017 bags = 733 scan tiles and a ragged tail; then 70,001 bags (18 tiles) on the same array
    for n in (3_000_017, 70_001):
        lens_np = rng.poisson(25.0, n).astype(np.int32)
        lens = torch.from_numpy(lens_np).to(dev)
        print(f"noalloc lengths_to_offsets n={n}", flush=True)
        got = _noalloc(lens, dev)
        ref = _with_scratch(lens, dev)
        torch.cuda.synchronize()
        assert torch.equal(got, ref)
        assert np.array_equal(got.cpu().numpy(), io.lengths_to_offsets(lens_np))


def test_noalloc_small_and_empty(gpu_device):
    dev = gpu_device
    for n in (0, 1, 5, 4096, 4097):
        lens_np = np.arange(n, dtype=np.int32) % 7
        lens = torch.from_numpy(lens_np).to(dev) if n else torch.empty(0, dtype=torch.int32, device=dev)
        got = _noalloc(lens, dev)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), io.lengths_to_offsets(lens_np))


def test_noalloc_rejects_sizes_beyond_its_maximum(gpu_device):
    dev = gpu_device
    limit = tbe.tbe_lengths_to_offsets_noalloc_max_bags()
    assert limit == 131071 * 4096
    lens = torch.zeros(16, dtype=torch.int32, device=dev)
    off = torch.zeros(17, dtype=torch.int64, device=dev)
    # only the size is beyond the limit; nothing is enqueued, the buffers are not touched
    assert tbe.lib().tbe_lengths_to_offsets_noalloc(lens.data_ptr(), limit + 1, off.data_ptr(), None) == tbe.TBE_ERR_UNSUPPORTED
    assert tbe.lib().tbe_lengths_to_offsets_noalloc(lens.data_ptr(), -1, off.data_ptr(), None) == tbe.TBE_ERR_INVALID_ARG
    assert tbe.lib().tbe_lengths_to_offsets_noalloc(None, 4, off.data_ptr(), None) == tbe.TBE_ERR_INVALID_ARG
