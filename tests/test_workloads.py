"""The synthetic input recipe: shapes of the five benchmark configurations and basic validity of
the generated batches (no arithmetic of the method is involved)."""
import numpy as np

from paper_2104_05158_amd import workloads as wl


def test_config_shapes():
    c0, c1, c2, c3, c4 = (wl.config(k) for k in range(5))
    assert (c0.T, int(c0.rows[0]), int(c0.dims[0]), c0.batch, c0.dtype) == (1, 10_000, 64, 256, 0)
    assert (c1.T, c1.batch, c1.dtype) == (8, 4096, 0) and np.all(c1.rows == 1_000_000) and np.all(c1.dims == 128)
    assert (c2.T, c2.batch, c2.dtype) == (64, 16384, 1)
    assert c2.rows.min() >= 1e5 and c2.rows.max() <= 1e7 and 1 <= c2.pooling_mean.min() and c2.pooling_mean.max() <= 100
    assert (c3.T, c3.batch) == (129, 32768) and int(c3.rows[-1]) == 50_000_000 and int(c3.dims[-1]) == 256
    assert set(np.unique(c3.dims)) <= {32, 64, 128, 256}
    assert (c4.T, c4.batch) == (400, 65536) and set(np.unique(c4.dims)) <= {64, 128}
    assert abs(c4.weight_bytes - 120e9) < 0.01 * 120e9
    for c in (c0, c1, c2, c3, c4):
        assert c.total_rows < 2 ** 32 - 1 and c.expected_lookups() < 2 ** 31 - 2 ** 24


def test_batches_are_valid_and_seeded():
    spec = wl.config(2, scale=1 / 256)
    a = wl.make_batch(spec, "cpu", it=0)
    b = wl.make_batch(spec, "cpu", it=0)
    c = wl.make_batch(spec, "cpu", it=1)
    assert np.array_equal(a.indices.numpy(), b.indices.numpy()) and np.array_equal(a.offsets.numpy(), b.offsets.numpy())
    assert not np.array_equal(a.offsets.numpy(), c.offsets.numpy())
    off, idx = a.offsets.numpy(), a.indices.numpy()
    assert off[0] == 0 and off[-1] == len(idx) == a.num_indices and np.all(np.diff(off) >= 0)
    B = spec.batch
    for t in range(spec.T):
        seg = idx[off[t * B]:off[(t + 1) * B]]
        assert seg.size == 0 or (seg.min() >= 0 and seg.max() < spec.rows[t])
    # Zipf skew: far fewer distinct rows than lookups, and the hottest row is a few percent of a table
    t = int(np.argmax(spec.pooling_mean))
    seg = idx[off[t * B]:off[(t + 1) * B]]
    cnt = np.bincount(seg)
    assert cnt.max() / seg.size > 0.03 and np.count_nonzero(cnt) < 0.8 * seg.size


def test_weights_and_grads():
    spec = wl.config(0)
    w = wl.make_weights(spec, "cpu").numpy()
    assert w.dtype == np.float32 and w.size == 640_000 and w.min() >= -0.01 and w.max() <= 0.01 and abs(w.mean()) < 1e-4
    g = wl.make_grad(spec, "cpu").numpy()
    assert g.shape == (256, 64) and abs(g.std() - 1) < 0.05
    m = wl.make_moments(spec, "cpu")
    assert m.numel() == 10_000 and not m.any()
