"""GPU parity on seeded random problem shapes: numbers of tables, heights, dims, batch sizes, pooling
factors and index distributions that no hand-written case pairs up (one-row tables next to wide ones,
a batch of one bag, pooling 0, dims at both ends of the range, both layouts and storage types).
Every case goes through the same element-by-element comparison with the CPU oracle as the other tests.
"""
import numpy as np
import pytest

from paper_2104_05158_amd import workloads as wl

import tbe_testlib as tl

pytestmark = pytest.mark.gpu


def _random_spec(seed):
    rng = np.random.default_rng(9000 + seed)
    T = int(rng.integers(1, 10))
    dims = (4 * rng.integers(1, 129, size=T)).astype(np.int32)            # 4 .. 512
    if rng.random() < 0.5:
        dims = (4 * rng.integers(1, 17, size=T)).astype(np.int32)        # narrow tables: 4 .. 64
    rows = np.where(rng.random(T) < 0.3, rng.integers(1, 8, size=T), rng.integers(8, 60_000, size=T)).astype(np.int64)
    B = int(rng.choice([1, 2, 3, 31, 64, 65, 200, 513, 900]))
    pooling = np.where(rng.random(T) < 0.2, 0.0, rng.uniform(0.3, 24.0, size=T))
    if B * pooling.sum() > 150_000:                                        # keep the oracle within seconds
        pooling *= 150_000 / (B * pooling.sum())
    dtype = int(rng.integers(0, 2))
    dist = "zipf" if rng.random() < 0.6 else "uniform"
    spec = wl.custom(rows, dims, dtype, B, pooling, index_dist=dist, zipf_s=float(rng.uniform(1.01, 1.4)),
                     name=f"rnd{seed}")
    return spec, int(rng.integers(0, 2))


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(gpu_device, seed):
    spec, layout = _random_spec(seed)
    b = wl.make_batch(spec, "cpu", seed=100 + seed)
    w = wl.make_weights(spec, "cpu", seed=200 + seed).numpy()
    g = wl.make_grad(spec, "cpu", seed=300 + seed).numpy()
    rng = np.random.default_rng(seed)
    m0 = (rng.random(spec.total_rows) * (rng.random() < 0.5)).astype(np.float32)   # zero or random moments
    r = tl.full_parity_step(spec, b.indices.numpy(), b.offsets.numpy(), w, g, gpu_device, lr=0.03, m0=m0,
                            what=f"rnd{seed}", layout=layout)
    print(f"rnd{seed}: T={spec.T} B={spec.batch} dims={spec.dims.tolist()} rows={spec.rows.tolist()} "
          f"dtype={spec.dtype} layout={layout} {r}")


@pytest.mark.parametrize("seed", range(12))
def test_random_shape_other_optimizers_and_gradient_types(gpu_device, seed):
    # the same random shapes through element-wise AdaGrad / lazy Adam (two steps each), with the gradient in
    # float32, float16 or bfloat16
    import test_gpu_optimizers as tgo
    from paper_2104_05158_amd import tbe

    spec, _ = _random_spec(seed)
    optimizer = tbe.TBE_OPT_ADAM if seed % 2 else tbe.TBE_OPT_ADAGRAD
    grad_dtype = [tbe.TBE_DTYPE_FP32, tbe.TBE_DTYPE_FP16, tbe.TBE_DTYPE_BF16][seed % 3]
    tgo._run(spec, optimizer, grad_dtype, gpu_device, steps=2, seed=500 + seed)
