"""GPU parity of the update kernel's run classes.  The kernel sorts the runs of a span of 256 sorted positions by
length and handles them in steps: several runs of one or two lookups per lane group, one run of up to four per
lane group, teams of 2, 4, ... lane groups for runs of up to 4 x team lookups, the whole wavefront in several steps
beyond that, and the queues of the other kernels beyond 512.  The tables below hold one run of every length on both
sides of each of those borders, for every lanes-per-row setting (D = 4 .. 512), in shuffled row order so that the
lengths mix inside a span, plus a crowd of single-lookup rows that fills the many-runs-per-group steps.
Everything is compared with the CPU oracle element by element; integer artefacts bit-exactly."""
import numpy as np
import pytest

import tbe_testlib as tl
from paper_2104_05158_amd import workloads as wl

pytestmark = pytest.mark.gpu

BORDERS = [1, 2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 64, 65, 128, 129, 255, 256, 257, 300, 511, 512, 513, 600]


def _explicit_case(dims, lens_per_table, batch, seed, dtype):
    """Table t has one row per entry of lens_per_table[t]; row r is looked up lens[r] times, by random bags
    (a bag may look a row up more than once).  Row ids are a random permutation, so lengths mix in sorted order."""
    rng = np.random.default_rng(seed)
    rows = [len(l) for l in lens_per_table]
    spec = wl.custom(rows, dims, dtype, batch, 1.0, name="run-classes")
    idx_parts, counts = [], []
    for t, lens in enumerate(lens_per_table):
        perm = rng.permutation(rows[t])
        row_of = np.repeat(perm, lens)                    # one entry per lookup
        bag_of = rng.integers(0, batch, size=row_of.size)
        order = np.argsort(bag_of, kind="stable")
        idx_parts.append(row_of[order].astype(np.int32))
        counts.append(np.bincount(bag_of, minlength=batch))
    idx = np.concatenate(idx_parts)
    off = np.concatenate([[0], np.cumsum(np.concatenate(counts))]).astype(np.int64)
    return spec, idx, off


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("dtype", [0, 1])
def test_every_length_class_for_every_lane_mapping(gpu_device, dtype, layout):
    dims = [4, 8, 16, 36, 64, 128, 256, 512]
    lens = [np.array(BORDERS + list(range(6, 41)) + [1] * 300 + [2] * 90 + [3] * 20) for _ in dims]
    spec, idx, off = _explicit_case(dims, lens, batch=53, seed=5 + dtype, dtype=dtype)
    w = wl.make_weights(spec, "cpu", seed=6).numpy()
    g = wl.make_grad(spec, "cpu", seed=7).numpy()
    m0 = np.random.default_rng(8).uniform(0, 1, spec.total_rows).astype(np.float32)
    print(f"N={idx.size} runs={sum(len(l) for l in lens)} dtype={dtype} layout={layout}", flush=True)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, lr=0.03, m0=m0, what="run-classes", layout=layout)


@pytest.mark.parametrize("dtype", [0, 1])
def test_spans_that_touch_many_tables(gpu_device, dtype):
    # thirty tables of a handful of rows each: a span of 256 sorted positions covers several tables, with
    # different lane mappings, and every table's runs are classified on their own
    rng = np.random.default_rng(11)
    dims = [int(d) for d in rng.choice([4, 8, 12, 32, 64, 100, 128, 260], size=30)]
    lens = [rng.choice([1, 1, 1, 2, 3, 4, 5, 7, 9, 18, 40], size=int(rng.integers(1, 12))) for _ in dims]
    spec, idx, off = _explicit_case(dims, lens, batch=17, seed=12, dtype=dtype)
    w = wl.make_weights(spec, "cpu", seed=13).numpy()
    g = wl.make_grad(spec, "cpu", seed=14).numpy()
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, lr=0.03, what="many-tables")


def test_other_optimizers_and_16bit_gradients_over_the_classes(gpu_device):
    import torch

    import test_gpu_optimizers as tgo
    from paper_2104_05158_amd import tbe

    dims = [8, 64, 128]
    lens = [np.array(BORDERS[:-2] + [1] * 150 + [2] * 40) for _ in dims]
    spec, idx, off = _explicit_case(dims, lens, batch=41, seed=21, dtype=1)
    for optimizer in (tbe.TBE_OPT_ADAGRAD, tbe.TBE_OPT_ADAM):
        tgo._run(spec, optimizer, tbe.TBE_DTYPE_FP32, gpu_device, steps=2, seed=22, batch=(idx, off))
    # row-wise AdaGrad with a bf16 gradient: the oracle gets exactly the values the library reads
    dev = gpu_device
    N, B = int(idx.size), spec.batch
    w0 = wl.make_weights(spec, "cpu", seed=24).numpy()
    m0 = np.zeros(spec.total_rows, np.float32)
    g_t = torch.from_numpy(wl.make_grad(spec, "cpu", seed=25).numpy()).to(torch.bfloat16)
    ref = tl.oracle_step(spec, idx, off, w0, m0, g_t.float().numpy(), 0.01, 1e-8)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, 1, B, N, device=dev,
                                       weights=torch.from_numpy(w0.copy()).to(dev), grad_dtype=tbe.TBE_DTYPE_BF16)
    op.backward_rowwise_adagrad(torch.from_numpy(idx).to(dev), torch.from_numpy(off).to(dev), B, g_t.to(dev),
                                0.01, 1e-8, num_indices=N)
    tl.assert_artifacts_equal(op.artifacts(), ref["art"], "bf16")
    tl.assert_update_close(spec, ref, w0, m0, op.weights.cpu().numpy(), op.state.cpu().numpy(), 0.01, 1e-8, "bf16")
    op.close()


@pytest.mark.parametrize("dtype", [0, 1])
def test_spans_of_single_lookup_rows_only(gpu_device, dtype):
    # every row once: a span holds 256 runs of one lookup, and for D = 4 (64 lane groups) one step takes all of
    # them; 1000 rows leave a ragged last span; a second table of two-lookup rows fills the two-runs-per-group steps
    dims = [4, 8, 64, 128, 512]
    lens = [np.ones(1000, np.int64) for _ in dims] + [np.full(700, 2, np.int64)]
    spec, idx, off = _explicit_case(dims + [16], lens, batch=29, seed=31 + dtype, dtype=dtype)
    w = wl.make_weights(spec, "cpu", seed=32).numpy()
    g = wl.make_grad(spec, "cpu", seed=33).numpy()
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, lr=0.03, what="single-lookup rows")
