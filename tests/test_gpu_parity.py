"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several sort tiles, update chunks and
ragged tails; plus the degenerate cases of the method (empty bags, empty batch, one hot row,
runs at the long-run threshold, every row touched, pure gather).
Integer artefacts must be bit-exact; floats within rtol 1e-5 (fp32) / 2e-3 (fp16-stored).
"""
import numpy as np
import pytest
import torch

from oracle import tbe_oracle as orc
from paper_2104_05158_amd import tbe
from paper_2104_05158_amd import workloads as wl

import tbe_testlib as tl

pytestmark = pytest.mark.gpu


def _np_case(spec, seed, device="cpu"):
    b = wl.make_batch(spec, device, seed=seed)
    w = wl.make_weights(spec, device, seed=seed + 1).cpu().numpy()
    g = wl.make_grad(spec, device, seed=seed + 2).cpu().numpy()
    return b.indices.cpu().numpy(), b.offsets.cpu().numpy(), w, g


def test_config0_full(gpu_device):
    spec = wl.config(0)
    idx, off, w, g = _np_case(spec, 1)
    assert int(off[-1]) == 2048
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, lr=spec.lr, eps=spec.eps, what="cfg0")
    print("cfg0", r)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_tables_heavy_duplicates(gpu_device, dtype, seed):
    spec, idx, off, w, g = wl.tiny_random(40 + seed, T=3, max_rows=16, dims=(4, 8, 12), B=4, max_len=5, dtype=dtype)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, lr=0.05, what=f"tiny{seed}")


@pytest.mark.parametrize("dtype", [0, 1])
def test_mixed_dims_all_lane_mappings(gpu_device, dtype):
    # D from 4 to 512 covers every lanes-per-row setting, the two-block path (D > 256) and, for
    # fp16, dims that are not multiples of 8 (4-element vectors)
    dims = [4, 8, 12, 32, 36, 64, 100, 128, 192, 256, 260, 384, 512]
    rows = [50, 7, 300, 1000, 33, 2000, 500, 4000, 129, 700, 90, 250, 64]
    spec = wl.custom(rows, dims, dtype, 37, 6.0, index_dist="zipf", zipf_s=1.05, name="mixed")
    idx, off, w, g = _np_case(spec, 5)
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="mixed-dims")
    print("mixed", r)


@pytest.mark.parametrize("dtype", [0, 1])
def test_table_major_output_and_gradient_layout(gpu_device, dtype):
    # one contiguous [B, D_t] block per table instead of [B, sumD] rows: same numbers, other addresses;
    # dims cover every lane mapping, the index distribution gives short, medium and long runs
    dims = [4, 8, 12, 32, 36, 64, 100, 128, 192, 256, 260, 384, 512]
    rows = [50, 7, 300, 1000, 33, 2000, 500, 4000, 129, 700, 90, 250, 1]
    spec = wl.custom(rows, dims, dtype, 611, 6.0, index_dist="zipf", zipf_s=1.05, name="table-major")
    idx, off, w, g = _np_case(spec, 6)
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="table-major", layout=1)
    print("table-major", r)


def test_fp16_dims_multiple_of_8_vector_path(gpu_device):
    spec = wl.custom([3000, 500, 100], [128, 32, 256], 1, 200, [20.0, 3.0, 40.0], index_dist="zipf", name="fp16x8")
    idx, off, w, g = _np_case(spec, 9)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="fp16x8")


@pytest.mark.parametrize("dtype", [0, 1])
def test_several_sort_tiles_and_ragged_tail(gpu_device, dtype):
    # N ~ 5 sort tiles + tail, 3 radix passes (2^17 < total rows < 2^24), uniform => long unique list
    spec = wl.custom([100_000, 50_001, 7], [64, 32, 16], dtype, 701, [30.0, 27.0, 2.0], name="tiles")
    idx, off, w, g = _np_case(spec, 11)
    assert int(off[-1]) > 4 * 8192 and int(off[-1]) % 8192 != 0
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="tiles")
    print("tiles", r)


@pytest.mark.parametrize("total_rows", [2, 255, 257, 70_000, 20_000_000])
def test_key_bit_budgets(gpu_device, total_rows):
    # the sort runs over the row-index bits of the tallest table: 1, 7, 8, 16 and 24 bits here, i.e.
    # 1 to 3 radix passes with even and uneven digit widths
    rows = [total_rows - total_rows // 2, total_rows // 2] if total_rows > 2 else [1, 1]
    spec = wl.custom(rows, [8, 4], 0, 97, 9.0, name=f"bits{total_rows}")
    idx, off, w, g = _np_case(spec, 13)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what=f"bits{total_rows}")


def test_widest_key_needs_four_passes(gpu_device):
    # 2^24 + 1 rows in one table: 25 row-index bits -> 4 passes (7,6,6,6); a 1-row table beside it
    spec = wl.custom([(1 << 24) + 1, 1], [4, 4], 0, 64, [40.0, 3.0], name="bits25")
    idx, off, w, g = _np_case(spec, 14)
    idx[:5] = [(1 << 24), 0, (1 << 24), 1 << 23, (1 << 24) - 1]     # the extreme rows occur, one of them twice
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="bits25")


def test_tables_with_different_pass_counts_in_one_sort(gpu_device):
    # row-index bits 2, 8, 9, 16, 17 and 25 side by side: 1, 1, 2, 2, 3 and 4 radix passes of different digit
    # widths; the short tables sit out the first launches and read the caller's indices later, and every
    # table must still end in the same buffer, several 8192-position tiles each
    rows = [3, 256, 300, 65536, 70_000, (1 << 24) + 5]
    spec = wl.custom(rows, [4, 8, 4, 4, 8, 4], 0, 1200, [30.0, 25.0, 20.0, 22.0, 28.0, 24.0], name="mixed_passes")
    idx, off, w, g = _np_case(spec, 21)
    idx[int(off[5 * 1200]):int(off[5 * 1200]) + 3] = [1 << 24, (1 << 24) + 4, 0]     # the tallest table's extreme rows occur
    assert int(off[1200]) > 2 * 8192
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="mixed_passes")


@pytest.mark.parametrize("batch", [65536, 65537, 70_000])
def test_sort_payloads_at_and_beyond_16_bits(gpu_device, batch):
    # the sort carries the bag number as 16 bits between its passes while the batch allows it (65536: the last bag
    # is 65535) and as 32 bits beyond; tables of 1, 2 and 3 passes; the last bags carry lookups of the extreme rows
    rows = [200, 300, 70_000]
    spec = wl.custom(rows, [4, 8, 4], 0, batch, [0.6, 0.9, 0.7], name=f"payload{batch}")
    idx, off, w, g = _np_case(spec, 31)
    for t in range(3):
        lo, hi = int(off[(t + 1) * batch - 1]), int(off[(t + 1) * batch])
        if hi > lo:
            idx[hi - 1] = rows[t] - 1
    assert int(off[-1]) > 3 * 8192
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what=f"payload{batch}")


def test_segmented_sort_tables_without_lookups(gpu_device):
    # tables 0, 2 and 4 receive no lookup at all: they own no sort tile and their rows stay untouched
    spec = wl.custom([50, 3000, 7, 120, 9000], [8, 16, 4, 32, 8], 0, 300, [0.0, 40.0, 0.0, 12.0, 0.0],
                     pooling_kind="poisson", name="holes")
    idx, off, w, g = _np_case(spec, 15)
    assert int(off[300]) == 0 and int(off[900]) == int(off[600]) and int(off[-1]) == int(off[1200]) > 8192
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="holes")


def test_first_pass_tile_spanning_more_bags_than_it_has_positions(gpu_device):
    # mean pooling 0.3: one 8192-position sort tile spans ~27k bags, more than the bag borders the first pass can
    # stage on chip, so payloads are found by bisection in global memory
    spec = wl.custom([5000, 800], [8, 4], 0, 60000, [0.3, 0.25], name="sparse_bags")
    idx, off, w, g = _np_case(spec, 16)
    assert int(off[60000]) > 2 * 8192
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="sparse_bags")


def test_many_small_tables(gpu_device):
    # 700 tables (more than one block of the table scan), most with a single partly filled sort tile
    rng = np.random.default_rng(17)
    rows = rng.integers(3, 400, 700)
    dims = rng.choice([4, 8, 16], 700)
    spec = wl.custom(rows, dims, 1, 24, rng.uniform(0.0, 6.0, 700), name="many_tables")
    idx, off, w, g = _np_case(spec, 18)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="many_tables")


@pytest.mark.parametrize("dtype", [0, 1])
def test_single_hot_row_long_run_path(gpu_device, dtype):
    # every lookup of table 0 hits one row: one run of ~5000 lookups across ~20 update chunks
    spec = wl.custom([1000, 50], [128, 64], dtype, 250, [20.0, 4.0], name="hot")
    idx, off, w, g = _np_case(spec, 17)
    n0 = int(off[spec.batch])
    idx[:n0] = 777
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="hot-row")
    assert n0 > 2048
    print("hot", r)


@pytest.mark.parametrize("run_len", [3, 4, 5, 127, 128, 129, 255, 256, 257, 511, 512, 513, 768, 1025])
def test_run_lengths_around_chunk_and_long_run_thresholds(gpu_device, run_len):
    # table of 3 rows: row 1 gets exactly run_len lookups, preceded and followed by shorter runs so
    # that the run starts inside a chunk, not on its border
    B = 64
    lens = np.zeros(B, np.int64)
    total = 100 + run_len + 300
    lens[:] = total // B
    lens[: total % B] += 1
    off = np.zeros(B + 1, np.int64)
    off[1:] = np.cumsum(lens)
    rng = np.random.default_rng(run_len)
    idx = np.concatenate([np.zeros(100), np.ones(run_len), np.full(300, 2)]).astype(np.int32)
    idx = rng.permutation(idx)
    spec = wl.custom([3], [64], 0, B, 0.0, name="thr")
    w = rng.uniform(-1, 1, 3 * 64).astype(np.float32)
    g = rng.normal(size=(B, 64)).astype(np.float32)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what=f"run{run_len}")


def test_every_row_touched_and_nonzero_initial_moments(gpu_device):
    spec = wl.custom([64, 10], [32, 8], 0, 128, [16.0, 8.0], name="all-rows")
    idx, off, w, g = _np_case(spec, 19)
    assert len(np.unique(idx[: off[spec.batch]])) == 64
    m0 = np.random.default_rng(0).uniform(0.0, 3.0, spec.total_rows).astype(np.float32)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, m0=m0, what="all-rows")


@pytest.mark.parametrize("dtype", [0, 1])
def test_pooling_one_unique_indices_is_bit_exact_gather(gpu_device, dtype):
    spec = wl.custom([5000, 300], [128, 48], dtype, 256, 1.0, pooling_kind="fixed", name="gather")
    rng = np.random.default_rng(23)
    idx = np.concatenate([rng.permutation(5000)[:256], rng.permutation(300)[:256]]).astype(np.int32)
    off = np.arange(2 * 256 + 1, dtype=np.int64)
    w = wl.make_weights(spec, "cpu", seed=3).numpy()
    op = tl.make_op(spec, gpu_device, max_indices=512, weights=torch.from_numpy(w.copy()).to(gpu_device))
    out = op.forward(torch.from_numpy(idx).to(gpu_device), torch.from_numpy(off).to(gpu_device), 256).cpu().numpy()
    ref = orc.forward(spec.rows, spec.dims, dtype, w, idx, off, 256)
    assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
    w0 = w[: 5000 * 128].reshape(5000, 128)
    assert np.array_equal(out[:, :128], w0[idx[:256]].astype(np.float32))


def test_empty_bags_and_empty_batch(gpu_device):
    spec = wl.custom([40, 9], [16, 8], 0, 8, 0.0, name="empty")
    lens = np.array([0, 3, 0, 0, 5, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0, 2], np.int64)
    off = np.zeros(17, np.int64)
    off[1:] = np.cumsum(lens)
    rng = np.random.default_rng(1)
    idx = np.concatenate([rng.integers(0, 40, int(lens[:8].sum())), rng.integers(0, 9, int(lens[8:].sum()))]).astype(np.int32)
    w = rng.uniform(-1, 1, spec.weight_elems).astype(np.float32)
    g = rng.normal(size=(8, 24)).astype(np.float32)
    tl.full_parity_step(spec, idx, off, w, g, gpu_device, what="empty-bags")
    # no lookups at all: output zero, nothing updated, U = 0
    off0 = np.zeros(17, np.int64)
    op = tl.make_op(spec, gpu_device, max_indices=16, weights=torch.from_numpy(w.copy()).to(gpu_device))
    d_off = torch.from_numpy(off0).to(gpu_device)
    d_idx = torch.zeros(0, dtype=torch.int32, device=gpu_device)
    out = op.forward(d_idx, d_off, 8)
    assert not out.any().item()
    op.backward_rowwise_adagrad(d_idx, d_off, 8, torch.from_numpy(g).to(gpu_device), 0.1, 1e-8)
    art = op.artifacts()
    assert art["num_unique"] == 0
    assert np.array_equal(op.weights.cpu().numpy(), w) and not op.state.any().item()


def test_backward_is_deterministic_run_to_run(gpu_device):
    spec = wl.custom([2000, 100], [128, 64], 1, 300, [25.0, 10.0], index_dist="zipf", name="det")
    idx, off, w, g = _np_case(spec, 29)
    res = []
    for _ in range(2):
        op = tl.make_op(spec, gpu_device, max_indices=len(idx), weights=torch.from_numpy(w.copy()).to(gpu_device))
        a = [torch.from_numpy(x).to(gpu_device) for x in (idx, off, g)]
        op.backward_rowwise_adagrad(a[0], a[1], spec.batch, a[2], 0.01, 1e-8)
        art = op.artifacts()
        res.append((op.weights.cpu().numpy().copy(), op.state.cpu().numpy().copy(),
                    art["sorted_vals"].cpu().numpy().copy(), art["seg_offsets"].cpu().numpy().copy()))
    for x, y in zip(*res):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


def test_split_backward_on_two_streams_matches_single_call(gpu_device):
    # sort on a side stream while forward runs on the main one, then the update: same bits as one call
    spec = wl.custom([3000, 200, 40_000], [128, 32, 64], 1, 400, [25.0, 6.0, 12.0], index_dist="zipf", name="split")
    idx, off, w, g = _np_case(spec, 47)
    a = [torch.from_numpy(x).to(gpu_device) for x in (idx, off, g)]
    ref = tl.make_op(spec, gpu_device, max_indices=len(idx), weights=torch.from_numpy(w.copy()).to(gpu_device))
    out_ref = ref.forward(a[0], a[1], spec.batch)
    ref.backward_rowwise_adagrad(a[0], a[1], spec.batch, a[2], 0.01, 1e-8)
    op = tl.make_op(spec, gpu_device, max_indices=len(idx), weights=torch.from_numpy(w.copy()).to(gpu_device))
    assert tbe.tbe_backward_update_rowwise_adagrad(op.h, a[2], 0.01, 1e-8) == tbe.TBE_ERR_INVALID_ARG  # no sort yet
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    for _ in range(3):      # repeated use of the same workspace must stay ordered by the caller's events
        side.wait_stream(main)
        op.backward_sort(a[0], a[1], spec.batch, stream=side)
        out = op.forward(a[0], a[1], spec.batch)
        main.wait_stream(side)
        op.backward_update_rowwise_adagrad(a[2], 0.0, 1e-8)          # lr 0: weights keep their bits
    torch.cuda.synchronize()
    assert torch.equal(out, out_ref)
    op.state.zero_()
    side.wait_stream(main)
    op.backward_sort(a[0], a[1], spec.batch, stream=side)
    main.wait_stream(side)
    op.backward_update_rowwise_adagrad(a[2], 0.01, 1e-8)
    torch.cuda.synchronize()
    assert torch.equal(op.weights, ref.weights) and torch.equal(op.state, ref.state)
    ar, ao = ref.artifacts(), op.artifacts()
    for k in ("sorted_keys", "sorted_vals", "unique_keys", "seg_offsets"):
        assert torch.equal(ar[k], ao[k])


def test_two_steps_carry_moments(gpu_device):
    # second step starts from the first step's weights and moments (Section 5.2: the moment accumulates)
    spec = wl.custom([500, 60], [64, 16], 0, 64, [12.0, 5.0], index_dist="zipf", name="two")
    idx, off, w, g = _np_case(spec, 31)
    idx2, off2, _, g2 = _np_case(spec, 37)
    m = np.zeros(spec.total_rows, np.float32)
    w_ref = w.copy()
    orc.backward_rowwise_adagrad(spec.rows, spec.dims, 0, w_ref, m, idx, off, spec.batch, g, 0.01, 1e-8)
    tl.full_parity_step(spec, idx2, off2, w_ref, g2, gpu_device, m0=m, what="second-step")


def test_check_inputs_reports_bad_batches(gpu_device):
    spec = wl.custom([10, 20], [8, 8], 0, 4, 2.0, pooling_kind="fixed", name="chk")
    op = tl.make_op(spec, gpu_device, max_indices=64)
    off = torch.arange(0, 17, 2, dtype=torch.int64, device=gpu_device)
    idx = torch.zeros(16, dtype=torch.int32, device=gpu_device)
    assert op.check_inputs(idx, off, 4) == tbe.TBE_OK
    bad = idx.clone()
    bad[3] = 10            # table 0 has rows 0..9
    assert op.check_inputs(bad, off, 4) == tbe.TBE_ERR_INDEX_OUT_OF_RANGE
    bad = idx.clone()
    bad[9] = -1
    assert op.check_inputs(bad, off, 4) == tbe.TBE_ERR_INDEX_OUT_OF_RANGE
    ok = idx.clone()
    ok[9] = 19             # table 1 has rows 0..19
    assert op.check_inputs(ok, off, 4) == tbe.TBE_OK
    boff = off.clone()
    boff[2] = 1            # decreasing
    assert op.check_inputs(idx, boff, 4) == tbe.TBE_ERR_INVALID_ARG
    boff = off.clone()
    boff[-1] = 15          # does not end at num_indices
    assert op.check_inputs(idx, boff, 4) == tbe.TBE_ERR_INVALID_ARG
    # host-side argument errors
    assert tbe.tbe_forward(op.h, idx, off, 16, 5, idx, None) == tbe.TBE_ERR_INVALID_ARG       # batch > max
    assert tbe.tbe_forward(op.h, idx, off, 65, 4, idx, None) == tbe.TBE_ERR_INVALID_ARG       # N > max
    assert tbe.tbe_forward(op.h, idx, None, 16, 4, idx, None) == tbe.TBE_ERR_INVALID_ARG      # null offsets
    rc, h2 = tbe.tbe_create([5], [8], 0, 4, 16)
    assert rc == tbe.TBE_OK
    assert tbe.tbe_forward(h2, idx, off, 16, 4, idx, None) == tbe.TBE_ERR_NOT_BOUND
    small = torch.empty(16, dtype=torch.uint8, device=gpu_device)
    assert tbe.tbe_bind(h2, op.weights, op.state, small) == tbe.TBE_ERR_WORKSPACE_TOO_SMALL
    tbe.tbe_destroy(h2)


@pytest.mark.parametrize("k,scale", [(2, 1 / 64), (3, 1 / 128), (4, 1 / 512)])
def test_miniatures_of_the_large_configs(gpu_device, k, scale):
    # same table-count, dim mix, Zipf skew and pooling as configs 2-4, heights and batch scaled down
    spec = wl.config(k, scale=scale)
    idx, off, w, g = _np_case(spec, 41 + k)
    r = tl.full_parity_step(spec, idx, off, w, g, gpu_device, what=f"mini-cfg{k}")
    print(f"mini-cfg{k}", spec.T, spec.batch, r)


def test_profile_slots(gpu_device):
    spec = wl.custom([1000], [64], 0, 64, 8.0, name="prof")
    idx, off, w, g = _np_case(spec, 43)
    op = tl.make_op(spec, gpu_device, max_indices=len(idx))
    a = [torch.from_numpy(x).to(gpu_device) for x in (idx, off, g)]
    op.profile_enable(4)
    for _ in range(3):
        op.forward(a[0], a[1], spec.batch)
        op.backward_rowwise_adagrad(a[0], a[1], spec.batch, a[2], 0.01, 1e-8)
    prof = op.profile_read()
    assert prof["forward"][0] == 3 and prof["reduce_update"][0] == 3 and prof["radix_scatter"][0] == 3 * 2
    assert all(ms >= 0 for _, ms in prof.values())
    op.profile_enable(0)


def test_step_captured_in_a_hip_graph_replays_like_eager(gpu_device):
    """forward + backward only enqueue kernels on the caller's stream (no allocation, no memset, no host
    synchronisation), so a caller can capture a whole step in a HIP graph.  Three replays, with eager work and
    synchronisations in between, must leave exactly the state that three eager steps leave."""
    spec = wl.custom([3000, 64, 900], [64, 16, 128], 1, 256, [20.0, 5.0, 9.0], index_dist="zipf", name="graph")
    idx, off, w, g = _np_case(spec, 41)
    dev = gpu_device
    N, B = int(off[-1]), spec.batch
    d_idx, d_off, d_g = (torch.from_numpy(x).to(dev) for x in (idx, off, g))

    def fresh():
        return tl.make_op(spec, dev, max_indices=N, weights=torch.from_numpy(w.copy()).to(dev))

    # eager reference: three steps, keeping the output of each forward
    op_e = fresh()
    outs_e = []
    for _ in range(3):
        outs_e.append(op_e.forward(d_idx, d_off, B, num_indices=N).clone())
        op_e.backward_rowwise_adagrad(d_idx, d_off, B, d_g, 0.05, 1e-8, num_indices=N)
    torch.cuda.synchronize()

    op_g = fresh()
    out_g = torch.empty(B, spec.sumD, dtype=torch.float32, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        op_g.forward(d_idx, d_off, B, out=out_g, num_indices=N)
        op_g.backward_rowwise_adagrad(d_idx, d_off, B, d_g, 0.05, 1e-8, num_indices=N)
    torch.cuda.synchronize()
    # capturing does not execute: the state is still the initial one
    assert torch.equal(op_g.weights, torch.from_numpy(w).to(dev)) and not op_g.state.any().item()
    scratch = torch.zeros(1 << 20, device=dev)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, outs_e[k]), f"replay {k}: forward output differs from the eager step"
        scratch.add_(1.0)                       # unrelated eager work between the replays
        assert float(scratch.sum().item()) == (k + 1) * scratch.numel()
    assert torch.equal(op_g.weights, op_e.weights) and torch.equal(op_g.state, op_e.state)
    op_e.close()
    op_g.close()
