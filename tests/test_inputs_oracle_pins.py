"""Pins of oracle/inputs_oracle.c against things that are not the oracle: hand-worked examples,
numpy's cumsum, pure-Python dictionary formulations, inverse/round-trip properties and the
degenerate cases (one worker, one shard, empty bags)."""
import os

import numpy as np
import pytest

from oracle import inputs_oracle as io

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_input_kernels.txt")


def _golden():
    d = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            d[k] = np.array([int(x) for x in v], np.int64)
    return d


def _random_bags(rng, n, max_len, hi):
    lens = rng.integers(0, max_len + 1, n).astype(np.int32)
    idx = rng.integers(0, hi, int(lens.sum())).astype(np.int32)
    return lens, idx


def test_handworked_examples():
    g = _golden()
    lo, oo, ix = io.permute_wtb_to_twb(2, 2, 2, g["perm_lengths_in"], g["perm_indices_in"])
    assert lo.tolist() == g["perm_lengths_out"].tolist()
    assert oo.tolist() == g["perm_offsets_out"].tolist()
    assert ix.tolist() == g["perm_indices_out"].tolist()
    lo, oo, ix = io.bucketize_rowwise(g["buck_rows"], 2, 3, g["buck_indices"], g["buck_offsets"])
    assert lo.tolist() == g["buck_lengths_out"].tolist()
    assert oo.tolist() == g["buck_offsets_out"].tolist()
    assert ix.tolist() == g["buck_indices_out"].tolist()


def test_lengths_to_offsets_is_exclusive_cumsum():
    rng = np.random.default_rng(0)
    lens = rng.integers(0, 50, 1000).astype(np.int32)
    off = io.lengths_to_offsets(lens)
    assert off[0] == 0 and np.array_equal(off[1:], np.cumsum(lens.astype(np.int64)))
    assert io.lengths_to_offsets(np.zeros(0, np.int32)).tolist() == [0]
    big = np.full(3, 2 ** 30, np.int32)               # sums past 2^31 must not wrap
    assert io.lengths_to_offsets(big).tolist() == [0, 2 ** 30, 2 ** 31, 3 * 2 ** 30]
    with pytest.raises(ValueError):
        io.lengths_to_offsets(np.array([1, -1], np.int32))


@pytest.mark.parametrize("seed", range(5))
def test_permute_against_dictionary_formulation(seed):
    rng = np.random.default_rng(seed)
    W, T, B = int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 6))
    lens, idx = _random_bags(rng, W * T * B, 4, 1000)
    off_in = np.concatenate([[0], np.cumsum(lens)])
    bags = {}
    for w in range(W):
        for t in range(T):
            for b in range(B):
                j = (w * T + t) * B + b
                bags[(t, w, b)] = idx[off_in[j]:off_in[j + 1]].tolist()
    lo, oo, ix = io.permute_wtb_to_twb(W, T, B, lens, idx)
    flat, ref_len = [], []
    for key in sorted(bags):                          # (t, w, b) lexicographic = output order
        flat += bags[key]
        ref_len.append(len(bags[key]))
    assert lo.tolist() == ref_len and ix.tolist() == flat
    assert np.array_equal(oo, np.concatenate([[0], np.cumsum(ref_len)]))
    # permuting back with the roles of W and T exchanged is the inverse
    lb, ob, ib = io.permute_wtb_to_twb(T, W, B, lo, ix)
    assert np.array_equal(lb, lens) and np.array_equal(ib, idx)


def test_permute_single_worker_or_single_table_is_identity():
    rng = np.random.default_rng(9)
    lens, idx = _random_bags(rng, 12, 5, 100)
    for W, T in ((1, 4), (4, 1)):
        lo, oo, ix = io.permute_wtb_to_twb(W, T, 3, lens, idx)
        assert np.array_equal(lo, lens) and np.array_equal(ix, idx)


@pytest.mark.parametrize("seed", range(5))
def test_bucketize_against_pure_python(seed):
    rng = np.random.default_rng(100 + seed)
    T, B, W = int(rng.integers(1, 4)), int(rng.integers(1, 6)), int(rng.integers(1, 6))
    rows = rng.integers(1, 40, T).astype(np.int64)
    lens = rng.integers(0, 7, T * B).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, rows[t], int(lens[t * B:(t + 1) * B].sum())) for t in range(T)]).astype(np.int32)
    lo, oo, ix = io.bucketize_rowwise(rows, B, W, idx, off)
    out = {}
    for t in range(T):
        blk = -(-int(rows[t]) // W)
        for b in range(B):
            for p in range(off[t * B + b], off[t * B + b + 1]):
                w = int(idx[p]) // blk
                out.setdefault((w, t, b), []).append(int(idx[p]) - w * blk)
    flat, ref_len = [], []
    for w in range(W):
        for t in range(T):
            for b in range(B):
                flat += out.get((w, t, b), [])
                ref_len.append(len(out.get((w, t, b), [])))
    assert lo.tolist() == ref_len and ix.tolist() == flat
    assert np.array_equal(oo, np.concatenate([[0], np.cumsum(ref_len)]))
    # nothing lost, every local id inside its shard, the last shard may be short
    assert int(lo.sum()) == len(idx)
    for t in range(T):
        blk = -(-int(rows[t]) // W)
        for w in range(W):
            for b in range(B):
                j = (w * T + t) * B + b
                seg = ix[oo[j]:oo[j + 1]]
                assert seg.size == 0 or (seg.min() >= 0 and seg.max() < min(blk, int(rows[t]) - w * blk))


def test_bucketize_one_shard_is_identity_and_preserves_order():
    rng = np.random.default_rng(5)
    rows = np.array([17, 5], np.int64)
    lens = rng.integers(0, 6, 8).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, 17, int(lens[:4].sum())), rng.integers(0, 5, int(lens[4:].sum()))]).astype(np.int32)
    lo, oo, ix = io.bucketize_rowwise(rows, 4, 1, idx, off)
    assert np.array_equal(lo, lens) and np.array_equal(oo, off) and np.array_equal(ix, idx)
    with pytest.raises(ValueError):
        io.bucketize_rowwise(rows, 4, 2, np.full_like(idx, 17), off)


def test_bucketize_then_permute_gives_each_shard_a_valid_embedding_input():
    # the two kernels compose as in Section 7.1: bucketize emits (W,T,B); a shard's slice of it is a
    # table-major (T,B) input whose indices are valid local rows of that shard
    rng = np.random.default_rng(3)
    T, B, W = 2, 3, 2
    rows = np.array([9, 4], np.int64)
    lens = rng.integers(1, 5, T * B).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, 9, int(lens[:3].sum())), rng.integers(0, 4, int(lens[3:].sum()))]).astype(np.int32)
    lo, oo, ix = io.bucketize_rowwise(rows, B, W, idx, off)
    for w in range(W):
        sl = lo[w * T * B:(w + 1) * T * B]
        seg = ix[oo[w * T * B]:oo[(w + 1) * T * B]]
        assert int(sl.sum()) == len(seg)
    recon = []
    for t in range(T):
        blk = -(-int(rows[t]) // W)
        for b in range(B):
            got = []
            for w in range(W):
                j = (w * T + t) * B + b
                got += (ix[oo[j]:oo[j + 1]] + w * blk).tolist()
            assert sorted(got) == sorted(idx[off[t * B + b]:off[t * B + b + 1]].tolist())
