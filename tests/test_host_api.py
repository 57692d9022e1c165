"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/tbe.h declares, and
its host-side logic (config validation, layout tables, workspace sizing, error strings) behaves as
the header says.  No kernel is launched and no device memory is touched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2104_05158_amd import tbe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header="tbe.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tbe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(tbe.EXPORTED)
    L = ctypes.CDLL(tbe.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    names = _declared_symbols("tbe_inputs.h")
    assert set(names) == set(tbe.EXPORTED_INPUTS)
    for n in names:
        assert hasattr(L, n), n


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(tbe, "_lib", None)
    monkeypatch.setattr(tbe, "LIB_PATH", "/nonexistent/libtbe.so")
    with pytest.raises(ImportError):
        tbe.lib()


def test_status_strings():
    seen = {tbe.status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert tbe.status_string(99) == "unknown status"


def test_create_validates_config():
    ok = lambda *a, **k: tbe.tbe_create(*a, **k)[0]
    assert ok([10], [8], 0, 4, 100) == tbe.TBE_OK
    assert ok([], [], 0, 4, 100) == tbe.TBE_ERR_INVALID_ARG
    assert ok([0], [8], 0, 4, 100) == tbe.TBE_ERR_INVALID_ARG
    assert ok([10], [0], 0, 4, 100) == tbe.TBE_ERR_INVALID_ARG
    assert ok([10], [8], 0, -1, 100) == tbe.TBE_ERR_INVALID_ARG
    assert ok([10], [8], 0, 4, -1) == tbe.TBE_ERR_INVALID_ARG
    assert ok([10], [6], 0, 4, 100) == tbe.TBE_ERR_UNSUPPORTED          # dim not a multiple of 4
    assert ok([10], [516], 0, 4, 100) == tbe.TBE_ERR_UNSUPPORTED        # dim too large
    assert ok([10], [8], 2, 4, 100) == tbe.TBE_ERR_UNSUPPORTED          # unknown storage type
    assert ok([10], [8], 0, 4, 100, pooling=1) == tbe.TBE_ERR_UNSUPPORTED
    assert ok([2 ** 31, 2 ** 31], [8, 8], 0, 4, 100) == tbe.TBE_ERR_UNSUPPORTED   # 2^32 rows
    assert ok([10], [8], 0, 4, 2 ** 31) == tbe.TBE_ERR_UNSUPPORTED
    # indices are int32: a single table of 2^31 rows or more cannot be addressed, whatever the sum is
    assert ok([2 ** 31], [8], 0, 4, 100) == tbe.TBE_ERR_UNSUPPORTED
    assert ok([5, 2 ** 31 + 7], [8, 8], 1, 4, 100) == tbe.TBE_ERR_UNSUPPORTED
    assert ok([2 ** 31 - 1], [8], 0, 4, 100) == tbe.TBE_OK
    assert ok([10] * 4, [8] * 4, 0, 2 ** 30, 100) == tbe.TBE_ERR_UNSUPPORTED     # T*B overflows
    assert tbe.lib().tbe_create(None, None) == tbe.TBE_ERR_INVALID_ARG
    assert tbe.tbe_destroy(None) == tbe.TBE_OK


def test_layout_tables_and_sizes():
    rows, dims = [10, 3, 7], [8, 128, 4]
    for dtype, es in ((0, 4), (1, 2)):
        rc, h = tbe.tbe_create(rows, dims, dtype, 16, 1000)
        assert rc == tbe.TBE_OK
        rc, q = tbe.tbe_query_sizes(h, 3)
        assert rc == tbe.TBE_OK
        assert q["weight_offsets"].tolist() == [0, 80, 80 + 384, 80 + 384 + 28]
        assert q["state_offsets"].tolist() == [0, 10, 13, 20]
        assert q["out_col_offsets"].tolist() == [0, 8, 136, 140]
        assert q["weight_bytes"] == (80 + 384 + 28) * es and q["state_bytes"] == 80
        # the sort needs two (key, payload) pairs of max_indices entries at the least
        assert q["workspace_bytes"] >= 4 * 4 * 1000 and q["workspace_bytes"] % 256 == 0
        tbe.tbe_destroy(h)
    # workspace grows with max_indices, and is computed (not allocated) for the largest config
    rc, h = tbe.tbe_create([5 * 10 ** 7] * 8, [128] * 8, 1, 65536, 800_000_000)
    assert rc == tbe.TBE_OK
    rc, q = tbe.tbe_query_sizes(h, 8)
    assert 16 * 800_000_000 < q["workspace_bytes"] < 40 * 800_000_000
    tbe.tbe_destroy(h)


def test_calls_on_unbound_or_null_handles():
    rc, h = tbe.tbe_create([10], [8], 0, 4, 100)
    L = tbe.lib()
    assert L.tbe_forward(h, None, None, 0, 0, None, None) == tbe.TBE_ERR_NOT_BOUND
    assert L.tbe_backward_rowwise_adagrad(h, None, None, 0, 0, None, 0.1, 1e-8, None) == tbe.TBE_ERR_NOT_BOUND
    assert tbe.tbe_backward_artifacts(h)[0] == tbe.TBE_ERR_NOT_BOUND
    assert L.tbe_forward(None, None, None, 0, 0, None, None) == tbe.TBE_ERR_INVALID_ARG
    assert L.tbe_bind(h, None, None, None, 0) == tbe.TBE_ERR_INVALID_ARG
    assert L.tbe_query_sizes(None, None, None, None, None, None, None) == tbe.TBE_ERR_INVALID_ARG
    assert tbe.tbe_last_hip_error(h) == ""
    tbe.tbe_destroy(h)


def test_input_side_entry_points_validate_on_the_host():
    """Every error below is detected before anything is enqueued (there is no GPU here)."""
    L = tbe.lib()
    assert tbe.tbe_inputs_scratch_bytes(0) >= 16 and tbe.tbe_inputs_scratch_bytes(0) % 256 == 0
    n = 10 ** 6
    need = tbe.tbe_inputs_scratch_bytes(n)
    assert 8 * (n + 1) <= need <= 8 * (n + 1) + 8 * (n // 4096 + 2) + 512
    fake = 0x10000  # an aligned non-null address that is never dereferenced on these paths
    bad = tbe.TBE_ERR_INVALID_ARG
    # lengths -> offsets
    assert L.tbe_lengths_to_offsets(fake, -1, fake, fake, need, None) == bad
    assert L.tbe_lengths_to_offsets(None, 5, fake, fake, need, None) == bad
    assert L.tbe_lengths_to_offsets(fake, 5, None, fake, need, None) == bad
    assert L.tbe_lengths_to_offsets(fake, 5, fake, None, need, None) == bad
    assert L.tbe_lengths_to_offsets(fake, n, fake, fake, need - 1, None) == bad          # scratch too small
    assert L.tbe_lengths_to_offsets(fake, 5, fake, fake + 8, need, None) == bad          # scratch misaligned
    assert L.tbe_lengths_to_offsets(fake + 4, 5, fake, fake, need, None) == bad          # lengths misaligned
    assert L.tbe_lengths_to_offsets(fake, 2 ** 31, fake, fake, 2 ** 40, None) == tbe.TBE_ERR_UNSUPPORTED
    # permute
    assert L.tbe_permute_wtb_to_twb(0, 1, 1, fake, fake, 1, fake, fake, fake, fake, need, None) == bad
    assert L.tbe_permute_wtb_to_twb(2, 2, 2, None, fake, 1, fake, fake, fake, fake, need, None) == bad
    assert L.tbe_permute_wtb_to_twb(2, 2, 2, fake, None, 1, fake, fake, fake, fake, need, None) == bad
    assert L.tbe_permute_wtb_to_twb(2, 2, 2, fake, fake, 1, fake, fake, fake, fake, 8, None) == bad
    assert L.tbe_permute_wtb_to_twb(2 ** 11, 2 ** 10, 2 ** 10, fake, fake, 1, fake, fake, fake, fake, 2 ** 40,
                                    None) == tbe.TBE_ERR_UNSUPPORTED
    # bucketize
    assert L.tbe_bucketize_rowwise(1, 4, 0, fake, fake, fake, 1, fake, fake, fake, fake, need, None) == bad
    assert L.tbe_bucketize_rowwise(1, 4, 2, None, fake, fake, 1, fake, fake, fake, fake, need, None) == bad
    assert L.tbe_bucketize_rowwise(1, 4, 2, fake, fake, fake, 1, fake, fake, fake, fake, 8, None) == bad
    assert L.tbe_bucketize_rowwise(1, 4, 1025, fake, fake, fake, 1, fake, fake, fake, fake, 2 ** 40,
                                   None) == tbe.TBE_ERR_UNSUPPORTED


def test_read_probe_validates_its_arguments_on_the_host():
    L = tbe.lib()
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    assert L.tbe_probe_read(None, sz(1 << 20), 1, vp(256), None) == tbe.TBE_ERR_INVALID_ARG      # null source
    assert L.tbe_probe_read(vp(256), sz(1 << 20), 1, None, None) == tbe.TBE_ERR_INVALID_ARG      # null sink
    assert L.tbe_probe_read(vp(264), sz(1 << 20), 1, vp(256), None) == tbe.TBE_ERR_INVALID_ARG   # source not 16-aligned
    assert L.tbe_probe_read(vp(256), sz(8), 1, vp(256), None) == tbe.TBE_ERR_INVALID_ARG         # less than one word
    assert L.tbe_probe_read(vp(256), sz(1 << 20), 0, vp(256), None) == tbe.TBE_ERR_INVALID_ARG   # no pass
    assert L.tbe_probe_read(vp(256), sz(1 << 20), 1, vp(258), None) == tbe.TBE_ERR_INVALID_ARG   # sink not 4-aligned


def test_optimizer_and_dtype_configuration():
    rows, dims = [10, 3], [8, 4]
    elems = 10 * 8 + 3 * 4
    for opt, want in ((tbe.TBE_OPT_ROWWISE_ADAGRAD, 4 * 13), (tbe.TBE_OPT_ADAGRAD, 4 * elems),
                      (tbe.TBE_OPT_ADAM, 8 * elems)):
        rc, h = tbe.tbe_create(rows, dims, 1, 4, 100, optimizer=opt, output_dtype=tbe.TBE_DTYPE_FP16,
                               grad_dtype=tbe.TBE_DTYPE_BF16)
        assert rc == tbe.TBE_OK
        assert tbe.tbe_query_sizes(h, 2)[1]["state_bytes"] == want
        tbe.tbe_destroy(h)
    bad = tbe.TBE_ERR_UNSUPPORTED
    assert tbe.tbe_create(rows, dims, 0, 4, 100, optimizer=3)[0] == bad
    assert tbe.tbe_create(rows, dims, 0, 4, 100, output_dtype=tbe.TBE_DTYPE_BF16)[0] == bad
    assert tbe.tbe_create(rows, dims, 0, 4, 100, grad_dtype=3)[0] == bad
    assert tbe.tbe_create(rows, dims, tbe.TBE_DTYPE_BF16, 4, 100)[0] == bad
    assert tbe.tbe_create(rows, dims, 0, 4, 100, layout=2)[0] == bad
    # entry points of another optimizer are refused before anything is enqueued (unbound handle: NOT_BOUND first)
    rc, h = tbe.tbe_create(rows, dims, 0, 4, 100, optimizer=tbe.TBE_OPT_ADAM)
    L = tbe.lib()
    assert L.tbe_backward_adam(h, None, None, 0, 0, None, 0.1, 0.9, 0.999, 1e-8, 1, None) == tbe.TBE_ERR_NOT_BOUND
    assert L.tbe_backward_update_adagrad(h, None, 0.1, 1e-8, None) == tbe.TBE_ERR_NOT_BOUND
    tbe.tbe_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in (r.stdout + r.stderr)
    assert not r.stdout.strip().startswith("{")     # no result line
