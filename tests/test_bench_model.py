"""The byte model behind bench.py's roofline figures, checked on a case small enough to count by hand."""
import numpy as np

import bench
from paper_2104_05158_amd import workloads as wl


def test_kernel_bytes_on_a_hand_counted_case():
    # two fp16 tables, D = 8 and 16, batch 4: table 0 gets 10 lookups on 3 distinct rows, table 1 gets 6 on 6
    spec = wl.custom([100, 50], [8, 16], 1, 4, 1.0)
    n_t, u_t = np.array([10.0, 6.0]), np.array([3.0, 6.0])
    comp, logical = bench.kernel_bytes(spec, n_t, u_t, np.zeros(2), np.zeros(2))
    N, U, bags, B = 16, 9, 8, 4
    io_fwd = N * 4 + bags * 8 + B * 4 * (8 + 16)                       # indices, offsets, fp32 output
    assert comp["forward"] == (3 * 8 + 6 * 16) * 2 + io_fwd == 752      # each distinct row once
    assert logical["forward"] == (10 * 8 + 6 * 16) * 2 + io_fwd == 864  # every lookup a row read
    rmw = 3 * (2 * 8 * 2 + 8) + 6 * (2 * 16 * 2 + 8)                    # row read + write, moment read + write
    grad_once = min(10 * 4 * 8, B * 4 * 8) + min(6 * 4 * 16, B * 4 * 16)  # a gradient row at most once per bag
    assert comp["reduce_update"] == N * 4 + U * 8 + grad_once + rmw == 1072
    assert logical["reduce_update"] == N * 4 + U * 8 + (10 * 4 * 8 + 6 * 4 * 16) + rmw == 1392
    assert comp["radix_hist"] == N * 4 and comp["radix_scatter"] == N * 16
    assert comp["runlength"] == N * 4 + U * 8
    assert comp["long_fixup"] == 0 and comp["dense_rows"] == 0


def test_long_runs_add_partial_rows_and_16_bit_types_halve_the_row_bytes():
    spec = wl.custom([1000], [64], 0, 2048, 1.0)
    n_t, u_t = np.array([5000.0]), np.array([100.0])
    base, _ = bench.kernel_bytes(spec, n_t, u_t, np.zeros(1), np.zeros(1))
    # one run of 1280 lookups: a partial fp32 row per 128 positions plus two ragged ends, written and read once
    with_long, _ = bench.kernel_bytes(spec, n_t, u_t, np.array([1280.0]), np.array([1.0]))
    rows = 1280 / 128 + 2
    # the update kernel no longer gathers that run nor updates its row; window_runs reads its payloads and gradient
    # rows and writes the partial rows (+ a 16-byte piece record read and written each); the fix-up reads them
    assert base["reduce_update"] - with_long["reduce_update"] == 1280 * 4 + (2 * 64 * 4 + 8)
    assert with_long["window_runs"] == 1280 * 4 + min(1280 * 4 * 64, 2048 * 4 * 64) + rows * (4 * 64 + 32)
    assert with_long["long_fixup"] == rows * 4 * 64 + (2 * 64 * 4 + 8)
    assert bench.window_count(65536, 128, 4) == 16 and bench.window_count(65536, 64, 4) == 8
    assert bench.window_count(700, 128, 4) == 1 and bench.window_count(1 << 20, 128, 4) == 16
    # the same run beyond the dense threshold: its lookups leave the update kernel; dense_rows reads their payloads
    # and the table's gradient block once and writes one partial row per 1024-bag slice (2 here)
    with_dense, _ = bench.kernel_bytes(spec, n_t, u_t, np.zeros(1), np.zeros(1), ndense_t=np.array([1280.0]),
                                       udense_t=np.array([1.0]))
    assert with_dense["dense_rows"] == 1280 * 4 + 2048 * 4 * 64 + 2 * 4 * 64
    assert with_dense["long_fixup"] == 2 * 4 * 64 + (2 * 64 * 4 + 8)
    assert base["reduce_update"] - with_dense["reduce_update"] == 1280 * 4 + (2 * 64 * 4 + 8)
    assert bench.dense_threshold(65536) == 8192 and bench.dense_threshold(700) == 1024 and bench.dense_threshold(16384) == 2048
    half, _ = bench.kernel_bytes(spec, n_t, u_t, np.zeros(1), np.zeros(1), so=2, sg=2)
    assert base["forward"] - half["forward"] == 2048 * 2 * 64
    assert base["reduce_update"] - half["reduce_update"] == min(5000, 2048) * 2 * 64


def test_sort_bytes_per_launch_follow_the_tables_pass_counts():
    # 300 rows -> 9 bits -> 2 passes; 70000 rows -> 17 bits -> 3 passes
    assert bench.sort_passes([300, 70000, 256, 2 ** 24, 2 ** 24 + 1]).tolist() == [2, 3, 1, 3, 4]
    spec = wl.custom([300, 70000], [8, 16], 1, 4, 1.0)
    n_t, u_t = np.array([10.0, 6.0]), np.array([3.0, 6.0])
    comp, _ = bench.kernel_bytes(spec, n_t, u_t, np.zeros(2), np.zeros(2), passes_t=bench.sort_passes(spec.rows))
    # three launches; batch <= 65536: the payload is 2 bytes between the passes.  First pass of a table: index in,
    # key + short payload out (10 bytes per lookup); middle pass 6 in + 6 out; last pass 6 in + 8 out
    assert comp["radix_scatter"] == (10 * (10 + 14) + 6 * (10 + 12 + 14)) / 3
    assert comp["radix_hist"] == (10 * 4 * 2 + 6 * 4 * 3) / 3
    big = wl.custom([300, 70000], [8, 16], 1, 70000, 1.0)
    comp, _ = bench.kernel_bytes(big, n_t, u_t, np.zeros(2), np.zeros(2), passes_t=bench.sort_passes(big.rows))
    assert comp["radix_scatter"] == (10 * (12 + 16) + 6 * (12 + 32)) / 3       # 4-byte payloads beyond 65536 bags
    one = wl.custom([200], [8], 1, 4, 1.0)
    comp, _ = bench.kernel_bytes(one, np.array([10.0]), np.array([3.0]), np.zeros(1), np.zeros(1),
                                 passes_t=bench.sort_passes(one.rows))
    assert comp["radix_scatter"] == 10 * 12                                     # an only pass: index in, key + payload out


def test_default_invocation_is_config_4_with_3_and_2_alongside():
    a = bench.parse_args([])
    assert a.config is None and a.others is None and a.gpus == 1
    assert bench.parse_args(["--config", "2"]).config == 2
