#!/usr/bin/env python3
"""Benchmark of the table-batched embedding-bag hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: tbe_forward, then
tbe_backward_rowwise_adagrad (sort plan, radix sort, run-length, fused reduce + row-wise AdaGrad,
long runs by bag window, dense hot rows, fix-up) on the same batch.  Inputs, weights and optimizer state are resident in HBM
before the timed region; a rotation of pre-generated batches (different seeds) is used so that no step
re-reads the previous step's index stream.

With no --config the headline workload is configuration 4 (the largest single-GPU share: 400 tables,
120 GB, 786 M lookups per step) and configurations 3 and 2 are run afterwards in the same process and
reported under "other_configs".  The timed steps run with the library's event profiling switched off;
the per-kernel durations come from a second loop of the same steps with profiling on.

Prints ONE JSON line: lookups/s of fwd+bwd (whole job = this one GPU), plus
  roofline      -- the dominant kernel's algorithmic (compulsory: each distinct byte once) bytes per launch /
                   its mean launch duration, measured with HIP events recorded by the library on the launch
                   stream; the every-lookup-counted ("logical") rate is given beside it
  cpu_baseline  -- the CPU oracle, as it stands, timed on a bounded sample of the same workload (one thread,
                   and one thread per host core on disjoint tables), and the parity of the GPU's first step
                   against it on that sample
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic.txt")


def parse_args(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="benchmark configuration 1..4; default: 4 as the headline, then 3 and 2 under other_configs")
    ap.add_argument("--others", type=str, default=None,
                    help="comma-separated configurations to run after the headline one (default 3,2 when "
                         "--config is not given, none otherwise)")
    ap.add_argument("--paper-membench", choices=["fp32", "fp16"], default=None,
                    help="run the Appendix A memory-benchmark shape instead of a config")
    ap.add_argument("--batch", type=int, default=None, help="batch override (memory benchmark sweep)")
    ap.add_argument("--zipf", type=float, default=None,
                    help="override the configuration's index distribution: Zipf exponent, 0 = uniform (sensitivity runs)")
    ap.add_argument("--rotation", type=int, default=4, help="number of pre-generated batches")
    ap.add_argument("--flush", action="store_true", help="write a 1 GiB scratch between steps (cold caches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-lookups", type=float, default=8e6)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference dispatch for HBM counter scaling)")
    ap.add_argument("--fwd-only", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture each batch's step in a HIP graph and time the replays")
    ap.add_argument("--optimizer", choices=["rowwise_adagrad", "adagrad", "adam"], default="rowwise_adagrad")
    ap.add_argument("--out-dtype", choices=["fp32", "fp16"], default="fp32",
                    help="type of the pooled output (Section 8.4 ships it through an FP16 all-to-all)")
    ap.add_argument("--layout", choices=["batch", "table"], default="batch",
                    help="layout of the pooled output and the upstream gradient: [B, sumD] rows, or one [B, D_t] "
                         "block per table")
    ap.add_argument("--grad-dtype", choices=["fp32", "fp16", "bf16"], default="fp32",
                    help="type of the upstream gradient (Section 8.4 receives it through a BF16 all-to-all)")
    ap.add_argument("--inputs", action="store_true",
                    help="time the input-side kernels (row-wise bucketize, (W,T,B)->(T,W,B) permute, lengths->offsets) "
                         "on the chosen config's batch instead of the embedding step")
    ap.add_argument("--shards", type=int, default=8, help="W for --inputs")
    ap.add_argument("--overlap", action="store_true",
                    help="run the backward's sort (it needs only the indices) on a second stream beside the "
                         "forward gather; measured: no gain, both kernels fill the chip on their own")
    return ap.parse_args(argv)


def per_table_counts(spec, batch):
    off = batch.offsets
    B = spec.batch
    bounds = off[:: B][: spec.T + 1] if B > 0 else off
    return np.diff(bounds.cpu().numpy())


LONG_RUN = 512    # runs longer than this are summed in pieces (kLongRun): by bag window, or as dense rows


def window_count(batch, D, grad_bytes):
    """Bag windows the library cuts a long run of a D-column table into (window_geom in the library): about 2 MiB
    of the table's gradient block per window, at most 16 windows."""
    bags = 1024
    while bags * 2 * D * grad_bytes <= (2 << 20):
        bags *= 2
    nwin = -(-batch // bags)
    if nwin > 16:
        bags = -(-(-(-batch // 16)) // 1024) * 1024
        nwin = -(-batch // bags)
    return max(nwin, 1)


def sort_passes(rows):
    """Radix passes (8 bits each at most) the library needs for a table of `rows` rows: the sort is segmented
    by table and only the bits of the table's own row index are sorted."""
    bits = np.maximum(1, np.ceil(np.log2(np.maximum(np.asarray(rows, np.float64), 2.0)))).astype(np.int64)
    return np.ceil(bits / 8.0)


DENSE_SLICE = 1024   # bags per partial row of a dense run (kDenseSlice)


def dense_threshold(batch):
    """Run length beyond which the library sums a run as counts x gradient block (dense_threshold in the library)."""
    nslices = -(-max(batch, 1) // DENSE_SLICE)
    return max(1024, batch // 8, 128 * ((nslices + 1) // 2 + 3))


def kernel_bytes(spec, n_t, u_t, nlong_t, ulong_t, so=4, sg=4, state_per_elem=0, passes_t=None,
                 ndense_t=None, udense_t=None, long_rows_t=None):
    """Bytes one launch of each kernel must move, two ways.
    compulsory: every distinct byte once -- what an ideal cache would leave for HBM; the roofline numerator.
    logical:    every lookup counted as a row read -- a throughput figure that caches can push past the HBM peak.
    n_t / u_t: lookups / distinct rows per table; nlong_t / ulong_t: lookups in / number of runs longer than LONG_RUN
    that window_runs_kernel sums piece by piece (long_rows_t: their partial rows, default one per 128 lookups + 2);
    ndense_t / udense_t: the same for the runs beyond the dense threshold, which dense_rows_kernel sums; so / sg: bytes per output / gradient element; state_per_elem: float32 optimizer
    states per weight element (0 = one moment per row); passes_t: radix passes per table (default: one pass for
    every table, the figure per pass).
    Sort figures are per launch: a table's first scatter pass reads the caller's 4-byte indices and writes key +
    payload, later passes read and write both; between the passes the payload is 2 bytes while the batch is at most
    65536 (10 / 12 / 14 bytes per lookup in a first / middle / last pass, 12 in an only pass), else 4 (12 / 16 / 16)."""
    sw = 4 if spec.dtype == 0 else 2
    D = spec.dims.astype(np.float64)
    B = float(spec.batch)
    N = float(n_t.sum())
    U = float(u_t.sum())
    if ndense_t is None:
        ndense_t, udense_t = np.zeros(spec.T), np.zeros(spec.T)
    bags = float(spec.T) * B
    io_fwd = N * 4 + bags * 8 + (B * so * D).sum()
    state_rw = 8 * D * state_per_elem if state_per_elem else 8.0
    row_rw = 2 * D * sw + state_rw                       # a table row and its optimizer state, read + written
    slab = B * sg * D
    partial_rows = nlong_t / 128.0 + 2 * ulong_t if long_rows_t is None else long_rows_t   # fp32 partial rows of long runs
    dense_rows = udense_t * float(-(-spec.batch // DENSE_SLICE))   # one fp32 partial row per 1024-bag slice
    n_upd = n_t - ndense_t - nlong_t                     # lookups the update kernel gathers itself
    if passes_t is None:
        scatter = N * 16
        hist = N * 4
    else:
        launches = float(np.max(passes_t))
        if spec.batch <= 65536:
            per_lookup = np.where(passes_t <= 1, 12.0, 10.0 + 12.0 * (passes_t - 2) + 14.0)
        else:
            per_lookup = 12.0 + 16.0 * (passes_t - 1)
        scatter = float((n_t * per_lookup).sum()) / launches
        hist = float((n_t * 4 * passes_t).sum()) / launches
    comp = {
        "forward": float((u_t * D * sw).sum() + io_fwd),
        "sort_plan": 0.0,
        "radix_hist": hist,
        "radix_scatter": scatter,
        "radix_scan": 0.0,
        "runlength": N * 4 + U * 8,
        # payloads + run descriptors + each gradient row once + the rows it updates itself
        "reduce_update": float(n_upd.sum() * 4 + U * 8 + np.minimum(n_upd * sg * D, slab).sum() +
                               ((u_t - ulong_t - udense_t) * row_rw).sum()),
        # payloads of the long runs + each gradient row they touch once + their partial rows + 16-byte piece records
        "window_runs": float(nlong_t.sum() * 4 + np.minimum(nlong_t * sg * D, slab).sum() +
                             (partial_rows * (4 * D + 32)).sum()),
        # payloads of the dense runs + the gradient block of every table that has dense runs + its partial rows
        "dense_rows": float(ndense_t.sum() * 4 + (np.where(udense_t > 0, slab, 0.0)).sum() + (dense_rows * 4 * D).sum()),
        "long_fixup": float(((partial_rows + dense_rows) * 4 * D + (ulong_t + udense_t) * row_rw).sum()),
    }
    logical = dict(comp)
    logical["forward"] = float((n_t * D * sw).sum() + io_fwd)
    logical["reduce_update"] = float(comp["reduce_update"] - np.minimum(n_upd * sg * D, slab).sum() + (n_upd * sg * D).sum())
    return comp, logical


# ---------------------------------------------------------------- CPU baseline (the oracle) and step-0 parity

def host_info():
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"nproc": os.cpu_count(), "usable_cores": usable, "cpu_model": model}


def pick_sample_tables(spec, n_t, target_lookups, byte_cap=24e9, start=0):
    """Tables (in order, from `start`) whose lookups add up to about `target_lookups`."""
    take, tot, wbytes = [], 0, 0
    for t in range(start, spec.T):
        tb = int(spec.rows[t]) * int(spec.dims[t]) * (4 if spec.dtype == 0 else 2)
        if take and (tot + n_t[t] > 1.5 * target_lookups or wbytes + tb > byte_cap):
            continue
        take.append(int(t))
        tot += int(n_t[t])
        wbytes += tb
        if tot >= target_lookups:
            break
    return take


def table_slices(spec):
    woffs = np.concatenate([[0], np.cumsum(spec.rows * spec.dims.astype(np.int64))])
    cols = np.concatenate([[0], np.cumsum(spec.dims)]).astype(np.int64)
    R = np.concatenate([[0], np.cumsum(spec.rows)]).astype(np.int64)
    return woffs, cols, R


def sub_problem(spec, batch, take, weights, state, grad32_cols):
    """Host copies of the tables in `take` as a problem of their own (tables are independent, so the oracle's
    result for them is exactly its result inside the full workload)."""
    B = spec.batch
    woffs, cols, R = table_slices(spec)
    off = batch.offsets
    idx_parts, len_parts, w_parts, m_parts = [], [], [], []
    for t in take:
        lo, hi = int(off[t * B]), int(off[(t + 1) * B])
        idx_parts.append(batch.indices[lo:hi].cpu().numpy())
        len_parts.append(np.diff(off[t * B:(t + 1) * B + 1].cpu().numpy()))
        w_parts.append(weights[int(woffs[t]):int(woffs[t + 1])].cpu().numpy())
        m_parts.append(state[int(R[t]):int(R[t + 1])].cpu().numpy())
    offsets = np.zeros(len(take) * B + 1, np.int64)
    offsets[1:] = np.cumsum(np.concatenate(len_parts))
    return dict(rows=spec.rows[take], dims=spec.dims[take],
                indices=np.concatenate(idx_parts).astype(np.int32), offsets=offsets,
                w=np.concatenate(w_parts), m=np.concatenate(m_parts),
                g=np.ascontiguousarray(np.concatenate([grad32_cols(t) for t in take], axis=1)))


def _err_stats(err):
    err = np.asarray(err, np.float64).ravel()
    if err.size == 0:
        return {"max": 0.0, "p9999": 0.0, "n": 0}
    return {"max": float(err.max()), "p9999": float(np.quantile(err, 0.9999)), "n": int(err.size)}


def cpu_baseline(spec, sample, gpu_step0, all_core_jobs):
    """Times the CPU oracle (single thread, as it stands) on the sampled tables of the first batch, compares
    the GPU's first step with it, and times it once more with one thread per usable host core, each thread on
    disjoint tables of its own (the oracle itself stays single-threaded: tables are independent)."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import tbe_oracle as orc

    B = spec.batch
    orc.build()
    p = sample
    t0 = time.perf_counter()
    out, absref = orc.forward(p["rows"], p["dims"], spec.dtype, p["w"], p["indices"], p["offsets"], B, want_absref=True)
    t1 = time.perf_counter()
    w1, m1 = p["w"].copy(), p["m"].copy()
    tc = time.perf_counter()
    orc.backward_rowwise_adagrad(p["rows"], p["dims"], spec.dtype, w1, m1, p["indices"], p["offsets"], B, p["g"],
                                 spec.lr, spec.eps)
    t2 = time.perf_counter()
    n = int(p["offsets"][-1])
    fwd_s, bwd_s = t1 - t0, t2 - tc
    info = host_info()
    res = {
        "value": n / (fwd_s + bwd_s), "unit": "lookups/s", "cores": 1, "kind": "oracle",
        "sample": f"tables {p['take'][0]}..{p['take'][-1]} ({len(p['take'])} of {spec.T}) of the first batch, {n} lookups, "
                  f"fwd {fwd_s:.2f}s + bwd {bwd_s:.2f}s; plain C -O2, fp64 accumulation",
        "fwd_s": fwd_s, "bwd_s": bwd_s, "lookups": n, **info,
    }

    # ---- parity of the GPU's first step on the same tables (the error is relative to the condition-aware
    # scale sum|terms| for the output; updated weights and moments are compared through the oracle's rounded
    # results, relative to |w_old| + |step| and to the new moment)
    if gpu_step0 is not None:
        art = orc.sort_artifacts(p["rows"], B, p["indices"], p["offsets"])
        g_out = gpu_step0["out"].astype(np.float64)
        scale = np.maximum(np.abs(out.astype(np.float64)), absref) + 1e-300
        e_f = np.abs(g_out - out.astype(np.float64)) / scale
        keys = art.unique_keys.astype(np.int64)
        Rs = np.concatenate([[0], np.cumsum(p["rows"])]).astype(np.int64)
        Ws = np.concatenate([[0], np.cumsum(p["rows"] * p["dims"].astype(np.int64))]).astype(np.int64)
        tt = np.searchsorted(Rs, keys, side="right") - 1
        e_w, e_m, sub_abs = [], [], []
        # fp16 storage: below the normal range (|w| < 2^-14) representable values are 2^-24 apart whatever the
        # magnitude, so a result there cannot be held to a relative bound; those elements are reported apart,
        # as an absolute error in units of that spacing
        normal_min = 2.0 ** -14 if spec.dtype == 1 else 0.0
        for j in range(len(p["rows"])):
            r = keys[tt == j] - Rs[j]
            D, H = int(p["dims"][j]), int(p["rows"][j])
            w_old = p["w"][Ws[j]:Ws[j + 1]].reshape(H, D)[r].astype(np.float64)
            w_ref = w1[Ws[j]:Ws[j + 1]].reshape(H, D)[r].astype(np.float64)
            w_gpu = gpu_step0["w"][Ws[j]:Ws[j + 1]].reshape(H, D)[r].astype(np.float64)
            ew = np.abs(w_gpu - w_ref) / (np.abs(w_old) + np.abs(w_ref - w_old) + 1e-300)
            normal = np.abs(w_ref) >= normal_min
            e_w.append(ew[normal])
            sub_abs.append(np.abs(w_gpu - w_ref)[~normal] / 2.0 ** -24)
            m_ref = m1[Rs[j]:Rs[j + 1]][r].astype(np.float64)
            e_m.append(np.abs(gpu_step0["m"][Rs[j]:Rs[j + 1]][r].astype(np.float64) - m_ref) / (m_ref + 1e-300))
        untouched = np.ones(int(Rs[-1]), bool)
        untouched[keys] = False
        same_m = bool(np.array_equal(gpu_step0["m"][untouched], p["m"][untouched]))
        res["parity_step0"] = {
            "forward_rel_err_vs_sum_abs_terms": _err_stats(e_f),
            "weights_rel_err_vs_abs_w_plus_abs_step": _err_stats(np.concatenate(e_w) if e_w else []),
            "weights_below_fp16_normal_range_abs_err_in_2^-24": _err_stats(np.concatenate(sub_abs) if sub_abs else []),
            "moments_rel_err": _err_stats(np.concatenate(e_m) if e_m else []),
            "sorted_keys_payloads_bit_exact": bool(np.array_equal(gpu_step0["sorted_keys"], art.sorted_keys)
                                                   and np.array_equal(gpu_step0["sorted_vals"], art.sorted_vals)),
            "untouched_moments_bit_identical": same_m,
            "tolerance": {"fp32_tables": 1e-5, "fp16_tables": 2e-3},
        }

    # ---- one oracle thread per usable core, each on its own tables
    if all_core_jobs:
        def job(q):
            a = time.perf_counter()
            orc.forward(q["rows"], q["dims"], spec.dtype, q["w"], q["indices"], q["offsets"], B)
            orc.backward_rowwise_adagrad(q["rows"], q["dims"], spec.dtype, q["w"], q["m"], q["indices"], q["offsets"],
                                         B, q["g"], spec.lr, spec.eps)
            return time.perf_counter() - a
        ta = time.perf_counter()
        with ThreadPoolExecutor(max_workers=len(all_core_jobs)) as ex:
            per = list(ex.map(job, all_core_jobs))
        wall = time.perf_counter() - ta
        tot = sum(int(q["offsets"][-1]) for q in all_core_jobs)
        res["all_cores"] = {
            "value": tot / wall, "unit": "lookups/s", "cores": len(all_core_jobs), "kind": "oracle",
            "sample": f"{len(all_core_jobs)} concurrent single-threaded oracle runs on disjoint tables of the first "
                      f"batch, {tot} lookups in {wall:.2f}s wall (slowest thread {max(per):.2f}s)",
        }
    return res


def bench_inputs(args, spec, dev):
    """Section 7.1 / Section 4 input-side kernels on one batch of `spec`: bucketize over W shards, permute of
    the bucketized (W,T,B) result to (T,W,B), and lengths -> offsets of its W*T*B lengths."""
    import torch

    from paper_2104_05158_amd import tbe
    from paper_2104_05158_amd import workloads as wl

    W, T, B = args.shards, spec.T, spec.batch
    b = wl.make_batch(spec, dev, it=0)
    N, n_in, n_out = b.num_indices, T * B, W * T * B
    rows = torch.from_numpy(spec.rows).to(dev)
    scratch = torch.empty(tbe.tbe_inputs_scratch_bytes(n_out), dtype=torch.uint8, device=dev)
    i32 = lambda n: torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    i64 = lambda n: torch.empty(n, dtype=torch.int64, device=dev)
    len_b, off_b, idx_b = i32(n_out), i64(n_out + 1), i32(N)
    len_p, off_p, idx_p = i32(n_out), i64(n_out + 1), i32(N)
    off_l = i64(n_out + 1)
    calls = {
        "bucketize_rowwise": (lambda: tbe.tbe_bucketize_rowwise(T, B, W, rows, b.indices, b.offsets, N, len_b, off_b,
                                                                idx_b, scratch),
                              8.0 * N + 8.0 * n_in + 12.0 * n_out),
        "permute_wtb_to_twb": (lambda: tbe.tbe_permute_wtb_to_twb(W, T, B, len_b, idx_b, N, len_p, off_p, idx_p,
                                                                  scratch),
                               8.0 * N + 16.0 * n_out),
        "lengths_to_offsets": (lambda: tbe.tbe_lengths_to_offsets(len_p, n_out, off_l, scratch), 12.0 * n_out),
    }
    res = {}
    for name, (fn, nbytes) in calls.items():
        for _ in range(args.warmup):
            assert fn() == tbe.TBE_OK
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            assert fn() == tbe.TBE_OK
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        res[name] = {"ms": round(ms, 5), "algorithmic_bytes": nbytes,
                     "algorithmic_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    assert torch.equal(off_l, off_p)
    print(json.dumps({"metric": "input_side_kernels", "unit": "ms", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "dtype": "int32", "data": "synthetic",
                      "config": {"workload": spec.name + "_inputs", "tables": T, "batch": B, "shards": W,
                                 "lookups": N, "bags_in": n_in, "bags_out": n_out},
                      "kernels": res}))


def stream_rates(dev):
    """What plain streaming kernels reach on this machine over 1 GiB of float32: torch's device copy (read + write),
    its read-only reduction and its write-only fill, and the library's read probe.  Second denominators beside
    the published peak."""
    import torch

    n = 1 << 28
    src = torch.empty(n, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)

    def rate(fn, nbytes, reps=10):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return round(nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

    r = {"copy_GBps": rate(lambda: dst.copy_(src), 8.0 * n),
         "read_only_GBps": rate(lambda: src.sum(), 4.0 * n),
         "write_only_GBps": rate(lambda: dst.fill_(2.0), 4.0 * n)}
    # the library's own read probe (coalesced 16-byte loads, nothing else): over the 1 GiB buffer (HBM) and over
    # its first 128 MiB read 8 times per launch (resident in the memory-side cache after the first pass)
    from paper_2104_05158_amd import tbe as _tbe
    sink = torch.zeros(1, dtype=torch.int32, device=dev)

    def probe(nbytes, passes):
        st = _tbe.tbe_probe_read(src, nbytes, passes, sink)
        if st != 0:
            raise RuntimeError(f"tbe_probe_read: status {st}")

    r["read_probe_GBps"] = rate(lambda: probe(4 * n, 4), 16.0 * n, reps=4)
    r["read_probe_cache_resident_GBps"] = rate(lambda: probe(128 << 20, 8), 8.0 * (128 << 20))
    del src, dst
    return r


def read_traffic(workload):
    """Measured L2<->fabric bytes per launch, stored by an earlier rocprofv3 --pmc run of this command
    (profiles/hbm_traffic.txt: workload, kernel, bytes per launch, launches per step)."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    per_kernel, step_total = {}, 0.0
    if not os.path.exists(path):
        return per_kernel, None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == workload and not line.startswith("#"):
            launches = float(f[3]) if len(f) >= 4 else 1.0
            per_kernel.setdefault(f[1], []).append((float(f[2]), launches))
            step_total += float(f[2]) * launches
    return per_kernel, (step_total if per_kernel else None)


def run_workload(args, spec, dev, headline):
    """Generates the workload, runs warm-up + timed steps + a profiled pass, returns the result dict."""
    import torch

    from paper_2104_05158_amd import tbe
    from paper_2104_05158_amd import workloads as wl

    t_setup = time.perf_counter()
    weights = wl.make_weights(spec, dev)
    batches = [wl.make_batch(spec, dev, it=i) for i in range(max(1, args.rotation))]
    opt_id = {"rowwise_adagrad": tbe.TBE_OPT_ROWWISE_ADAGRAD, "adagrad": tbe.TBE_OPT_ADAGRAD,
              "adam": tbe.TBE_OPT_ADAM}[args.optimizer]
    dt_id = {"fp32": tbe.TBE_DTYPE_FP32, "fp16": tbe.TBE_DTYPE_FP16, "bf16": tbe.TBE_DTYPE_BF16}
    nmax = max(b.num_indices for b in batches)
    table_major = args.layout == "table"
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, spec.dtype, spec.batch, nmax, device=dev,
                                       weights=weights, optimizer=opt_id, output_dtype=dt_id[args.out_dtype],
                                       grad_dtype=dt_id[args.grad_dtype],
                                       layout=tbe.TBE_LAYOUT_TABLE_MAJOR if table_major else 0)
    grad = wl.make_grad(spec, dev)
    if args.grad_dtype != "fp32":
        grad = grad.to(op.grad_torch_dtype)
    woffs, cols, R = table_slices(spec)
    if table_major:
        grad_arg = torch.cat([grad[:, int(cols[t]):int(cols[t + 1])].reshape(-1) for t in range(spec.T)])
    else:
        grad_arg = grad
    out = torch.empty(spec.batch, spec.sumD, dtype=op.out_torch_dtype, device=dev)

    def backward(b):
        if opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD:
            op.backward_rowwise_adagrad(b.indices, b.offsets, spec.batch, grad_arg, spec.lr, spec.eps,
                                        num_indices=b.num_indices)
        elif opt_id == tbe.TBE_OPT_ADAGRAD:
            op.backward_adagrad(b.indices, b.offsets, spec.batch, grad_arg, spec.lr, spec.eps, num_indices=b.num_indices)
        else:
            op.backward_adam(b.indices, b.offsets, spec.batch, grad_arg, spec.lr, 0.9, 0.999, spec.eps, 1,
                             num_indices=b.num_indices)

    flush_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if args.flush else None
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    overlap = args.overlap and not args.fwd_only
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream() if overlap else None

    def step(i):
        b = batches[i % len(batches)]
        if flush_buf is not None:
            flush_buf.fill_(i & 0xFF)
        if overlap:
            # a2-a4 (keys, sort, run-length) depend only on the indices: they run beside the forward
            side_stream.wait_stream(main_stream)
            op.backward_sort(b.indices, b.offsets, spec.batch, stream=side_stream, num_indices=b.num_indices)
            op.forward(b.indices, b.offsets, spec.batch, out=out, num_indices=b.num_indices)
            main_stream.wait_stream(side_stream)
            op.backward_update_rowwise_adagrad(grad_arg, spec.lr, spec.eps)
            return
        op.forward(b.indices, b.offsets, spec.batch, out=out, num_indices=b.num_indices)
        if not args.fwd_only:
            backward(b)

    # ---- the first step from fresh state, with everything the oracle comparison needs kept on the host
    want_cpu = (headline and not args.no_cpu_baseline and opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD
                and not args.fwd_only)
    sample = gpu_step0 = None
    all_core_jobs = []
    if want_cpu:
        b0 = batches[0]
        n_t0 = per_table_counts(spec, b0)
        take = pick_sample_tables(spec, n_t0, args.cpu_sample_lookups)
        g32 = lambda t: grad[:, int(cols[t]):int(cols[t + 1])].float().cpu().numpy()
        sample = sub_problem(spec, b0, take, weights, op.state, g32)
        sample["take"] = take
        step(0)
        torch.cuda.synchronize()
        art = op.artifacts()
        B = spec.batch
        sk, sv = [], []
        base = 0
        for t in take:
            lo, hi = int(b0.offsets[t * B]), int(b0.offsets[(t + 1) * B])
            # the oracle numbers the sampled tables' rows from 0: shift each table's keys accordingly
            k = (art["sorted_keys"][lo:hi].to(torch.int64) & 0xFFFFFFFF) - int(R[t]) + base
            sk.append(k.cpu().numpy().astype(np.uint32))
            sv.append(art["sorted_vals"][lo:hi].cpu().numpy())
            base += int(spec.rows[t])
        if table_major:
            o = [out.view(-1)[B * int(cols[t]):B * int(cols[t + 1])].view(B, -1) for t in take]
        else:
            o = [out[:, int(cols[t]):int(cols[t + 1])] for t in take]
        gpu_step0 = dict(out=torch.cat(o, dim=1).float().cpu().numpy(),
                         w=np.concatenate([weights[int(woffs[t]):int(woffs[t + 1])].cpu().numpy() for t in take]),
                         m=np.concatenate([op.state[int(R[t]):int(R[t + 1])].cpu().numpy() for t in take]),
                         sorted_keys=np.concatenate(sk), sorted_vals=np.concatenate(sv))
        # disjoint table groups for the all-core run (timing only: whatever state the tables are in)
        cores = host_info()["usable_cores"]
        nxt = take[-1] + 1
        for _ in range(cores):
            grp = pick_sample_tables(spec, n_t0, args.cpu_sample_lookups / 4, byte_cap=2e9, start=nxt % spec.T)
            if not grp:
                break
            all_core_jobs.append(sub_problem(spec, b0, grp, weights, op.state, g32))
            nxt = grp[-1] + 1
        del art

    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        a.normal_()
        c = torch.empty_like(a)
        c.copy_(a)
        torch.cuda.synchronize()
        del a, c

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    lookups = sum(batches[(args.warmup + i) % len(batches)].num_indices for i in range(args.steps))
    if args.graph:
        # one captured step per batch of the rotation; the library only enqueues kernels, so capture is legal
        assert not overlap and flush_buf is None, "--graph is timed without --overlap / --flush"
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graphs = []
        for j in range(len(batches)):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=cap):
                step(j)
            graphs.append(gph)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % len(graphs)].replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        # the timed region: EXACTLY `steps` steps, profiling off, synchronised on both sides
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    # per-kernel durations: the same steps once more with the library's HIP events on the launch stream
    op.profile_enable(args.steps + 1)
    torch.cuda.synchronize()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    prof = op.profile_read()
    op.profile_enable(0)

    # workload statistics of the last batch used (for the byte model)
    last = batches[(args.warmup + args.steps - 1) % len(batches)]
    n_t = per_table_counts(spec, last).astype(np.float64)
    nlong_t = np.zeros(spec.T)
    ulong_t = np.zeros(spec.T)
    ndense_t = np.zeros(spec.T)
    udense_t = np.zeros(spec.T)
    long_rows_t = None
    longest_run = 0
    if args.fwd_only:
        u_t = np.zeros(spec.T)
        num_unique = 0
    else:
        art = op.artifacts()
        num_unique = art["num_unique"]
        Rt = torch.tensor(R, device=dev)
        uk = art["unique_keys"].to(torch.int64) & 0xFFFFFFFF
        tab = torch.searchsorted(Rt, uk, right=True) - 1
        u_t = torch.bincount(tab, minlength=spec.T).cpu().numpy().astype(np.float64)
        lens = torch.diff(art["seg_offsets"].to(torch.int64))
        longest_run = int(lens.max().item()) if lens.numel() else 0
        thr = dense_threshold(spec.batch)
        is_dense = lens > (thr if last.num_indices > thr else (1 << 62))
        is_long = (lens > LONG_RUN) & ~is_dense
        nlong_t = torch.bincount(tab[is_long], weights=lens[is_long].double(), minlength=spec.T).cpu().numpy()
        ulong_t = torch.bincount(tab[is_long], minlength=spec.T).cpu().numpy().astype(np.float64)
        # partial rows of a long run: one per window piece; a run with fewer slots than windows (two per fully
        # covered 128-position chunk) merges windows in twos or fours
        nwin_t = torch.tensor([window_count(spec.batch, int(d), grad.element_size()) for d in spec.dims], device=dev)
        seg = art["seg_offsets"].to(torch.int64)
        slots = 2 * ((seg[1:] - 1) // 128 - seg[:-1] // 128 - 1)
        nw = nwin_t[tab]
        step = torch.ones_like(nw)
        for _ in range(4):
            step = torch.where(-(-nw // step) > slots, step * 2, step)
        pieces = -(-nw // step)
        long_rows_t = torch.bincount(tab[is_long], weights=pieces[is_long].double(), minlength=spec.T).cpu().numpy()
        del seg, slots, nw, pieces, step
        ndense_t = torch.bincount(tab[is_dense], weights=lens[is_dense].double(), minlength=spec.T).cpu().numpy()
        udense_t = torch.bincount(tab[is_dense], minlength=spec.T).cpu().numpy().astype(np.float64)
        del art, uk, tab, lens, is_long, is_dense
    comp, logical = kernel_bytes(spec, n_t, u_t, nlong_t, ulong_t, so=out.element_size(), sg=grad.element_size(),
                                 state_per_elem={0: 0, 1: 1, 2: 2}[opt_id], passes_t=sort_passes(spec.rows),
                                 ndense_t=ndense_t, udense_t=udense_t, long_rows_t=long_rows_t)

    kernels = {}
    for name, (launches, ms) in prof.items():
        if launches:
            per = ms / launches
            gbps = lambda d: round(d.get(name, 0.0) / (per * 1e-3) / 1e9, 1) if per > 0 else None
            kernels[name] = {"launches_per_step": launches / args.steps, "ms_per_launch": round(per, 5),
                             "ms_per_step": round(ms / args.steps, 5), "compulsory_GBps": gbps(comp),
                             "logical_GBps": gbps(logical)}
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    dom_ms = kernels[dominant]["ms_per_launch"]
    achieved = comp[dominant] / (dom_ms * 1e-3) / 1e9
    # achieved = compulsory algorithmic bytes of that kernel / its mean duration (HIP events on the launch stream)
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                "algorithmic_bytes_per_launch": comp[dominant], "ms_per_launch": dom_ms,
                "logical_bytes_per_launch": logical[dominant],
                "logical_GBps": round(logical[dominant] / (dom_ms * 1e-3) / 1e9, 1)}
    # The counters were collected for the default variant only (fp32 output and gradient, [B, sumD] rows,
    # row-wise AdaGrad, forward + backward).  They are STORED values of an earlier rocprofv3 --pmc run of this
    # same command, not measured in this run, and they count bytes at the L2 <-> fabric boundary: reads that the
    # memory-side Infinity Cache serves are included, so this is an upper bound of the HBM traffic.
    default_variant = (args.out_dtype == "fp32" and args.grad_dtype == "fp32" and args.layout == "batch"
                       and opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD and not args.fwd_only)
    step_traffic = None
    if default_variant:
        per_kernel, step_traffic = read_traffic(spec.name)
        ent = per_kernel.get(dominant + "_kernel")
        if ent:
            tb = sum(b * l for b, l in ent) / sum(l for _, l in ent)
            roofline["traffic"] = tb
            roofline["traffic_GBps"] = round(tb / (dom_ms * 1e-3) / 1e9, 1)
            roofline["traffic_over_algorithmic"] = round(tb / comp[dominant], 2)
            roofline["traffic_source"] = (TRAFFIC_FILE + ": stored rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE of an earlier "
                                          "run of this command; L2<->fabric bytes incl. Infinity-Cache hits, not HBM-only")

    ms_per_step = elapsed / args.steps * 1e3
    fwd_ms = kernels.get("forward", {}).get("ms_per_step", 0.0)
    bwd_ms = sum(v["ms_per_step"] for k, v in kernels.items() if k != "forward")
    result = {
        "metric": (f"tbe_fwd_bwd_{args.optimizer}_lookups_per_s") if not args.fwd_only else "tbe_fwd_lookups_per_s",
        "value": lookups / elapsed,
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": spec.name,
            "tables": spec.T,
            "batch": spec.batch,
            "storage": "fp32" if spec.dtype == 0 else "fp16",
            "optimizer": args.optimizer,
            "output_dtype": args.out_dtype,
            "grad_dtype": args.grad_dtype,
            "layout": args.layout,
            "lookups_per_step": lookups / args.steps,
            "unique_rows_last_step": num_unique,
            "longest_duplicate_run_last_step": longest_run,
            "dense_runs_last_step": int(udense_t.sum()),
            "lookups_in_dense_runs_last_step": int(ndense_t.sum()),
            "table_bytes": spec.weight_bytes,
            "workspace_bytes": int(op.sizes["workspace_bytes"]),
            "index_dist": spec.index_dist if spec.index_dist == "uniform" else f"zipf({spec.zipf_s})",
            "rotation": len(batches),
            "cache_flush": bool(args.flush),
            "streams": 2 if overlap else 1,
            "hip_graph": bool(args.graph),
            "profiling_during_timed_steps": False,
        },
        "roofline": roofline,
        "kernels": kernels,
        "fwd_ms": fwd_ms,
        "bwd_ms": round(bwd_ms, 5),
        "step_compulsory_GBps": round(sum(comp[k] * kernels[k]["launches_per_step"] for k in kernels if k in comp)
                                      / (ms_per_step * 1e-3) / 1e9, 1) if not args.fwd_only else None,
        # all kernels of a step, each weighted by its launches per step: stored L2<->fabric bytes over the step's wall time
        "step_traffic_GBps": round(step_traffic / (ms_per_step * 1e-3) / 1e9, 1) if step_traffic else None,
        "setup_s": round(setup_s, 2),
    }
    if want_cpu:
        result["cpu_baseline"] = cpu_baseline(spec, sample, gpu_step0, all_core_jobs)
    else:
        result["cpu_baseline"] = None
    op.close()
    del op, weights, batches, grad, grad_arg, out, flush_buf
    gc.collect()
    torch.cuda.empty_cache()
    return result


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (the operator runs on one GPU's share of the tables; "
              "no collectives are part of it). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2104_05158_amd import tbe
    from paper_2104_05158_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tbe.lib()  # fail loudly if the HIP library is missing

    others = []
    if args.paper_membench:
        spec = wl.paper_memory_benchmark(0 if args.paper_membench == "fp32" else 1, args.batch or 4096)
    else:
        k = 4 if args.config is None else args.config
        spec = wl.config(k)
        if args.others is not None:
            others = [int(x) for x in args.others.split(",") if x.strip()]
        elif args.config is None and not (args.batch or args.zipf is not None or args.inputs):
            others = [3, 2]
        if args.batch:
            spec.batch = args.batch
            spec.name += f"-B{args.batch}"
        if args.zipf is not None:
            # sensitivity runs: the same tables with another index distribution (0 = uniform)
            spec.index_dist = "zipf" if args.zipf > 0 else "uniform"
            spec.zipf_s = args.zipf
            spec.name += f"-zipf{args.zipf:g}" if args.zipf > 0 else "-uniform"
    if args.inputs:
        bench_inputs(args, spec, dev)
        return
    rates = stream_rates(dev) if args.steps >= 5 else {}
    result = run_workload(args, spec, dev, headline=True)
    if rates:
        result["roofline"].update(rates)
        result["roofline"]["frac_of_copy"] = round(result["roofline"]["achieved"] / rates["copy_GBps"], 4)
        if result["roofline"].get("traffic_GBps"):
            # the dominant kernel's L2<->fabric rate against what plain coalesced reads reach on this machine
            result["roofline"]["traffic_rate_over_read_probe"] = round(
                result["roofline"]["traffic_GBps"] / rates["read_probe_GBps"], 4)
    extra = []
    for k in others:
        r = run_workload(args, wl.config(k), dev, headline=False)
        extra.append({"workload": r["config"]["workload"], "value": r["value"], "unit": r["unit"],
                      "ms_per_step": r["ms_per_step"], "lookups_per_step": r["config"]["lookups_per_step"],
                      "unique_rows_last_step": r["config"]["unique_rows_last_step"],
                      "longest_duplicate_run_last_step": r["config"]["longest_duplicate_run_last_step"],
                      "roofline": r["roofline"], "kernels": r["kernels"], "fwd_ms": r["fwd_ms"], "bwd_ms": r["bwd_ms"],
                      "step_compulsory_GBps": r["step_compulsory_GBps"], "step_traffic_GBps": r["step_traffic_GBps"]})
    if extra:
        result["other_configs"] = extra
    print(json.dumps(result))


if __name__ == "__main__":
    main()
