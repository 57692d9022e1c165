#!/usr/bin/env python3
"""Benchmark of the table-batched embedding-bag hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: tbe_forward, then
tbe_backward_rowwise_adagrad (sort plan, radix sort, run-length, fused reduce + row-wise AdaGrad,
long-run fix-up) on the same batch.  Inputs, weights and optimizer state are resident in HBM before
the timed region; a rotation of pre-generated batches (different seeds) is used so that no step
re-reads the previous step's index stream.

Prints ONE JSON line: lookups/s of fwd+bwd (whole job = this one GPU), plus
  roofline      -- the dominant kernel's algorithmic (compulsory: each distinct byte once) bytes per launch /
                   its mean launch duration, measured with HIP events recorded by the library on the launch
                   stream; the every-lookup-counted ("logical") rate is given beside it
  cpu_baseline  -- the CPU oracle, as it stands, timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..4 (default 2)")
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
                    help="capture each batch's step in a HIP graph and time the replays (the per-kernel figures "
                         "then come from the same number of eager steps run afterwards)")
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
    return ap.parse_args()


def per_table_counts(spec, batch):
    off = batch.offsets
    B = spec.batch
    bounds = off[:: B][: spec.T + 1] if B > 0 else off
    return np.diff(bounds.cpu().numpy())


LONG_RUN = 512    # runs longer than this are cut at 128-position chunk borders by the library (kLongRun)


def kernel_bytes(spec, n_t, u_t, nlong_t, ulong_t, so=4, sg=4, state_per_elem=0):
    """Bytes one launch of each kernel must move, two ways.
    compulsory: every distinct byte once -- what an ideal cache would leave for HBM; the roofline numerator.
    logical:    every lookup counted as a row read -- a throughput figure that caches can push past the HBM peak.
    n_t / u_t: lookups / distinct rows per table; nlong_t / ulong_t: lookups in / number of runs longer than LONG_RUN;
    so / sg: bytes per output / gradient element; state_per_elem: float32 optimizer states per weight element
    (0 = one moment per row)."""
    sw = 4 if spec.dtype == 0 else 2
    D = spec.dims.astype(np.float64)
    B = float(spec.batch)
    N = float(n_t.sum())
    U = float(u_t.sum())
    bags = float(spec.T) * B
    io_fwd = N * 4 + bags * 8 + (B * so * D).sum()
    state_rw = 8 * D * state_per_elem if state_per_elem else 8.0
    rmw = (u_t * (2 * D * sw + state_rw)).sum()
    slab = B * sg * D
    partial_rows = nlong_t / 128.0 + 2 * ulong_t    # one fp32 partial row per chunk a long run touches
    comp = {
        "forward": float((u_t * D * sw).sum() + io_fwd),
        "sort_plan": 0.0,
        "radix_hist": N * 4,
        "radix_scatter": N * 16,
        "radix_scan": 0.0,
        "runlength": N * 4 + U * 8,
        "reduce_update": float(N * 4 + U * 8 + np.minimum(n_t * sg * D, slab).sum() + rmw +
                               (partial_rows * 4 * D).sum()),
        "long_fixup": float((partial_rows * 4 * D + ulong_t * (2 * D * sw + state_rw)).sum()),
    }
    logical = dict(comp)
    logical["forward"] = float((n_t * D * sw).sum() + io_fwd)
    logical["reduce_update"] = float(N * 4 + U * 8 + (n_t * sg * D).sum() + rmw + (partial_rows * 4 * D).sum())
    return comp, logical


def cpu_baseline(spec, batch, weights, grad, target_lookups):
    """Times the CPU oracle (single thread, as it stands) on the first tables of the workload whose
    lookups add up to about `target_lookups`; exact for those tables because tables are independent."""
    import torch

    from oracle import tbe_oracle as orc

    B = spec.batch
    n_t = per_table_counts(spec, batch)
    order = np.arange(spec.T)
    take, tot, wbytes = [], 0, 0
    for t in order:
        tb = int(spec.rows[t]) * int(spec.dims[t]) * (4 if spec.dtype == 0 else 2)
        if take and (tot + n_t[t] > 1.5 * target_lookups or wbytes + tb > 24e9):
            continue
        take.append(int(t))
        tot += int(n_t[t])
        wbytes += tb
        if tot >= target_lookups:
            break
    take.sort()
    woffs = np.concatenate([[0], np.cumsum(spec.rows * spec.dims.astype(np.int64))])
    cols = np.concatenate([[0], np.cumsum(spec.dims)])
    off = batch.offsets
    idx_parts, len_parts, w_parts, g_parts = [], [], [], []
    for t in take:
        lo, hi = int(off[t * B]), int(off[(t + 1) * B])
        idx_parts.append(batch.indices[lo:hi].cpu().numpy())
        len_parts.append(np.diff(off[t * B:(t + 1) * B + 1].cpu().numpy()))
        w_parts.append(weights[int(woffs[t]):int(woffs[t + 1])].cpu().numpy())
        g_parts.append(grad[:, int(cols[t]):int(cols[t + 1])].float().cpu().numpy())
    rows = spec.rows[take]
    dims = spec.dims[take]
    indices = np.concatenate(idx_parts).astype(np.int32)
    offsets = np.zeros(len(take) * B + 1, np.int64)
    offsets[1:] = np.cumsum(np.concatenate(len_parts))
    w = np.concatenate(w_parts)
    g = np.ascontiguousarray(np.concatenate(g_parts, axis=1))
    m = np.zeros(int(rows.sum()), np.float32)
    orc.build()
    t0 = time.perf_counter()
    orc.forward(rows, dims, spec.dtype, w, indices, offsets, B)
    t1 = time.perf_counter()
    orc.backward_rowwise_adagrad(rows, dims, spec.dtype, w, m, indices, offsets, B, g, spec.lr, spec.eps)
    t2 = time.perf_counter()
    n = int(offsets[-1])
    return {
        "value": n / (t2 - t0),
        "unit": "lookups/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"tables {take[0]}..{take[-1]} ({len(take)} of {spec.T}) of the same batch, {n} lookups, "
                  f"fwd {t1 - t0:.2f}s + bwd {t2 - t1:.2f}s; plain C -O2, fp64 accumulation",
        "fwd_s": t1 - t0,
        "bwd_s": t2 - t1,
        "lookups": n,
    }


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

    if args.paper_membench:
        spec = wl.paper_memory_benchmark(0 if args.paper_membench == "fp32" else 1, args.batch or 4096)
    else:
        spec = wl.config(args.config)
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
    t_setup = time.perf_counter()
    weights = wl.make_weights(spec, dev)
    batches = [wl.make_batch(spec, dev, it=i) for i in range(max(1, args.rotation))]
    opt_id = {"rowwise_adagrad": tbe.TBE_OPT_ROWWISE_ADAGRAD, "adagrad": tbe.TBE_OPT_ADAGRAD,
              "adam": tbe.TBE_OPT_ADAM}[args.optimizer]
    dt_id = {"fp32": tbe.TBE_DTYPE_FP32, "fp16": tbe.TBE_DTYPE_FP16, "bf16": tbe.TBE_DTYPE_BF16}
    nmax = max(b.num_indices for b in batches)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, spec.dtype, spec.batch, nmax, device=dev,
                                       weights=weights, optimizer=opt_id, output_dtype=dt_id[args.out_dtype],
                                       grad_dtype=dt_id[args.grad_dtype],
                                       layout=tbe.TBE_LAYOUT_TABLE_MAJOR if args.layout == "table" else 0)
    grad = wl.make_grad(spec, dev)
    if args.grad_dtype != "fp32":
        grad = grad.to(op.grad_torch_dtype)
    out = torch.empty(spec.batch, spec.sumD, dtype=op.out_torch_dtype, device=dev)

    def backward(b):
        if opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD:
            op.backward_rowwise_adagrad(b.indices, b.offsets, spec.batch, grad, spec.lr, spec.eps,
                                        num_indices=b.num_indices)
        elif opt_id == tbe.TBE_OPT_ADAGRAD:
            op.backward_adagrad(b.indices, b.offsets, spec.batch, grad, spec.lr, spec.eps, num_indices=b.num_indices)
        else:
            op.backward_adam(b.indices, b.offsets, spec.batch, grad, spec.lr, 0.9, 0.999, spec.eps, 1,
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
            op.backward_update_rowwise_adagrad(grad, spec.lr, spec.eps)
            return
        op.forward(b.indices, b.offsets, spec.batch, out=out, num_indices=b.num_indices)
        if not args.fwd_only:
            backward(b)

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
        op.profile_enable(args.steps + 1)
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
    else:
        op.profile_enable(args.steps + 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    prof = op.profile_read()
    op.profile_enable(0)

    # workload statistics of the last batch used (for the byte model)
    last = batches[(args.warmup + args.steps - 1) % len(batches)]
    n_t = per_table_counts(spec, last).astype(np.float64)
    nlong_t = np.zeros(spec.T)
    ulong_t = np.zeros(spec.T)
    if args.fwd_only:
        u_t = np.zeros(spec.T)
        num_unique = 0
    else:
        art = op.artifacts()
        num_unique = art["num_unique"]
        R = torch.tensor(np.concatenate([[0], np.cumsum(spec.rows)]), device=dev)
        uk = art["unique_keys"].to(torch.int64) & 0xFFFFFFFF
        tab = torch.searchsorted(R, uk, right=True) - 1
        u_t = torch.bincount(tab, minlength=spec.T).cpu().numpy().astype(np.float64)
        lens = torch.diff(art["seg_offsets"].to(torch.int64))
        is_long = lens > LONG_RUN
        nlong_t = torch.bincount(tab[is_long], weights=lens[is_long].double(), minlength=spec.T).cpu().numpy()
        ulong_t = torch.bincount(tab[is_long], minlength=spec.T).cpu().numpy().astype(np.float64)
    comp, logical = kernel_bytes(spec, n_t, u_t, nlong_t, ulong_t, so=out.element_size(), sg=grad.element_size(),
                                 state_per_elem={0: 0, 1: 1, 2: 2}[opt_id])

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
    # measured L2<->fabric bytes per launch of that kernel (two rocprofv3 --pmc runs, summarised in profiles/)
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    step_traffic = None
    if os.path.exists(traffic_file):
        for line in open(traffic_file):
            f = line.split()
            if len(f) == 3 and f[0] == spec.name:
                step_traffic = (step_traffic or 0.0) + float(f[2])
                if f[1] == dominant + "_kernel":
                    roofline["traffic"] = float(f[2])
                    roofline["traffic_GBps"] = round(float(f[2]) / (dom_ms * 1e-3) / 1e9, 1)
    # the counters were collected for the default variant only (fp32 output and gradient, [B, sumD] rows,
    # row-wise AdaGrad, forward + backward)
    default_variant = (args.out_dtype == "fp32" and args.grad_dtype == "fp32" and args.layout == "batch"
                       and opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD and not args.fwd_only)
    if not default_variant:
        roofline["traffic"] = None
        roofline.pop("traffic_GBps", None)
        step_traffic = None

    # what a plain device-to-device copy reaches on this machine, as a second denominator beside the published peak
    if args.steps >= 5:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(2):
            dst.copy_(src)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        roofline["copy_GBps"] = round(2 * src.numel() * 4 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        roofline["frac_of_copy"] = round(achieved / roofline["copy_GBps"], 4)
        del src, dst

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
            "table_bytes": spec.weight_bytes,
            "index_dist": spec.index_dist if spec.index_dist == "uniform" else f"zipf({spec.zipf_s})",
            "rotation": len(batches),
            "cache_flush": bool(args.flush),
            "streams": 2 if overlap else 1,
            "hip_graph": bool(args.graph),
        },
        "roofline": roofline,
        "kernels": kernels,
        "fwd_ms": fwd_ms,
        "bwd_ms": round(bwd_ms, 5),
        "step_compulsory_GBps": round(sum(comp.values()) / (ms_per_step * 1e-3) / 1e9, 1) if not args.fwd_only else None,
        # all kernels of a step: measured L2<->fabric bytes (profiles/hbm_traffic.txt) over the step's wall time
        "step_traffic_GBps": round(step_traffic / (ms_per_step * 1e-3) / 1e9, 1) if step_traffic else None,
        "setup_s": round(setup_s, 2),
    }
    if not args.no_cpu_baseline and opt_id == tbe.TBE_OPT_ROWWISE_ADAGRAD:
        result["cpu_baseline"] = cpu_baseline(spec, last, weights, grad, args.cpu_sample_lookups)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
