"""GPU parity at the full benchmark sizes (configs 1-4), in the launch configuration bench.py times.

The tables do not fit in host memory, so the oracle is applied to sampled outputs, each computed
exactly on a reduced problem (tables are independent, and a row's update depends only on the
lookups that hit that row):
  forward   sampled bags of sampled tables (incl. the longest bag and an empty one)
  backward  sampled rows of sampled tables (incl. the hottest row = the longest duplicate run,
            runs near the split threshold, random touched rows) + every untouched row bit-identical,
            proven by regenerating the seeded initial weights chunk by chunk
  integers  whole-array exact comparison with the oracle's sort where it finishes in seconds
            (configs 1, 2); for configs 3, 4 exact comparison on sampled tables (the sorted array
            is table-major, so a table's slice is its own sort) plus whole-array properties:
            keys non-decreasing, payloads non-decreasing inside a run, run lengths equal to the
            key histogram, segment offsets strictly increasing and ending at N.
"""
import gc

import numpy as np
import pytest
import torch

from oracle import tbe_oracle as orc
from paper_2104_05158_amd import tbe
from paper_2104_05158_amd import workloads as wl

import tbe_testlib as tl

pytestmark = pytest.mark.gpu


def _regen_chunks(spec, device, chunk_elems=1 << 28):
    """Yields (lo, hi, initial weights chunk) exactly as workloads.make_weights produced them."""
    g = torch.Generator(device=device)
    g.manual_seed(wl.BASE_SEED + 17)
    n = spec.weight_elems
    dt = torch.float32 if spec.dtype == 0 else torch.float16
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        r = torch.rand(hi - lo, generator=g, device=device, dtype=torch.float32)
        yield lo, hi, (r * 0.02 - 0.01).to(dt)


def _sample_tables(spec, rng, extra=3):
    T = spec.T
    sizes = spec.rows * spec.dims
    pick = {int(np.argmin(sizes)), int(np.argmax(sizes)), int(np.argmax(spec.pooling_mean)), T - 1}
    for d in np.unique(spec.dims):
        pick.add(int(np.flatnonzero(spec.dims == d)[0]))
    while len(pick) < min(T, 4 + extra + len(np.unique(spec.dims))):
        pick.add(int(rng.integers(0, T)))
    return sorted(pick)


@pytest.mark.parametrize("k,variant", [(1, "fp32"), (2, "fp32"), (3, "fp32"), (4, "fp32"), (2, "16bit"), (4, "16bit"),
                                       (2, "table"), (3, "table"), (2, "all3"), (4, "all3")])
def test_full_size_config(gpu_device, k, variant):
    """variant "16bit": float16 pooled output and bfloat16 upstream gradient (the oracle is fed the float32
    values of exactly those bfloat16 numbers; the output tolerance gains one fp16 rounding).
    variant "table": output and gradient in the table-major layout (one [B, D_t] block per table).
    variant "all3": both together, the types and layout of a table-wise all-to-all."""
    _full_size_check(gpu_device, wl.config(k), variant, k, 1000 + k)


@pytest.mark.parametrize("dtype,batch", [(0, 8192), (1, 8192), (1, 32768)])
def test_paper_memory_benchmark_shape(gpu_device, dtype, batch):
    """The shape of the paper's own memory benchmark (Appendix A): 64 tables x 1M rows x dim 128, pooling 32,
    uniform indices, FP32 and FP16 tables, at full size."""
    _full_size_check(gpu_device, wl.paper_memory_benchmark(dtype, batch), "fp32", f"-membench-{dtype}-{batch}",
                     2000 + dtype)


def _full_size_check(dev, spec, variant, k, seed):
    sixteen = variant in ("16bit", "all3")
    table_major = variant in ("table", "all3")
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info(dev)
    need = spec.weight_bytes + 40 * spec.expected_lookups() + 10 * spec.batch * spec.sumD + (8 << 30)
    if free < need:
        pytest.skip(f"config {k} needs ~{need / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free")
    rng = np.random.default_rng(seed)
    print(f"\n[cfg{k}] generating {spec.weight_bytes / 1e9:.1f} GB of tables", flush=True)
    weights = wl.make_weights(spec, dev)
    batch = wl.make_batch(spec, dev, it=0)
    grad = wl.make_grad(spec, dev)
    if sixteen:
        grad = grad.to(torch.bfloat16)
    N, B, T = batch.num_indices, spec.batch, spec.T
    cols = np.concatenate([[0], np.cumsum(spec.dims)])
    # what the library is handed: the [B, sumD] gradient itself, or its per-table blocks one after another
    grad_arg = grad
    if table_major:
        grad_arg = torch.cat([grad[:, int(cols[t]):int(cols[t + 1])].reshape(-1) for t in range(T)])
    print(f"[cfg{k}] N={N} T={T} B={B}", flush=True)
    op = tbe.TableBatchedEmbeddingBags(spec.rows, spec.dims, spec.dtype, B, N, device=dev, weights=weights,
                                       output_dtype=tbe.TBE_DTYPE_FP16 if sixteen else tbe.TBE_DTYPE_FP32,
                                       grad_dtype=tbe.TBE_DTYPE_BF16 if sixteen else tbe.TBE_DTYPE_FP32,
                                       layout=tbe.TBE_LAYOUT_TABLE_MAJOR if table_major else tbe.TBE_LAYOUT_BATCH_MAJOR)
    assert op.check_inputs(batch.indices, batch.offsets, B, num_indices=N) == tbe.TBE_OK

    R = np.concatenate([[0], np.cumsum(spec.rows)])
    woffs = np.concatenate([[0], np.cumsum(spec.rows * spec.dims.astype(np.int64))])
    tables = _sample_tables(spec, rng)
    tab_off = batch.offsets[::B].cpu().numpy()          # positions where each table's lookups start

    # ---------------- forward
    out = op.forward(batch.indices, batch.offsets, B, num_indices=N)
    torch.cuda.synchronize()
    worst_f = worst_plain = 0.0
    for t in tables:
        D, H = int(spec.dims[t]), int(spec.rows[t])
        offs_t = batch.offsets[t * B:(t + 1) * B + 1].cpu().numpy()
        lens = np.diff(offs_t)
        bags = set(rng.integers(0, B, 48).tolist()) | {int(np.argmax(lens)), int(np.argmin(lens))}
        bags = np.array(sorted(bags))
        idx_t = batch.indices[int(offs_t[0]):int(offs_t[-1])].cpu().numpy()
        pieces = [idx_t[offs_t[b] - offs_t[0]:offs_t[b + 1] - offs_t[0]] for b in bags]
        need_rows, inv = np.unique(np.concatenate(pieces) if pieces else np.zeros(0, np.int32), return_inverse=True)
        if need_rows.size == 0:
            need_rows = np.zeros(1, np.int64)
            inv = np.zeros(0, np.int64)
        Wt = weights[int(woffs[t]):int(woffs[t + 1])].view(H, D)
        sub_w = Wt[torch.from_numpy(need_rows.astype(np.int64)).to(dev)].cpu().numpy().ravel()
        sub_off = np.zeros(len(bags) + 1, np.int64)
        sub_off[1:] = np.cumsum([len(p) for p in pieces])
        ref, absref = orc.forward(np.array([len(need_rows)], np.int64), np.array([D], np.int32), spec.dtype, sub_w,
                                  inv.astype(np.int32), sub_off, len(bags), want_absref=True)
        if table_major:
            out_t = out.view(-1)[B * int(cols[t]):B * int(cols[t + 1])].view(B, D)
        else:
            out_t = out[:, int(cols[t]):int(cols[t + 1])]
        got = out_t[torch.from_numpy(bags).to(dev)].float().cpu().numpy()
        if sixteen:
            # one extra rounding of the fp32 sum to fp16 (2^-11 relative, 2^-25 absolute for subnormals)
            r64 = ref.astype(np.float64)
            tol = tl.RTOL_FP32 * np.maximum(np.abs(r64), absref) + 2.0 ** -11 * np.abs(r64) + 2.0 ** -25
            assert (np.abs(got.astype(np.float64) - r64) <= tol).all(), f"cfg{k} table {t} fp16 output"
        else:
            worst_f = max(worst_f, tl.assert_forward_close(got, ref, absref, f"cfg{k} table {t}"))
            # also the plain relative error, on elements that are not the result of heavy cancellation
            big = np.abs(ref) > 0.05 * absref
            if big.any():
                worst_plain = max(worst_plain, float(np.max(np.abs(got[big].astype(np.float64) - ref[big]) / np.abs(ref[big]))))
    print(f"[cfg{k}] forward sampled ok, worst rel err {worst_f:.2e} (plain relative, |ref| > 5% of sum|terms|: "
          f"{worst_plain:.2e})", flush=True)

    # ---------------- backward: record what the oracle needs before the in-place update
    samples = {}
    for t in tables:
        D, H = int(spec.dims[t]), int(spec.rows[t])
        lo, hi = int(tab_off[t]), int(tab_off[t + 1])
        idx_t = batch.indices[lo:hi]
        cnt = torch.bincount(idx_t.to(torch.int64), minlength=H)
        touched = torch.nonzero(cnt).flatten()
        if touched.numel() == 0:
            continue
        c_t = cnt[touched]
        pick = [touched[torch.argmax(c_t)].item()]
        for thr in (256, 512, 513, 1024):            # runs at / just past the chunk and split thresholds
            near = touched[(c_t >= thr) & (c_t <= thr + 40)]
            if near.numel():
                pick.append(near[0].item())
        perm = torch.from_numpy(rng.permutation(touched.numel())[:150]).to(dev)
        pick += touched[perm].tolist()
        rows_s = np.unique(np.array(pick, np.int64))
        Wt = weights[int(woffs[t]):int(woffs[t + 1])].view(H, D)
        samples[t] = dict(rows=rows_s, w_old=Wt[torch.from_numpy(rows_s).to(dev)].cpu().numpy().copy(),
                          counts=cnt[torch.from_numpy(rows_s).to(dev)].cpu().numpy())
    op.backward_rowwise_adagrad(batch.indices, batch.offsets, B, grad_arg, spec.lr, spec.eps, num_indices=N)
    art = op.artifacts()
    U = art["num_unique"]
    print(f"[cfg{k}] backward done, U={U} ({U / N:.3f} of N)", flush=True)

    # ---------------- integer artefacts
    sk, sv, uk, so = art["sorted_keys"], art["sorted_vals"], art["unique_keys"], art["seg_offsets"]
    if N <= 40_000_000:
        ref_art = orc.sort_artifacts(spec.rows, B, batch.indices.cpu().numpy(), batch.offsets.cpu().numpy())
        tl.assert_artifacts_equal(art, ref_art, f"cfg{k}")
        print(f"[cfg{k}] integer artefacts bit-exact against the oracle (whole arrays)", flush=True)
    skl = sk.to(torch.int64) & 0xFFFFFFFF
    assert bool((skl[1:] >= skl[:-1]).all()), "sorted keys must not decrease"
    same = skl[1:] == skl[:-1]
    assert bool((sv[1:][same] >= sv[:-1][same]).all()), "payload order inside a run (stability)"
    heads = torch.cat([torch.ones(1, dtype=torch.bool, device=dev), ~same])
    assert int(heads.sum().item()) == U
    assert torch.equal(torch.nonzero(heads).flatten().to(torch.int32), so[:-1]) and int(so[-1].item()) == N
    assert torch.equal(sk[heads], uk)
    del same, heads
    for t in tables:                                      # exact, per sampled table
        lo, hi = int(tab_off[t]), int(tab_off[t + 1])
        if hi - lo > 30_000_000:
            continue
        offs_t = (batch.offsets[t * B:(t + 1) * B + 1] - lo).cpu().numpy()
        ref_t = orc.sort_artifacts(spec.rows[t:t + 1], B, batch.indices[lo:hi].cpu().numpy(), offs_t)
        assert np.array_equal((skl[lo:hi] - int(R[t])).cpu().numpy().astype(np.uint32), ref_t.sorted_keys), f"table {t} keys"
        assert np.array_equal(sv[lo:hi].cpu().numpy(), ref_t.sorted_vals), f"table {t} payloads"
    print(f"[cfg{k}] integer artefacts: properties + sampled tables exact", flush=True)
    del skl

    # ---------------- updated rows vs oracle on reduced problems
    worst_w = worst_m = 0.0
    rtol = tl.rtol_for(spec.dtype)
    for t, s in samples.items():
        D, H = int(spec.dims[t]), int(spec.rows[t])
        lo, hi = int(tab_off[t]), int(tab_off[t + 1])
        idx_t = batch.indices[lo:hi].cpu().numpy()
        offs_t = (batch.offsets[t * B:(t + 1) * B + 1] - lo).cpu().numpy()
        rows_s = s["rows"]
        pos = np.flatnonzero(np.isin(idx_t, rows_s))
        bag_of = np.searchsorted(offs_t, pos, side="right") - 1
        sub_idx = np.searchsorted(rows_s, idx_t[pos]).astype(np.int32)
        sub_off = np.zeros(B + 1, np.int64)
        sub_off[1:] = np.cumsum(np.bincount(bag_of, minlength=B))
        g_t = np.ascontiguousarray(grad[:, int(cols[t]):int(cols[t + 1])].float().cpu().numpy())
        w_ref = s["w_old"].ravel().copy()
        m_ref = np.zeros(len(rows_s), np.float32)
        det = orc.backward_rowwise_adagrad(np.array([len(rows_s)], np.int64), np.array([D], np.int32), spec.dtype,
                                           w_ref, m_ref, sub_idx, sub_off, B, g_t, spec.lr, spec.eps, want_detail=True)
        Wt = weights[int(woffs[t]):int(woffs[t + 1])].view(H, D)
        sel = torch.from_numpy(rows_s).to(dev)
        w_gpu = Wt[sel].cpu().numpy()
        m_gpu = op.state[int(R[t]):int(R[t + 1])][sel].cpu().numpy()
        gabs = det.Gabs.reshape(-1, D)
        lr, eps = float(np.float32(spec.lr)), float(np.float32(spec.eps))
        scale = np.abs(s["w_old"].astype(np.float64)) + lr * gabs / (np.sqrt(det.m_new)[:, None] + eps)
        rel = np.abs(w_gpu.astype(np.float64) - w_ref.reshape(-1, D).astype(np.float64)) / (scale + 1e-300)
        assert rel.max() <= rtol, f"cfg{k} table {t}: weight rel err {rel.max():.3e} (run length {s['counts'][np.argmax(rel.max(1))]})"
        rel_m = np.abs(m_gpu.astype(np.float64) - m_ref.astype(np.float64)) / ((gabs ** 2).mean(1) + 1e-300)
        assert rel_m.max() <= tl.RTOL_FP32, f"cfg{k} table {t}: moment rel err {rel_m.max():.3e}"
        worst_w, worst_m = max(worst_w, float(rel.max())), max(worst_m, float(rel_m.max()))
    print(f"[cfg{k}] sampled rows ok ({sum(len(s['rows']) for s in samples.values())} rows, longest run "
          f"{max(int(s['counts'].max()) for s in samples.values())}), worst rel err w {worst_w:.2e} m {worst_m:.2e}", flush=True)

    # ---------------- nothing but touched rows was written
    touched_mask = torch.zeros(spec.total_rows, dtype=torch.bool, device=dev)
    touched_mask[uk.to(torch.int64) & 0xFFFFFFFF] = True
    assert bool((op.state[~touched_mask] == 0).all()), "moment of an untouched row changed"
    # element -> linear row id, per table, in chunks aligned with the regenerated initial weights
    changed_rows = torch.zeros(spec.total_rows, dtype=torch.bool, device=dev)
    for lo, hi, w0 in _regen_chunks(spec, dev):
        diff = torch.nonzero(weights[lo:hi] != w0).flatten() + lo
        if diff.numel():
            tt = torch.searchsorted(torch.from_numpy(woffs).to(dev), diff, right=True) - 1
            Dt = torch.from_numpy(spec.dims.astype(np.int64)).to(dev)[tt]
            rid = torch.from_numpy(R).to(dev)[tt] + (diff - torch.from_numpy(woffs).to(dev)[tt]) // Dt
            changed_rows[rid] = True
        del w0, diff
    assert not bool((changed_rows & ~touched_mask).any()), "a row that was never looked up was written"
    print(f"[cfg{k}] untouched rows bit-identical; {int(changed_rows.sum().item())} of {U} touched rows changed bits",
          flush=True)
    op.close()
