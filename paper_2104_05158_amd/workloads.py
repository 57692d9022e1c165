"""Seeded synthetic DLRM-shaped inputs for the table-batched embedding-bag operator.

This module holds NO arithmetic of the method itself (no pooling, no sort, no optimizer):
it only draws table shapes, jagged (indices, offsets) batches, initial weights and
upstream gradients.  It is the one module both the HIP path's callers and the CPU
oracle's callers may use, so that the two are fed identical inputs.

Shapes follow the five benchmark configurations (1 table fp32 toy case; 8 x 1M x 128
fp32 uniform; 64 tables fp16 Zipf(1.05); 128+1 mixed-dim tables fp16 Zipf(1.1) with a
50M x 256 row-wise shard; 400 tables / ~120 GB fp16) which are in turn consistent with
the production model shapes of Table 3 of arxiv 2104.05158 (dims 4..384, average
pooling 15..70) and with the memory benchmark of its Appendix A (64 tables x 1M rows x
dim 128, pooling 32).  They stand in for production models and traces, which are not
public.

Everything is generated with torch on the requested device (CPU for small parity
cases, the GPU for the large ones whose tables do not fit in host memory); the seed
fixes the result for a given device type.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

BASE_SEED = 20210405
_ZIPF_SCATTER_PRIME = 2147483647  # 2^31-1 > every table height, hence coprime to it


@dataclass
class TableSpec:
    rows: np.ndarray            # int64[T]
    dims: np.ndarray            # int32[T]
    dtype: int                  # 0 fp32, 1 fp16 storage
    pooling_mean: np.ndarray    # float64[T]; mean bag length per table
    pooling_kind: str           # "fixed" | "poisson"
    index_dist: str             # "uniform" | "zipf"
    zipf_s: float = 0.0
    batch: int = 0
    name: str = ""
    lr: float = 0.01
    eps: float = 1e-8
    notes: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return len(self.rows)

    @property
    def sumD(self) -> int:
        return int(self.dims.sum())

    @property
    def weight_elems(self) -> int:
        return int((self.rows * self.dims.astype(np.int64)).sum())

    @property
    def weight_bytes(self) -> int:
        return self.weight_elems * (4 if self.dtype == 0 else 2)

    @property
    def total_rows(self) -> int:
        return int(self.rows.sum())

    def expected_lookups(self) -> float:
        return float(self.pooling_mean.sum() * self.batch)


def _loguniform_int(rng, lo, hi, n):
    return np.floor(10.0 ** rng.uniform(math.log10(lo), math.log10(hi), size=n)).astype(np.int64)


def config(k: int, seed_offset: int = 0, scale: float = 1.0) -> TableSpec:
    """Benchmark configuration k in 0..4.  `scale` < 1 shrinks table heights and batch by the
    same factor (parity-test miniatures of the large configurations); 1.0 is the real size."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * k + seed_offset))
    sc = lambda x: max(1, int(round(x * scale)))
    if k == 0:
        return TableSpec(np.array([sc(10_000)], np.int64), np.array([64], np.int32), 0,
                         np.array([8.0]), "fixed", "uniform", batch=sc(256), name="cfg0")
    if k == 1:
        T = 8
        return TableSpec(np.full(T, sc(1_000_000), np.int64), np.full(T, 128, np.int32), 0,
                         np.full(T, 20.0), "poisson", "uniform", batch=sc(4096), name="cfg1")
    if k == 2:
        T = 64
        rows = np.maximum(1, (_loguniform_int(rng, 1e5, 1e7, T) * scale).astype(np.int64))
        lam = 10.0 ** rng.uniform(0.0, 2.0, size=T)
        return TableSpec(rows, np.full(T, 128, np.int32), 1, lam, "poisson", "zipf", 1.05,
                         batch=sc(16384), name="cfg2")
    if k == 3:
        T = 128
        rows = np.maximum(1, (_loguniform_int(rng, 1e4, 2e7, T) * scale).astype(np.int64))
        dims = rng.choice(np.array([32, 64, 128, 256], np.int32), size=T)
        rows = np.concatenate([rows, np.array([sc(50_000_000)], np.int64)])
        dims = np.concatenate([dims, np.array([256], np.int32)]).astype(np.int32)
        return TableSpec(rows, dims, 1, np.full(T + 1, 30.0), "poisson", "zipf", 1.1,
                         batch=sc(32768), name="cfg3")
    if k == 4:
        T = 400
        rows = _loguniform_int(rng, 1e5, 5e7, T)
        dims = rng.choice(np.array([64, 128], np.int32), size=T).astype(np.int32)
        target = 120e9 * scale
        f = target / float((rows * dims).sum() * 2)
        rows = np.maximum(1, np.floor(rows * f).astype(np.int64))
        return TableSpec(rows, dims, 1, np.full(T, 30.0), "poisson", "zipf", 1.05,
                         batch=sc(65536), name="cfg4", notes={"row_rescale": f})
    raise ValueError("config index must be 0..4")


def paper_memory_benchmark(dtype: int, batch: int, tables: int = 64) -> TableSpec:
    """Appendix A memory benchmark shape: 64 tables x 1M rows x dim 128, pooling 32, uniform."""
    return TableSpec(np.full(tables, 1_000_000, np.int64), np.full(tables, 128, np.int32), dtype,
                     np.full(tables, 32.0), "fixed", "uniform", batch=batch,
                     name=f"paper_membench_{'fp32' if dtype == 0 else 'fp16'}_b{batch}")


def custom(rows, dims, dtype, batch, pooling_mean, pooling_kind="poisson", index_dist="uniform",
           zipf_s=1.05, name="custom") -> TableSpec:
    rows = np.asarray(rows, np.int64)
    dims = np.asarray(dims, np.int32)
    pm = np.broadcast_to(np.asarray(pooling_mean, np.float64), rows.shape).copy()
    return TableSpec(rows, dims, dtype, pm, pooling_kind, index_dist, zipf_s, batch=batch, name=name)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


@dataclass
class Batch:
    indices: torch.Tensor   # int32[N]
    offsets: torch.Tensor   # int64[T*B+1]
    num_indices: int


def make_batch(spec: TableSpec, device="cpu", it: int = 0, seed: Optional[int] = None) -> Batch:
    """One jagged batch in table-major order (bag id = t*B + b)."""
    device = torch.device(device)
    seed = BASE_SEED + 7919 * (it + 1) if seed is None else seed
    g = _gen(device, seed)
    T, B = spec.T, spec.batch
    if spec.pooling_kind == "fixed":
        lens = torch.tensor(np.repeat(np.round(spec.pooling_mean).astype(np.int64), B), device=device)
    else:
        lam = torch.tensor(np.repeat(spec.pooling_mean, B), dtype=torch.float32, device=device)
        lens = torch.poisson(lam, generator=g).to(torch.int64)
    offsets = torch.zeros(T * B + 1, dtype=torch.int64, device=device)
    torch.cumsum(lens, 0, out=offsets[1:])
    per_table = lens.view(T, B).sum(1).cpu().numpy()
    N = int(per_table.sum())
    indices = torch.empty(N, dtype=torch.int32, device=device)
    pos = 0
    for t in range(T):
        n = int(per_table[t])
        H = int(spec.rows[t])
        if n == 0:
            continue
        if spec.index_dist == "uniform":
            idx = torch.randint(0, H, (n,), generator=g, device=device, dtype=torch.int64)
        else:
            # bounded Zipf(s) over ranks 1..H by inverting the continuous power-law CDF, then the
            # ranks are scattered over the table with a fixed bijection so that hot rows are not
            # neighbours in memory (production ids are hashed)
            s = spec.zipf_s
            u = torch.rand(n, generator=g, device=device, dtype=torch.float64)
            x = (((H + 1.0) ** (1.0 - s) - 1.0) * u + 1.0) ** (1.0 / (1.0 - s))
            rank = x.floor().to(torch.int64).clamp_(1, H)
            idx = ((rank - 1) * _ZIPF_SCATTER_PRIME) % H
        indices[pos:pos + n] = idx.to(torch.int32)
        pos += n
    return Batch(indices, offsets, N)


def make_weights(spec: TableSpec, device="cpu", seed: Optional[int] = None,
                 chunk_elems: int = 1 << 28) -> torch.Tensor:
    """Flat table storage, U(-0.01, 0.01), in the storage type; generated in chunks so that the
    fp32 staging of a 100+ GB fp16 table never exceeds `chunk_elems` elements."""
    device = torch.device(device)
    g = _gen(device, BASE_SEED + 17 if seed is None else seed)
    n = spec.weight_elems
    dt = torch.float32 if spec.dtype == 0 else torch.float16
    w = torch.empty(n, dtype=dt, device=device)
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        r = torch.rand(hi - lo, generator=g, device=device, dtype=torch.float32)
        w[lo:hi] = (r * 0.02 - 0.01).to(dt)
    return w


def make_moments(spec: TableSpec, device="cpu") -> torch.Tensor:
    return torch.zeros(spec.total_rows, dtype=torch.float32, device=device)


def make_grad(spec: TableSpec, device="cpu", it: int = 0, seed: Optional[int] = None,
              std: float = 1.0) -> torch.Tensor:
    """Upstream gradient of the pooled output, N(0, std^2), float32 [B, sumD]."""
    device = torch.device(device)
    g = _gen(device, BASE_SEED + 104729 * (it + 1) if seed is None else seed)
    out = torch.empty(spec.batch, spec.sumD, dtype=torch.float32, device=device)
    rows_per = max(1, (1 << 28) // max(1, spec.sumD))
    for lo in range(0, spec.batch, rows_per):
        hi = min(spec.batch, lo + rows_per)
        out[lo:hi].normal_(0.0, std, generator=g)
    return out


def tiny_random(seed: int, T: int = 3, max_rows: int = 16, dims=(4, 8), B: int = 4, max_len: int = 5,
                dtype: int = 0, dup_heavy: bool = True):
    """Small numpy-only case for brute-force checks: returns (spec, indices, offsets, weights, grad)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = rng.integers(1, max_rows + 1, size=T).astype(np.int64)
    d = rng.choice(np.asarray(dims, np.int32), size=T).astype(np.int32)
    lens = rng.integers(0, max_len + 1, size=T * B)
    offsets = np.zeros(T * B + 1, np.int64)
    offsets[1:] = np.cumsum(lens)
    idx: List[np.ndarray] = []
    for t in range(T):
        n = int(lens[t * B:(t + 1) * B].sum())
        hi = int(rows[t]) if not dup_heavy else max(1, min(int(rows[t]), 4))
        idx.append(rng.integers(0, hi, size=n))
    indices = np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32)
    spec = custom(rows, d, dtype, B, 0.0, name="tiny")
    wdt = np.float32 if dtype == 0 else np.float16
    weights = rng.uniform(-1, 1, size=spec.weight_elems).astype(wdt)
    grad = rng.normal(size=(B, spec.sumD)).astype(np.float32)
    return spec, indices, offsets, weights, grad


def make_wtb_input(W: int, T: int, B: int, rows, pooling_mean: float, device="cpu", seed: int = 0,
                   max_len: Optional[int] = None):
    """Combined-format input as it arrives after the all-to-alls of table-wise sharding (Section 7.1):
    int32 lengths of the W*T*B bags in (W, T, B) order and their concatenated int32 indices (uniform
    rows of the bag's table).  `max_len` draws lengths uniformly in [0, max_len] instead of Poisson."""
    device = torch.device(device)
    g = _gen(device, BASE_SEED + 31 * seed + 5)
    n = W * T * B
    if max_len is None:
        lens = torch.poisson(torch.full((n,), float(pooling_mean), device=device), generator=g).to(torch.int32)
    else:
        lens = torch.randint(0, max_len + 1, (n,), generator=g, device=device, dtype=torch.int32)
    total = int(lens.sum().item())
    H = torch.as_tensor(np.asarray(rows, np.int64), device=device)
    bag_table = torch.arange(T, device=device).repeat_interleave(B).repeat(W)           # table of bag (w,t,b)
    pos_table = bag_table.repeat_interleave(lens.to(torch.int64), output_size=total)
    u = torch.rand(total, generator=g, device=device, dtype=torch.float64)
    indices = (u * H[pos_table].to(torch.float64)).floor().to(torch.int64)
    indices = torch.minimum(indices, H[pos_table] - 1).to(torch.int32)
    return lens, indices
