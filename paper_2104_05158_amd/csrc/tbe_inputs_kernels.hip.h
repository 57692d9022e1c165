// Device kernels of the input-side operations that sit next to the embedding operator
// (arxiv 2104.05158, Section 7.1: combined lengths format, (W,T,B) -> (T,W,B) permute; Section 4
// "Row-wise parallelism" + Section 7.1: bucketize).  gfx950, wave64.
//
// All of it is integer streaming work bound by memory bandwidth: coalesced 4-byte or 16-byte
// accesses, wavefront ballots for ranks, no atomics except integer counters (whose result does not
// depend on their order), so every output is exact and identical run to run.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbe_in {

constexpr int kWave = 64;
constexpr int kThreads = 256;
constexpr int kScanGroups = 4;                         // int4 groups per thread
constexpr int kScanTile = kThreads * 4 * kScanGroups;  // 4096 lengths per workgroup
constexpr int kCopyPerThread = 16;
constexpr int kCopyTile = kThreads * kCopyPerThread;   // 4096 index positions per workgroup
constexpr int kMaxShards = 1024;

// ---------------------------------------------------------------- lengths -> offsets (Section 7.1)
//
// Exclusive prefix sum of int32 lengths into int64 offsets in three launches: per-tile totals, one
// workgroup scans the totals, every tile rescans itself with its base.  Inside a tile a thread
// owns one int4 of each of kScanGroups consecutive 1024-length groups, so loads are 16 bytes per
// lane and contiguous across the wavefront.

__device__ __forceinline__ int64_t block_exclusive_scan64(int64_t v, int64_t* s_wave /*[4]*/, int64_t& block_total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    int64_t incl = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int64_t up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    if (lane == kWave - 1)
        s_wave[wave] = incl;
    __syncthreads();
    int64_t woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) {
        const int64_t c = s_wave[w];
        if (w < wave)
            woff += c;
        tot += c;
    }
    block_total = tot;
    __syncthreads();
    return woff + incl - v;
}

__device__ __forceinline__ int4 load_lengths4(const int32_t* __restrict__ lengths, int64_t i, int64_t n)
{
    if (i + 4 <= n)
        return *reinterpret_cast<const int4*>(lengths + i);
    int4 v = make_int4(0, 0, 0, 0);
    if (i < n) v.x = lengths[i];
    if (i + 1 < n) v.y = lengths[i + 1];
    if (i + 2 < n) v.z = lengths[i + 2];
    return v;
}

__global__ __launch_bounds__(kThreads) void scan64_reduce_kernel(const int32_t* __restrict__ lengths,
                                                                 int64_t* __restrict__ block_sums, int64_t n)
{
    __shared__ int64_t s_wave[kThreads / kWave];
    const int64_t tile = (int64_t)blockIdx.x * kScanTile;
    int64_t s = 0;
#pragma unroll
    for (int g = 0; g < kScanGroups; ++g) {
        const int4 v = load_lengths4(lengths, tile + g * (kThreads * 4) + threadIdx.x * 4, n);
        s += (int64_t)v.x + v.y + v.z + v.w;
    }
    int64_t tot;
    (void)block_exclusive_scan64(s, s_wave, tot);
    if (threadIdx.x == 0)
        block_sums[blockIdx.x] = tot;
}

// one workgroup: exclusive scan of block_sums[nb] in place, kTopPerThread consecutive sums per thread
constexpr int kTopPerThread = 8;
__global__ __launch_bounds__(kThreads) void scan64_top_kernel(int64_t* __restrict__ block_sums, int32_t nb)
{
    __shared__ int64_t s_wave[kThreads / kWave];
    int64_t carry = 0;
    for (int base = 0; base < nb; base += kThreads * kTopPerThread) {
        const int i0 = base + threadIdx.x * kTopPerThread;
        int64_t v[kTopPerThread];
        int64_t s = 0;
#pragma unroll
        for (int k = 0; k < kTopPerThread; ++k) {
            v[k] = i0 + k < nb ? block_sums[i0 + k] : 0;
            s += v[k];
        }
        int64_t tot;
        int64_t run = carry + block_exclusive_scan64(s, s_wave, tot);
#pragma unroll
        for (int k = 0; k < kTopPerThread; ++k) {
            if (i0 + k < nb)
                block_sums[i0 + k] = run;
            run += v[k];
        }
        carry += tot;
    }
}

__global__ __launch_bounds__(kThreads) void scan64_apply_kernel(const int32_t* __restrict__ lengths,
                                                                const int64_t* __restrict__ block_sums,
                                                                int64_t* __restrict__ offsets, int64_t n)
{
    __shared__ int64_t s_wave[kThreads / kWave];
    const int64_t tile = (int64_t)blockIdx.x * kScanTile;
    int64_t carry = block_sums[blockIdx.x];
#pragma unroll
    for (int g = 0; g < kScanGroups; ++g) {
        const int64_t i = tile + g * (kThreads * 4) + threadIdx.x * 4;
        const int4 v = load_lengths4(lengths, i, n);
        const int64_t s = (int64_t)v.x + v.y + v.z + v.w;
        int64_t tot;
        const int64_t o0 = carry + block_exclusive_scan64(s, s_wave, tot);
        const int64_t o1 = o0 + v.x, o2 = o1 + v.y, o3 = o2 + v.z, o4 = o3 + v.w;
        if (i + 4 <= n) {
            // offsets + i is 32-byte aligned (i is a multiple of 4)
            *reinterpret_cast<longlong2*>(offsets + i) = make_longlong2(o0, o1);
            *reinterpret_cast<longlong2*>(offsets + i + 2) = make_longlong2(o2, o3);
            if (i + 4 == n)
                offsets[n] = o4;
        } else if (i < n) {
            offsets[i] = o0;
            if (i + 1 < n) offsets[i + 1] = o1; else offsets[n] = o1;
            if (i + 2 < n) offsets[i + 2] = o2; else if (i + 2 == n) offsets[n] = o2;
            if (i + 3 == n) offsets[n] = o3;
        }
        carry += tot;
    }
}

__global__ __launch_bounds__(kThreads) void fill_i32_kernel(int32_t* __restrict__ p, int64_t n, int32_t value)
{
    const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i + 4 <= n) {
        *reinterpret_cast<int4*>(p + i) = make_int4(value, value, value, value);
    } else {
        for (int64_t k = i; k < n; ++k)
            p[k] = value;
    }
}

__global__ void write_zero_offset_kernel(int64_t* __restrict__ offsets) { offsets[0] = 0; }

// ---------------------------------------------------------------- (W,T,B) -> (T,W,B) permute (Section 7.1)
//
// Bags (w,t,0..B-1) are consecutive on both sides, so the lengths move in rows of B and the indices
// move as W*T contiguous blocks whose borders are offsets[q*B].

// One workgroup per 256*VEC bags of one output row q = t*W + w; VEC = 4 (16-byte accesses) needs B % 4 == 0.
template <int VEC>
__global__ __launch_bounds__(kThreads) void permute_lengths_kernel(const int32_t* __restrict__ lengths_in,
                                                                   int32_t* __restrict__ lengths_out, int32_t W,
                                                                   int32_t T, int32_t B, int32_t blocks_per_row)
{
    const int q = blockIdx.x / blocks_per_row;
    const int b = ((blockIdx.x - q * blocks_per_row) * kThreads + threadIdx.x) * VEC;
    if (b >= B)
        return;
    const int t = q / W;
    const int w = q - t * W;
    const int64_t dst = (int64_t)q * B + b, src = ((int64_t)w * T + t) * B + b;
    if (VEC == 4)
        *reinterpret_cast<int4*>(lengths_out + dst) = *reinterpret_cast<const int4*>(lengths_in + src);
    else
        lengths_out[dst] = lengths_in[src];
}

// last q in [lo, hi] with offsets[q*B] <= p   (offsets[lo*B] <= p is given)
__device__ __forceinline__ int find_block(const int64_t* __restrict__ offsets, int64_t B, int lo, int hi, int64_t p)
{
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (offsets[(int64_t)mid * B] <= p)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// Every workgroup copies kCopyTile consecutive OUTPUT positions.  The output rows the tile touches
// are bracketed once per workgroup; when they are few (the usual case: a row holds B bags) their
// borders and source shifts are staged in LDS, so a position costs a short LDS search, one load and
// one store, all loads of a thread issued before its stores.
constexpr int kCopyLdsRows = 64;
__global__ __launch_bounds__(kThreads) void permute_indices_kernel(const int32_t* __restrict__ indices_in,
                                                                   const int64_t* __restrict__ offsets_in,
                                                                   const int64_t* __restrict__ offsets_out,
                                                                   int32_t* __restrict__ indices_out, int32_t W,
                                                                   int32_t T, int32_t B, int64_t n)
{
    __shared__ int s_q[2];
    __shared__ int64_t s_start[kCopyLdsRows];   // first output position of row q_lo + i
    __shared__ int64_t s_shift[kCopyLdsRows];   // source position minus output position inside that row
    const int64_t tile = (int64_t)blockIdx.x * kCopyTile;
    const int64_t tile_end = min(tile + kCopyTile, n);
    const int rows = W * T;
    if (threadIdx.x < 2)
        s_q[threadIdx.x] = find_block(offsets_out, B, 0, rows - 1, threadIdx.x == 0 ? tile : tile_end - 1);
    __syncthreads();
    const int q_lo = s_q[0], q_hi = s_q[1];
    const int nrows = q_hi - q_lo + 1;
    const bool staged = nrows <= kCopyLdsRows;
    if (staged && (int)threadIdx.x < nrows) {
        const int q = q_lo + threadIdx.x;
        const int t = q / W;
        const int w = q - t * W;
        const int64_t start = offsets_out[(int64_t)q * B];
        s_start[threadIdx.x] = start;
        s_shift[threadIdx.x] = offsets_in[((int64_t)w * T + t) * B] - start;
    }
    __syncthreads();
    int64_t src[kCopyPerThread];
#pragma unroll
    for (int i = 0; i < kCopyPerThread; ++i) {
        const int64_t p = min(tile + i * kThreads + threadIdx.x, tile_end - 1);
        if (staged) {
            int lo = 0, hi = nrows - 1;   // last row with s_start <= p
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (s_start[mid] <= p)
                    lo = mid;
                else
                    hi = mid - 1;
            }
            src[i] = p + s_shift[lo];
        } else {
            const int q = find_block(offsets_out, B, q_lo, q_hi, p);
            const int t = q / W;
            const int w = q - t * W;
            src[i] = offsets_in[((int64_t)w * T + t) * B] + (p - offsets_out[(int64_t)q * B]);
        }
    }
    int32_t v[kCopyPerThread];
#pragma unroll
    for (int i = 0; i < kCopyPerThread; ++i)
        v[i] = indices_in[src[i]];
#pragma unroll
    for (int i = 0; i < kCopyPerThread; ++i) {
        const int64_t p = tile + i * kThreads + threadIdx.x;
        if (p < tile_end)
            indices_out[p] = v[i];
    }
}

// ---------------------------------------------------------------- row-wise bucketize (Section 4, Section 7.1)
//
// Shard w of table t owns rows [w*blk_t, (w+1)*blk_t), blk_t = ceil(H_t / W).  The output order
// (w, t, b), with the input order kept inside every bag, makes the region of shard w a STABLE
// FILTER of the input stream: the elements of shard w, in input order.  So bucketize is one stable
// multi-way split of the index stream by shard, plus per-(shard, bag) counts:
//
//   pass 1 (count):  a workgroup owns `nbags` consecutive input bags, walks their positions with
//                    coalesced loads and counts (shard, bag) pairs with integer LDS atomics; the
//                    counts go out as rows of lengths_out (consecutive b for each shard).
//   prefix sum:      lengths_out -> offsets_out (the scan kernels above).
//   pass 2 (place):  the same bags per workgroup.  offsets_out at the workgroup's first bag is,
//                    for every shard, exactly where the workgroup's elements of that shard start.
//                    Positions are handled in sub-tiles: ballot-matched stable ranks per wavefront,
//                    prefix over wavefronts and shards in LDS, the sub-tile is reordered by shard
//                    inside LDS and written out in contiguous runs.
// WMAX bounds the number of shards the LDS tables are sized for.
__device__ __forceinline__ uint64_t match_key(uint32_t key, bool valid, int bits)
{
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
        const bool bit = (key >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
    }
    return peers;
}

constexpr int kBuckMaxBags = 256;   // bags per workgroup (fewer when W is large: nbags * W <= 8192)
constexpr int kBuckPerThread = 8;
constexpr int kBuckTile = kThreads * kBuckPerThread;  // 2048 positions per sub-tile

struct BuckBags {
    int32_t off[kBuckMaxBags + 1];   // bag borders relative to the workgroup's first position
    uint32_t blk[kBuckMaxBags];      // rows per shard of the bag's table
    float rcp[kBuckMaxBags];         // 1 / blk
    int32_t tab[kBuckMaxBags];       // table of the bag
};

// loads the workgroup's bag borders, tables and shard sizes; returns the first position (absolute)
__device__ __forceinline__ int64_t load_bags(BuckBags& sb, const int64_t* __restrict__ rows,
                                             const int64_t* __restrict__ offsets, int j0, int nb, int32_t B, int32_t W)
{
    const int64_t base = offsets[j0];
    for (int i = threadIdx.x; i <= nb; i += kThreads)
        sb.off[i] = (int32_t)(offsets[j0 + i] - base);
    for (int i = threadIdx.x; i < nb; i += kThreads) {
        const int t = (j0 + i) / B;
        sb.tab[i] = t;
        const uint32_t blk = (uint32_t)((rows[t] + W - 1) / W);
        sb.blk[i] = blk;
        sb.rcp[i] = 1.0f / (float)blk;
    }
    __syncthreads();
    return base;
}

// last a in [0, nb) with off[a] <= p; nb <= 256: eight branch-free halvings, so that the searches of
// the positions a thread holds overlap their LDS latencies
__device__ __forceinline__ int find_bag(const int32_t* off, int nb, int p)
{
    int a = 0, c = nb;
#pragma unroll
    for (int step = 0; step < 8; ++step) {
        const int mid = (a + c) >> 1;
        const bool up = off[mid] <= p;       // mid == a once c - a <= 1: then a stays
        a = up ? mid : a;
        c = up ? c : max(mid, a + 1);
    }
    return a;
}

// floor(r / blk) for r < 2^31, 1 <= blk < 2^31, quotient <= 1024 in every valid case: the float estimate is off by
// at most one, which the remainder corrects.  (Invalid rows may give a wrong large value; callers clamp.)
__device__ __forceinline__ uint32_t div_rows(uint32_t r, uint32_t blk, float rcp_blk)
{
    uint32_t q = (uint32_t)((float)r * rcp_blk);
    const int32_t rem = (int32_t)(r - q * blk);
    q = rem < 0 ? q - 1 : q;
    q = rem >= (int32_t)blk ? q + 1 : q;
    return q;
}

__global__ __launch_bounds__(kThreads) void bucketize_count_kernel(const int64_t* __restrict__ rows,
                                                                   const int32_t* __restrict__ indices,
                                                                   const int64_t* __restrict__ offsets,
                                                                   int32_t* __restrict__ lengths_out, int32_t T,
                                                                   int32_t B, int32_t W, int32_t num_bags,
                                                                   int32_t nbags)
{
    __shared__ BuckBags sb;
    __shared__ int32_t s_cnt[8192];  // [W][nbags]
    const int j0 = blockIdx.x * nbags;
    const int nb = min(nbags, num_bags - j0);
    for (int i = threadIdx.x; i < W * nbags; i += kThreads)
        s_cnt[i] = 0;
    const int64_t base = load_bags(sb, rows, offsets, j0, nb, B, W);
    const int total = sb.off[nb];
    // Counting does not depend on the order, so a thread takes kBuckPerThread CONSECUTIVE positions: one bag
    // search for the first of them, then it only steps over the bag borders it meets.
    for (int p0 = threadIdx.x * kBuckPerThread; p0 < total; p0 += kThreads * kBuckPerThread) {
        uint32_t r[kBuckPerThread];
#pragma unroll
        for (int u = 0; u < kBuckPerThread; ++u)
            r[u] = (uint32_t)indices[base + min(p0 + u, total - 1)];
        int a = find_bag(sb.off, nb, p0);
        int next = sb.off[a + 1];
        uint32_t blk = sb.blk[a];
        float rcp = sb.rcp[a];
#pragma unroll
        for (int u = 0; u < kBuckPerThread; ++u) {
            const int p = p0 + u;
            if (p < total) {
                while (p >= next && a + 1 < nb) {   // p < total = off[nb]: a stays below nb even for bad offsets
                    ++a;
                    next = sb.off[a + 1];
                    blk = sb.blk[a];
                    rcp = sb.rcp[a];
                }
                const uint32_t w = min(div_rows(r[u], blk, rcp), (uint32_t)(W - 1));  // clamp: invalid rows only
                atomicAdd(&s_cnt[w * nbags + a], 1);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < W * nbags; i += kThreads) {
        const int w = i / nbags;
        const int a = i - w * nbags;
        if (a < nb) {
            const int t = sb.tab[a];
            lengths_out[((int64_t)w * T + t) * B + (j0 + a - t * B)] = s_cnt[i];
        }
    }
}

template <int WMAX>
__global__ __launch_bounds__(kThreads) void bucketize_place_kernel(const int64_t* __restrict__ rows,
                                                                   const int32_t* __restrict__ indices,
                                                                   const int64_t* __restrict__ offsets,
                                                                   const int64_t* __restrict__ offsets_out,
                                                                   int32_t* __restrict__ indices_out, int32_t T,
                                                                   int32_t B, int32_t W, int32_t wbits,
                                                                   int32_t num_bags, int32_t nbags)
{
    constexpr int kWaves = kThreads / kWave;
    constexpr int kDpt = (WMAX + kThreads - 1) / kThreads;  // shards per thread in the shard prefix sum
    __shared__ BuckBags sb;
    __shared__ uint32_t s_whist[kWaves][WMAX];
    __shared__ uint32_t s_dstart[WMAX];   // first slot of the shard inside the reordered sub-tile
    __shared__ int64_t s_goff[WMAX];      // output position of slot 0 of the shard, minus the slot
    __shared__ int64_t s_next[WMAX];      // output position of the shard's next element
    __shared__ int32_t s_val[kBuckTile];
    __shared__ uint16_t s_dig[kBuckTile];
    __shared__ uint32_t s_wave[kWaves];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int j0 = blockIdx.x * nbags;
    const int nb = min(nbags, num_bags - j0);
    const int64_t base = load_bags(sb, rows, offsets, j0, nb, B, W);
    const int total = sb.off[nb];
    {
        const int t0 = sb.tab[0];
        for (int d = threadIdx.x; d < W; d += kThreads)
            s_next[d] = offsets_out[((int64_t)d * T + t0) * B + (j0 - t0 * B)];
    }
    const uint64_t lt = (1ull << lane) - 1ull;

    for (int tile0 = 0; tile0 < total; tile0 += kBuckTile) {
        const int tile_cnt = min(kBuckTile, total - tile0);
        for (int i = threadIdx.x; i < kWaves * WMAX; i += kThreads)
            (&s_whist[0][0])[i] = 0;
        __syncthreads();

        // order inside the sub-tile: (wavefront, round, lane) = ascending position
        const int wbase = tile0 + wave * (kBuckTile / kWaves);
        uint32_t r[kBuckPerThread];
#pragma unroll
        for (int k = 0; k < kBuckPerThread; ++k)
            r[k] = (uint32_t)indices[base + min(wbase + k * kWave + lane, total - 1)];
        uint32_t dig[kBuckPerThread], rank[kBuckPerThread];
        int32_t local[kBuckPerThread];
#pragma unroll
        for (int k = 0; k < kBuckPerThread; ++k) {
            const int p = wbase + k * kWave + lane;
            const bool valid = p < total;
            const int a = find_bag(sb.off, nb, min(p, total - 1));
            const uint32_t blk = sb.blk[a];
            const uint32_t w = min(div_rows(r[k], blk, sb.rcp[a]), (uint32_t)(W - 1));
            local[k] = (int32_t)(r[k] - w * blk);
            dig[k] = w;
            const uint64_t peers = match_key(w, valid, wbits);
            const uint32_t pre = s_whist[wave][w];    // indexed as the LDS array it is (no generic pointer)
            const uint32_t below = (uint32_t)__popcll(peers & lt);
            if (valid && below == 0)
                s_whist[wave][w] = pre + (uint32_t)__popcll(peers);
            rank[k] = pre + below;
        }
        __syncthreads();

        // per shard: exclusive prefix over the wavefronts and the sub-tile total; then the exclusive
        // prefix of the totals over the shards (kDpt consecutive shards per thread)
        uint32_t tot[kDpt];
        uint32_t mine = 0;
#pragma unroll
        for (int i = 0; i < kDpt; ++i) {
            const int d = threadIdx.x * kDpt + i;
            uint32_t run = 0;
            if (d < W) {
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const uint32_t c = s_whist[w][d];
                    s_whist[w][d] = run;
                    run += c;
                }
            }
            tot[i] = run;
            mine += run;
        }
        uint32_t incl = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o);
            if (lane >= o)
                incl += up;
        }
        if (lane == kWave - 1)
            s_wave[wave] = incl;
        __syncthreads();
        uint32_t ex = incl - mine;
        for (int w = 0; w < wave; ++w)
            ex += s_wave[w];
#pragma unroll
        for (int i = 0; i < kDpt; ++i) {
            const int d = threadIdx.x * kDpt + i;
            if (d < W) {
                const int64_t nxt = s_next[d];
                s_dstart[d] = ex;
                s_goff[d] = nxt - (int64_t)ex;
                s_next[d] = nxt + tot[i];
            }
            ex += tot[i];
        }
        __syncthreads();

#pragma unroll
        for (int k = 0; k < kBuckPerThread; ++k) {
            const int p = wbase + k * kWave + lane;
            if (p < total) {
                const uint32_t pos = s_dstart[dig[k]] + s_whist[wave][dig[k]] + rank[k];
                s_val[pos] = local[k];
                s_dig[pos] = (uint16_t)dig[k];
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kBuckPerThread; ++k) {
            const int q = threadIdx.x + k * kThreads;
            if (q < tile_cnt)
                indices_out[s_goff[s_dig[q]] + q] = s_val[q];
        }
        __syncthreads();
    }
}

}  // namespace tbe_in
