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
constexpr int kMaxBagsPerWave = 32;

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

// one workgroup: exclusive scan of block_sums[nb] in place
__global__ __launch_bounds__(kThreads) void scan64_top_kernel(int64_t* __restrict__ block_sums, int32_t nb)
{
    __shared__ int64_t s_wave[kThreads / kWave];
    int64_t carry = 0;
    for (int base = 0; base < nb; base += kThreads) {
        const int i = base + threadIdx.x;
        const int64_t v = i < nb ? block_sums[i] : 0;
        int64_t tot;
        const int64_t ex = block_exclusive_scan64(v, s_wave, tot);
        if (i < nb)
            block_sums[i] = carry + ex;
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

// One workgroup per 256 bags of one output row q = t*W + w.
__global__ __launch_bounds__(kThreads) void permute_lengths_kernel(const int32_t* __restrict__ lengths_in,
                                                                   int32_t* __restrict__ lengths_out, int32_t W,
                                                                   int32_t T, int32_t B, int32_t blocks_per_row)
{
    const int q = blockIdx.x / blocks_per_row;
    const int b = (blockIdx.x - q * blocks_per_row) * kThreads + threadIdx.x;
    if (b >= B)
        return;
    const int t = q / W;
    const int w = q - t * W;
    lengths_out[(int64_t)q * B + b] = lengths_in[((int64_t)w * T + t) * B + b];
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
// are bracketed once per workgroup; each position then bisects inside that (usually 1-2 wide) bracket.
__global__ __launch_bounds__(kThreads) void permute_indices_kernel(const int32_t* __restrict__ indices_in,
                                                                   const int64_t* __restrict__ offsets_in,
                                                                   const int64_t* __restrict__ offsets_out,
                                                                   int32_t* __restrict__ indices_out, int32_t W,
                                                                   int32_t T, int32_t B, int64_t n)
{
    __shared__ int s_q[2];
    const int64_t tile = (int64_t)blockIdx.x * kCopyTile;
    const int64_t tile_end = min(tile + kCopyTile, n);
    const int rows = W * T;
    if (threadIdx.x < 2)
        s_q[threadIdx.x] = find_block(offsets_out, B, 0, rows - 1, threadIdx.x == 0 ? tile : tile_end - 1);
    __syncthreads();
    const int q_lo = s_q[0], q_hi = s_q[1];
#pragma unroll 4
    for (int i = 0; i < kCopyPerThread; ++i) {
        const int64_t p = tile + i * kThreads + threadIdx.x;
        if (p < tile_end) {
            const int q = find_block(offsets_out, B, q_lo, q_hi, p);
            const int t = q / W;
            const int w = q - t * W;
            const int64_t src = offsets_in[((int64_t)w * T + t) * B] + (p - offsets_out[(int64_t)q * B]);
            indices_out[p] = indices_in[src];
        }
    }
}

// ---------------------------------------------------------------- row-wise bucketize (Section 4, Section 7.1)
//
// Shard w of table t owns rows [w*blk_t, (w+1)*blk_t), blk_t = ceil(H_t / W).  A wavefront owns
// `bags_per_wave` consecutive input bags and walks their lookup positions 64 at a time in input
// order.  Lanes that hold the same (bag, shard) pair find each other by ballots: the number of
// lower lanes in that group is the position's rank inside the 64, and a small wavefront-private LDS
// table (one tagged counter per shard) carries the count of the one bag that continues into the
// next 64 positions.  Pass 1 (PLACE = false) adds the group sizes to lengths_out; after the
// prefix sum, pass 2 (PLACE = true) writes each local row id at offsets_out[bag'] + rank, which
// keeps the input order inside every output bag.
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

template <bool PLACE>
__global__ __launch_bounds__(kThreads) void bucketize_kernel(const int64_t* __restrict__ rows,
                                                             const int32_t* __restrict__ indices,
                                                             const int64_t* __restrict__ offsets,
                                                             int32_t* __restrict__ lengths_out,
                                                             const int64_t* __restrict__ offsets_out,
                                                             int32_t* __restrict__ indices_out, int32_t T, int32_t B,
                                                             int32_t W, int32_t wbits, int32_t num_bags,
                                                             int32_t bags_per_wave)
{
    __shared__ int32_t s_tag_all[PLACE ? kThreads / kWave : 1][PLACE ? kMaxShards : 1];
    __shared__ int32_t s_cnt_all[PLACE ? kThreads / kWave : 1][PLACE ? kMaxShards : 1];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    const int j0 = __builtin_amdgcn_readfirstlane((blockIdx.x * (kThreads / kWave) + wv) * bags_per_wave);
    if (j0 >= num_bags)
        return;
    const int nb = min(bags_per_wave, num_bags - j0);  // <= 32 < 64: lane nb holds the end offset
    const int64_t my_o64 = offsets[j0 + min(lane, nb)];
    const int64_t base = __shfl(my_o64, 0);
    const int my_o = (int)(my_o64 - base);
    const int total = __shfl(my_o, nb);
    const int my_t = (j0 + min(lane, nb - 1)) / B;
    const uint32_t my_blk = (uint32_t)((rows[my_t] + W - 1) / W);
    volatile int32_t* s_tag = s_tag_all[PLACE ? wv : 0];
    volatile int32_t* s_cnt = s_cnt_all[PLACE ? wv : 0];
    if (PLACE) {
        for (int i = lane; i < W; i += kWave)
            s_tag[i] = -1;
        __builtin_amdgcn_wave_barrier();
    }
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int c0 = 0; c0 < total; c0 += kWave) {
        const int p = c0 + lane;
        const bool valid = p < total;
        // bag a of position p: last a in [0, nb) with my_o[a] <= p (empty bags are skipped);
        // five halvings cover nb <= 32, every lane takes part in every shuffle
        int a = 0, c = nb;
#pragma unroll
        for (int step = 0; step < 5; ++step) {
            const int mid = (a + c) >> 1;
            const int v = __shfl(my_o, mid);
            if (c - a > 1) {
                if (v <= p)
                    a = mid;
                else
                    c = mid;
            }
        }
        const uint32_t r = (uint32_t)indices[base + min(p, total - 1)];
        const int t = __shfl(my_t, a);
        const uint32_t blk = (uint32_t)__shfl((int)my_blk, a);
        const uint32_t w = min(r / blk, (uint32_t)(W - 1));  // the clamp only matters for invalid rows
        const int32_t local = (int32_t)(r - w * blk);
        const uint64_t peers = match_key(((uint32_t)a << wbits) | w, valid, wbits + 5);
        const int below = __popcll(peers & lt);
        const int group = __popcll(peers);
        const int64_t dst_bag = ((int64_t)w * T + t) * B + (j0 + a - t * B);
        if (!PLACE) {
            if (valid && below == 0)
                atomicAdd(&lengths_out[dst_bag], group);
        } else {
            const int last_a = __shfl(a, min(kWave - 1, total - c0 - 1));
            const int prior = (valid && s_tag[w] == j0 + a) ? s_cnt[w] : 0;
            __builtin_amdgcn_wave_barrier();
            if (valid && a == last_a && (peers >> lane) == 1ull) {  // highest lane of its group
                s_tag[w] = j0 + a;
                s_cnt[w] = prior + group;
            }
            __builtin_amdgcn_wave_barrier();
            if (valid)
                indices_out[offsets_out[dst_bag] + prior + below] = local;
        }
    }
}

}  // namespace tbe_in
