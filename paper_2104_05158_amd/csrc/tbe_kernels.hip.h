// Device kernels of the table-batched embedding-bag library for gfx950 (CDNA4, wave64).
//
// Forward: Section 2 "Embedding operators" + Section 5.1 (all tables in one launch).
// Backward: Section 5.1 (gradient sorting by rows, on-chip aggregation, fused optimizer) and
// Section 5.2 (row-wise AdaGrad) of arxiv 2104.05158.
//
// Everything on this path is a gather / scan / sort bound by HBM bandwidth: no MFMA.  The lane
// mapping is the same everywhere: a row of D elements is covered by LPR = pow2ceil(D / EPL) lanes
// (EPL contiguous elements per lane, vector loads), and the 64 / LPR lane groups of a wavefront
// fetch different rows at the same time; sums across groups and across a row use xor-shuffles.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbe {

constexpr int kWave = 64;

// ---- geometry constants shared by host and device ----
constexpr int kFwdThreads = 256;          // 4 wavefronts per workgroup, each with its own block of bags
constexpr int kFwdUnroll = 4;             // row loads in flight per lane group (8 costs occupancy and is slower)
constexpr int kFwdStage = 512;            // indices staged in LDS per wavefront
constexpr int kFwdMaxBagsPerWave = 8;     // measured best on configs 2-4 (4..32 tried)
constexpr int kKeyBags = 256;             // bags per workgroup in the key build
constexpr int kSortThreads = 512;         // 8 wavefronts
constexpr int kSortKeysPerThread = 16;
constexpr int kSortTile = kSortThreads * kSortKeysPerThread;  // 8192 keys staged in LDS
constexpr int kScanThreads = 256;
constexpr int kScanPerThread = 16;
constexpr int kScanTile = kScanThreads * kScanPerThread;      // 4096
constexpr int kRlThreads = 256;
constexpr int kRlPerThread = 16;
constexpr int kRlTile = kRlThreads * kRlPerThread;            // 4096 sorted positions
constexpr int kChunk = 128;               // sorted positions owned by one wavefront in the update
constexpr int kLongRun = 512;             // runs longer than this are split over their chunks
constexpr int kBwdThreads = 256;          // 4 wavefronts = 4 chunks per workgroup
constexpr int kBwdUnroll = 4;             // gradient rows in flight per lane group (long runs)
constexpr int kShortRun = 4;              // runs up to this length are handled one per lane group
constexpr int kMaxDim = 512;

struct TableMeta {      // 32 bytes, one per table, in the workspace head
    int64_t woff;       // first element of the table in the flat weight array
    uint32_t rbase;     // linear id of the table's row 0
    int32_t dim;        // D_t
    int32_t col;        // first output column
    int32_t lpr_fwd;    // log2 lanes per row, forward (EPL elements per lane)
    int32_t lpr_bwd;    // log2 lanes per row, backward (2 x 4 floats per lane)
    int32_t pad;
};

struct Counters {       // workspace scalars
    int64_t num_unique;
    uint32_t long_count;
    uint32_t check_flags;
    uint32_t pad[4];
};

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <typename WT, int EPL>
struct RowIO;

template <>
struct RowIO<float, 4> {
    __device__ static __forceinline__ void load(const float* p, float (&f)[4])
    {
        float4 v = *reinterpret_cast<const float4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static __forceinline__ void store(float* p, const float (&f)[4])
    {
        *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
    }
};

template <>
struct RowIO<__half, 4> {
    __device__ static __forceinline__ void load(const __half* p, float (&f)[4])
    {
        uint2 v = *reinterpret_cast<const uint2*>(p);
        float2 a = __half22float2(*reinterpret_cast<__half2*>(&v.x));
        float2 b = __half22float2(*reinterpret_cast<__half2*>(&v.y));
        f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
    }
    __device__ static __forceinline__ void store(__half* p, const float (&f)[4])
    {
        uint2 v;
        *reinterpret_cast<__half2*>(&v.x) = __floats2half2_rn(f[0], f[1]);
        *reinterpret_cast<__half2*>(&v.y) = __floats2half2_rn(f[2], f[3]);
        *reinterpret_cast<uint2*>(p) = v;
    }
};

template <>
struct RowIO<__half, 8> {
    __device__ static __forceinline__ void load(const __half* p, float (&f)[8])
    {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        float2 a = __half22float2(*reinterpret_cast<__half2*>(&v.x));
        float2 b = __half22float2(*reinterpret_cast<__half2*>(&v.y));
        float2 c = __half22float2(*reinterpret_cast<__half2*>(&v.z));
        float2 d = __half22float2(*reinterpret_cast<__half2*>(&v.w));
        f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
        f[4] = c.x; f[5] = c.y; f[6] = d.x; f[7] = d.y;
    }
};

// ---------------------------------------------------------------- forward (Section 2, Section 5.1)
//
// One launch for all tables.  A wavefront takes a block of consecutive bags (bag id = t*B + b),
// reads their offsets with one coalesced load and stages the block's indices, which are contiguous
// in memory, in wavefront-private LDS.  The bags are then pooled G at a time, one bag per lane
// group (LPR = pow2ceil(D/EPL) lanes x EPL-element vector loads cover a row): every group streams
// its own bag's rows with kFwdUnroll row loads in flight, accumulates in fp32 registers and writes
// its D_t pooled values with one coalesced store -- no cross-group reduction is needed.  Bags of one
// batch always belong to one table, so the lane mapping is uniform inside a batch.
template <typename WT, int EPL, int KMAX>
__global__ __launch_bounds__(kFwdThreads) void forward_kernel(
    const TableMeta* __restrict__ meta, const WT* __restrict__ weights,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    float* __restrict__ out, int32_t B, int32_t num_bags, int32_t sumD, int32_t bags_per_wave)
{
    constexpr int kWaves = kFwdThreads / kWave;
    __shared__ int32_t s_idx_all[kWaves][kFwdStage];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    int32_t* s_idx = s_idx_all[wv];
    const int j0 = uniform((blockIdx.x * kWaves + wv) * bags_per_wave);
    if (j0 >= num_bags)
        return;
    const int nbags = min(bags_per_wave, num_bags - j0);  // <= 63

    const int my_o = lane <= nbags ? (int)offsets[j0 + lane] : 0;
    const int p_begin = __builtin_amdgcn_readlane(my_o, 0);
    const int p_end = __shfl(my_o, nbags);
    const int stage_n = min(p_end - p_begin, kFwdStage);
    for (int i = lane; i < stage_n; i += kWave)
        s_idx[i] = indices[p_begin + i];
    __threadfence_block();
    __builtin_amdgcn_wave_barrier();

    int r = 0;
    while (r < nbags) {
        const int j = j0 + r;
        const int t = j / B;
        const TableMeta m = meta[t];
        const int D = m.dim;
        const int lprl = m.lpr_fwd;
        const int LPR = 1 << lprl;
        const int G = kWave >> lprl;
        const int sub = lane & (LPR - 1);
        const int grp = lane >> lprl;
        const int same_table = (t + 1) * B - j;  // bags from j on that still belong to table t
        const int nb = min(G, min(nbags - r, same_table));
        const bool active = grp < nb;
        const int rr = active ? r + grp : r;
        // both shuffles run with every lane enabled: a bpermute cannot read a disabled lane
        const int start = __shfl(my_o, rr);
        const int next = __shfl(my_o, rr + 1);
        const int len = active ? next - start : 0;
        const WT* __restrict__ wbase = weights + m.woff;

        float acc[KMAX][EPL];
#pragma unroll
        for (int k = 0; k < KMAX; ++k)
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                acc[k][e] = 0.f;

        for (int it = 0; __ballot(it < len) != 0ull; it += kFwdUnroll) {
            float v[kFwdUnroll][KMAX][EPL];
#pragma unroll
            for (int u = 0; u < kFwdUnroll; ++u) {
                const int p = it + u;
                const bool ok = p < len;
                const int rel = start + p - p_begin;
                const int idx = ok ? (rel < stage_n ? s_idx[rel] : indices[start + p]) : 0;
                const WT* rp = wbase + (int64_t)idx * D;
#pragma unroll
                for (int k = 0; k < KMAX; ++k) {
                    const int e0 = (sub + k * LPR) * EPL;
                    if (ok && e0 < D) {
                        RowIO<WT, EPL>::load(rp + e0, v[u][k]);
                    } else {
#pragma unroll
                        for (int e = 0; e < EPL; ++e)
                            v[u][k][e] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kFwdUnroll; ++u)
#pragma unroll
                for (int k = 0; k < KMAX; ++k)
#pragma unroll
                    for (int e = 0; e < EPL; ++e)
                        acc[k][e] += v[u][k][e];
        }

        if (active) {
            const int b = j - t * B + grp;
            float* op = out + (int64_t)b * sumD + m.col;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const int e0 = (sub + k * LPR) * EPL;
                if (e0 < D) {
#pragma unroll
                    for (int q = 0; q < EPL; q += 4)
                        *reinterpret_cast<float4*>(op + e0 + q) =
                            make_float4(acc[k][q], acc[k][q + 1], acc[k][q + 2], acc[k][q + 3]);
                }
            }
        }
        r += nb;
    }
}

// ---------------------------------------------------------------- key build (Section 5.1, "sorting by rows")
//
// key[p] = rbase_t + indices[p] (the row's linear id over all tables), val[p] = b, for every lookup
// position p.  A workgroup takes kKeyBags consecutive bags, keeps their offsets in LDS and walks the
// positions they cover with coalesced loads/stores; the bag of a position is found by bisection in LDS.
__global__ __launch_bounds__(256) void build_keys_kernel(
    const uint32_t* __restrict__ row_base, const int32_t* __restrict__ indices,
    const int64_t* __restrict__ offsets, uint32_t* __restrict__ keys, int32_t* __restrict__ vals,
    int32_t B, int32_t num_bags, Counters* __restrict__ counters)
{
    __shared__ int32_t soff[kKeyBags + 1];
    const int j0 = blockIdx.x * kKeyBags;
    const int nb = min(kKeyBags, num_bags - j0);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        counters->num_unique = 0;
        counters->long_count = 0;
    }
    for (int i = threadIdx.x; i <= nb; i += 256)
        soff[i] = (int32_t)offsets[j0 + i];
    __syncthreads();
    const int lo = soff[0], hi = soff[nb];
    for (int p = lo + threadIdx.x; p < hi; p += 256) {
        int a = 0, c = nb;  // soff[a] <= p < soff[c]
        while (c - a > 1) {
            const int mid = (a + c) >> 1;
            if (soff[mid] <= p)
                a = mid;
            else
                c = mid;
        }
        const int j = j0 + a;
        const int t = j / B;
        keys[p] = row_base[t] + (uint32_t)indices[p];
        vals[p] = j - t * B;
    }
}

// ---------------------------------------------------------------- LSD radix sort (stable), LDS-staged
//
// Per pass: (1) per-tile digit histogram, (2) exclusive scan of the digit-major histogram table,
// (3) scatter: every wavefront ranks its 16 x 64 keys with ballot-based digit matching into per-wave
// LDS counters, the tile is reordered by digit inside LDS and then written out in runs that are
// contiguous in global memory.  Order inside a tile is (wavefront, round, lane) = ascending position,
// so equal digits keep their input order and the whole sort is stable.

__device__ __forceinline__ uint64_t match_digit(uint32_t dg, bool valid, int bits)
{
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
        const bool bit = (dg >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
    }
    return peers;
}

__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(
    const uint32_t* __restrict__ keys, uint32_t* __restrict__ hist, int32_t n, int32_t num_tiles,
    int shift, int bits)
{
    __shared__ uint32_t s_hist[kSortThreads / kWave][256];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int nd = 1 << bits;
    const uint32_t mask = nd - 1;
    for (int i = threadIdx.x; i < (kSortThreads / kWave) * 256; i += kSortThreads)
        (&s_hist[0][0])[i] = 0;
    __syncthreads();
    volatile uint32_t* wh = s_hist[wave];
    const int base = blockIdx.x * kSortTile + wave * (kSortTile / (kSortThreads / kWave));
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll 4
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        const bool valid = q < n;
        const uint32_t dg = valid ? ((keys[q] >> shift) & mask) : 0u;
        const uint64_t peers = match_digit(dg, valid, bits);
        if (valid && (peers & lt) == 0)
            wh[dg] = wh[dg] + (uint32_t)__popcll(peers);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < nd; d += kSortThreads) {
        uint32_t s = 0;
#pragma unroll
        for (int w = 0; w < kSortThreads / kWave; ++w)
            s += s_hist[w][d];
        hist[(int64_t)d * num_tiles + blockIdx.x] = s;
    }
}

__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(
    const uint32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in,
    uint32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out,
    const uint32_t* __restrict__ hist_scanned, int32_t n, int32_t num_tiles, int shift, int bits)
{
    constexpr int kWaves = kSortThreads / kWave;
    __shared__ uint32_t s_keys[kSortTile];
    __shared__ int32_t s_vals[kSortTile];
    __shared__ uint32_t s_whist[kWaves][256];
    __shared__ uint32_t s_dstart[256];
    __shared__ uint32_t s_goff[256];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int nd = 1 << bits;
    const uint32_t mask = nd - 1;
    const int tile = blockIdx.x;
    const int tile_base = tile * kSortTile;
    const int tile_cnt = min(kSortTile, n - tile_base);

    for (int i = threadIdx.x; i < kWaves * 256; i += kSortThreads)
        (&s_whist[0][0])[i] = 0;
    __syncthreads();

    uint32_t key[kSortKeysPerThread];
    int32_t val[kSortKeysPerThread];
    uint32_t rank[kSortKeysPerThread];
    const int base = tile_base + wave * (kSortTile / kWaves);
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        const bool valid = q < n;
        key[r] = valid ? keys_in[q] : 0xffffffffu;
        val[r] = valid ? vals_in[q] : 0;
    }
    volatile uint32_t* wh = s_whist[wave];
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        const bool valid = q < n;
        const uint32_t dg = (key[r] >> shift) & mask;
        const uint64_t peers = match_digit(dg, valid, bits);
        const uint32_t pre = valid ? wh[dg] : 0u;
        const uint32_t below = (uint32_t)__popcll(peers & lt);
        if (valid && below == 0)
            wh[dg] = pre + (uint32_t)__popcll(peers);
        rank[r] = pre + below;
    }
    __syncthreads();

    // per digit: exclusive prefix over the wavefronts, and the tile total
    if ((int)threadIdx.x < nd) {
        uint32_t run = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const uint32_t c = s_whist[w][threadIdx.x];
            s_whist[w][threadIdx.x] = run;
            run += c;
        }
        s_dstart[threadIdx.x] = run;
    }
    __syncthreads();
    // exclusive scan of the (up to 256) digit totals by wavefront 0: 4 digits per lane
    if (wave == 0) {
        uint32_t c[4];
        uint32_t s = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int d = lane * 4 + i;
            c[i] = d < nd ? s_dstart[d] : 0u;
            s += c[i];
        }
        uint32_t incl = s;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o);
            if (lane >= o)
                incl += up;
        }
        uint32_t ex = incl - s;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int d = lane * 4 + i;
            if (d < nd) {
                s_dstart[d] = ex;
                s_goff[d] = hist_scanned[(int64_t)d * num_tiles + tile] - ex;
            }
            ex += c[i];
        }
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        if (q < n) {
            const uint32_t dg = (key[r] >> shift) & mask;
            const uint32_t pos = s_dstart[dg] + s_whist[wave][dg] + rank[r];
            s_keys[pos] = key[r];
            s_vals[pos] = val[r];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortKeysPerThread; ++i) {
        const int p = threadIdx.x + i * kSortThreads;
        if (p < tile_cnt) {
            const uint32_t k = s_keys[p];
            const uint32_t g = s_goff[(k >> shift) & mask] + (uint32_t)p;
            keys_out[g] = k;
            vals_out[g] = s_vals[p];
        }
    }
}

// ---------------------------------------------------------------- device-wide exclusive scan (uint32)

__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* s_wave /*[4]*/,
                                                             uint32_t& block_total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o)
            incl += up;
    }
    if (lane == kWave - 1)
        s_wave[wave] = incl;
    __syncthreads();
    uint32_t woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t c = s_wave[w];
        if (w < wave)
            woff += c;
        tot += c;
    }
    block_total = tot;
    __syncthreads();
    return woff + incl - v;
}

__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(
    const uint32_t* __restrict__ data, uint32_t* __restrict__ block_sums, int64_t n)
{
    __shared__ uint32_t s_wave[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    uint32_t s = 0;
    if (base + kScanPerThread <= n) {
        const uint4* p = reinterpret_cast<const uint4*>(data + base);
#pragma unroll
        for (int i = 0; i < kScanPerThread / 4; ++i) {
            const uint4 v = p[i];
            s += v.x + v.y + v.z + v.w;
        }
    } else {
        for (int i = 0; i < kScanPerThread; ++i)
            if (base + i < n)
                s += data[base + i];
    }
    uint32_t tot;
    (void)block_exclusive_scan_256(s, s_wave, tot);
    if (threadIdx.x == 0)
        block_sums[blockIdx.x] = tot;
}

// single workgroup: exclusive scan of block_sums[nb] in place; optional total (as int64) to *total_out
__global__ __launch_bounds__(kScanThreads) void scan_top_kernel(uint32_t* __restrict__ block_sums,
                                                                int32_t nb, int64_t* total_out)
{
    __shared__ uint32_t s_wave[4];
    uint32_t carry = 0;
    for (int base = 0; base < nb; base += kScanThreads) {
        const int i = base + threadIdx.x;
        const uint32_t v = i < nb ? block_sums[i] : 0u;
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan_256(v, s_wave, tot);
        if (i < nb)
            block_sums[i] = carry + ex;
        carry += tot;
    }
    if (total_out && threadIdx.x == 0)
        *total_out = (int64_t)carry;
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(
    uint32_t* __restrict__ data, const uint32_t* __restrict__ block_sums, int64_t n)
{
    __shared__ uint32_t s_wave[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
    uint32_t v[kScanPerThread];
    const bool full = base + kScanPerThread <= n;
    if (full) {
        const uint4* p = reinterpret_cast<const uint4*>(data + base);
#pragma unroll
        for (int i = 0; i < kScanPerThread / 4; ++i) {
            const uint4 x = p[i];
            v[4 * i] = x.x; v[4 * i + 1] = x.y; v[4 * i + 2] = x.z; v[4 * i + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kScanPerThread; ++i)
            v[i] = base + i < n ? data[base + i] : 0u;
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i)
        s += v[i];
    uint32_t tot;
    uint32_t run = block_exclusive_scan_256(s, s_wave, tot) + block_sums[blockIdx.x];
#pragma unroll
    for (int i = 0; i < kScanPerThread; ++i) {
        const uint32_t c = v[i];
        v[i] = run;
        run += c;
    }
    if (full) {
        uint4* p = reinterpret_cast<uint4*>(data + base);
#pragma unroll
        for (int i = 0; i < kScanPerThread / 4; ++i)
            p[i] = make_uint4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
    } else {
#pragma unroll
        for (int i = 0; i < kScanPerThread; ++i)
            if (base + i < n)
                data[base + i] = v[i];
    }
}

// ---------------------------------------------------------------- run-length segmentation (Section 5.1)
//
// A sorted position q is a run head when q == 0 or key[q] != key[q-1].  Pass 1 counts heads per
// tile, a scan turns the counts into the index of each tile's first run, pass 2 writes
// unique_keys / seg_offsets and, for every kChunk-aligned position, the number of heads before it.

__device__ __forceinline__ void rl_load(const uint32_t* __restrict__ keys, int32_t n, int base,
                                        uint32_t (&k)[kRlPerThread], uint32_t& prev)
{
    if (base + kRlPerThread <= n) {
        const uint4* p = reinterpret_cast<const uint4*>(keys + base);
#pragma unroll
        for (int i = 0; i < kRlPerThread / 4; ++i) {
            const uint4 x = p[i];
            k[4 * i] = x.x; k[4 * i + 1] = x.y; k[4 * i + 2] = x.z; k[4 * i + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kRlPerThread; ++i)
            k[i] = base + i < n ? keys[base + i] : 0u;
    }
    prev = (base > 0 && base < n) ? keys[base - 1] : 0u;
}

__global__ __launch_bounds__(kRlThreads) void runlength_count_kernel(
    const uint32_t* __restrict__ keys, uint32_t* __restrict__ tile_heads, int32_t n)
{
    __shared__ uint32_t s_wave[4];
    const int base = blockIdx.x * kRlTile + threadIdx.x * kRlPerThread;
    uint32_t k[kRlPerThread], prev;
    rl_load(keys, n, base, k, prev);
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < kRlPerThread; ++i) {
        const int q = base + i;
        const bool head = q < n && (q == 0 || k[i] != (i == 0 ? prev : k[i - 1]));
        c += head ? 1u : 0u;
    }
    uint32_t tot;
    (void)block_exclusive_scan_256(c, s_wave, tot);
    if (threadIdx.x == 0)
        tile_heads[blockIdx.x] = tot;
}

__global__ __launch_bounds__(kRlThreads) void runlength_write_kernel(
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ tile_first_run,
    uint32_t* __restrict__ unique_keys, int32_t* __restrict__ seg_offsets,
    int32_t* __restrict__ chunk_first_run, Counters* __restrict__ counters, int32_t n,
    int32_t num_chunks)
{
    __shared__ uint32_t s_wave[4];
    const int base = blockIdx.x * kRlTile + threadIdx.x * kRlPerThread;
    uint32_t k[kRlPerThread], prev;
    rl_load(keys, n, base, k, prev);
    bool head[kRlPerThread];
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < kRlPerThread; ++i) {
        const int q = base + i;
        head[i] = q < n && (q == 0 || k[i] != (i == 0 ? prev : k[i - 1]));
        c += head[i] ? 1u : 0u;
    }
    uint32_t tot;
    uint32_t r = block_exclusive_scan_256(c, s_wave, tot) + tile_first_run[blockIdx.x];
#pragma unroll
    for (int i = 0; i < kRlPerThread; ++i) {
        const int q = base + i;
        if (q < n) {
            if ((q & (kChunk - 1)) == 0)
                chunk_first_run[q / kChunk] = (int32_t)r;
            if (head[i]) {
                unique_keys[r] = k[i];
                seg_offsets[r] = q;
                ++r;
            }
            if (q == n - 1) {
                seg_offsets[r] = n;
                chunk_first_run[num_chunks] = (int32_t)r;
                counters->num_unique = (int64_t)r;
            }
        }
    }
}

// ---------------------------------------------------------------- fused aggregation + row-wise AdaGrad
//
// Section 5.1: all gradients of one row are aggregated on chip and the optimizer runs once per row.
// Section 5.2: m += mean_d(G_d^2); w -= lr * G / (sqrt(m) + eps)  (updated moment, eps outside the root).
//
// Each wavefront owns kChunk consecutive sorted positions and every run that STARTS inside them.
// The chunk's run descriptors and payloads are staged in LDS once.  Lane mapping: a row of D floats
// is covered by LPR = pow2ceil(D/8) lanes, two float4 blocks per lane, so G = 64/LPR rows are
// fetched per load instruction.
//   * runs of at most kShortRun lookups (the vast majority) are handled G at a time, one per lane
//     group: all their gradient rows, weight rows and moments are requested before anything is
//     consumed, the sum stays inside the group, and all groups apply their update together;
//   * longer runs use the whole wavefront (groups take alternate lookups, xor butterfly at the end);
//     up to kLongRun lookups the owner follows the run past its chunk and finishes it;
//   * a run longer than kLongRun is cut at chunk borders: every chunk it touches writes one fp32
//     partial row to the workspace and the run is queued for the fix-up kernel, which adds the
//     partials in chunk order and applies the single update.
// Either way each touched row is read, updated and written exactly once, nothing is accumulated
// with atomics, and the summation order is fixed: results are bit-identical run to run.

__device__ __forceinline__ int find_table(const uint32_t* __restrict__ row_base, int T, uint32_t key)
{
    int a = 0, c = T;  // row_base[a] <= key < row_base[c]
    while (c - a > 1) {
        const int mid = (a + c) >> 1;
        if (row_base[mid] <= key)
            a = mid;
        else
            c = mid;
    }
    return a;
}

struct BwdArgs {
    const TableMeta* meta;
    const uint32_t* row_base;
    const uint32_t* sorted_keys;
    const int32_t* sorted_vals;
    const uint32_t* unique_keys;
    const int32_t* seg_offsets;
    const int32_t* chunk_first_run;
    Counters* counters;
    const float* grad_out;
    void* weights;
    float* moments;
    float* partials;      // [num_chunks][2][dpad]
    uint32_t* long_list;
    int32_t n;
    int32_t num_chunks;
    int32_t T;
    int32_t sumD;
    int32_t dpad;
    float lr;
    float eps;
};

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void acc4(float (&a)[4], const float4 v)
{
    a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w;
}

// Whole-wavefront sum of the fp32 rows rowptr(i), i in [p0, p1).  Afterwards every lane group holds
// the complete sums (lane `sub` of a group: elements (sub + k*LPR)*4 .. +3, k = 0, 1).
template <typename RowPtr>
__device__ __forceinline__ void wave_gather_sum(RowPtr rowptr, int p0, int p1, int D, int lprl, int lane,
                                                float (&acc)[2][4])
{
    const int LPR = 1 << lprl;
    const int G = kWave >> lprl;
    const int sub = lane & (LPR - 1);
    const int grp = lane >> lprl;
    const int e0 = sub * 4, e1 = (sub + LPR) * 4;
    const bool c0 = e0 < D, c1 = e1 < D;
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc[k][e] = 0.f;
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = p0; i0 < p1; i0 += G * kBwdUnroll) {
        float4 v[kBwdUnroll][2];
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            const int i = i0 + u * G + grp;
            const bool ok = i < p1;
            const float* rp = rowptr(ok ? i : p0);
            v[u][0] = (ok && c0) ? ld4(rp + e0) : z;
            v[u][1] = (ok && c1) ? ld4(rp + e1) : z;
        }
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            acc4(acc[0], v[u][0]);
            acc4(acc[1], v[u][1]);
        }
    }
    for (int s = LPR; s < kWave; s <<= 1) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[k][e] += __shfl_xor(acc[k][e], s);
    }
}

// The AdaGrad epilogue for the row held by this lane's group (w: the row's old values, already loaded).
template <typename WT>
__device__ __forceinline__ void adagrad_epilogue(WT* __restrict__ wrow, float* __restrict__ mptr, float m_old,
                                                 float (&w)[2][4], const float (&acc)[2][4], int D, int lprl,
                                                 int lane, bool writer, float lr, float eps)
{
    const int LPR = 1 << lprl;
    const int sub = lane & (LPR - 1);
    const int e0 = sub * 4, e1 = (sub + LPR) * 4;
    float ss = 0.f;
    if (e0 < D)
        ss += acc[0][0] * acc[0][0] + acc[0][1] * acc[0][1] + acc[0][2] * acc[0][2] + acc[0][3] * acc[0][3];
    if (e1 < D)
        ss += acc[1][0] * acc[1][0] + acc[1][1] * acc[1][1] + acc[1][2] * acc[1][2] + acc[1][3] * acc[1][3];
    for (int s = 1; s < LPR; s <<= 1)
        ss += __shfl_xor(ss, s);
    const float m_new = m_old + ss / (float)D;
    const float scale = lr / (sqrtf(m_new) + eps);
    if (writer) {
        if (e0 < D) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[0][e] -= scale * acc[0][e];
            RowIO<WT, 4>::store(wrow + e0, w[0]);
        }
        if (e1 < D) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[1][e] -= scale * acc[1][e];
            RowIO<WT, 4>::store(wrow + e1, w[1]);
        }
        if (sub == 0)
            *mptr = m_new;
    }
}

template <typename WT>
__device__ __forceinline__ void load_row(const WT* __restrict__ wrow, int D, int lprl, int lane, bool active,
                                         float (&w)[2][4])
{
    const int LPR = 1 << lprl;
    const int sub = lane & (LPR - 1);
    const int e0 = sub * 4, e1 = (sub + LPR) * 4;
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[k][e] = 0.f;
    if (active && e0 < D)
        RowIO<WT, 4>::load(wrow + e0, w[0]);
    if (active && e1 < D)
        RowIO<WT, 4>::load(wrow + e1, w[1]);
}

__device__ __forceinline__ void store_partial(float* __restrict__ dst, const float (&acc)[2][4], int D, int lprl,
                                              int lane)
{
    const int LPR = 1 << lprl;
    const int sub = lane & (LPR - 1);
    if ((lane >> lprl) == 0) {
        if (sub * 4 < D)
            *reinterpret_cast<float4*>(dst + sub * 4) = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
        if ((sub + LPR) * 4 < D)
            *reinterpret_cast<float4*>(dst + (sub + LPR) * 4) =
                make_float4(acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
    }
}

template <typename WT>
__global__ __launch_bounds__(kBwdThreads) void reduce_update_kernel(BwdArgs a)
{
    constexpr int kWaves = kBwdThreads / kWave;
    __shared__ int32_t s_seg_all[kWaves][kChunk + 2];
    __shared__ uint32_t s_key_all[kWaves][kChunk + 1];
    __shared__ int32_t s_val_all[kWaves][kChunk];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    const int k = uniform(blockIdx.x * kWaves + wv);
    if (k >= a.num_chunks)
        return;
    int32_t* s_seg = s_seg_all[wv];
    uint32_t* s_key = s_key_all[wv];
    int32_t* s_val = s_val_all[wv];

    const int q0 = k * kChunk;
    const int q1 = min(a.n, q0 + kChunk);
    const int ub = a.chunk_first_run[k];
    const int ue = a.chunk_first_run[k + 1];
    const int U = (int)a.counters->num_unique;
    const int nruns = ue - ub;  // runs that start in [q0, q1): at most kChunk
    WT* __restrict__ weights = static_cast<WT*>(a.weights);
    const int32_t* __restrict__ vals = a.sorted_vals;
    const int64_t sumD = a.sumD;

    // stage the chunk's run descriptors and payloads (wavefront-private LDS)
    for (int i = lane; i <= nruns; i += kWave)
        s_seg[i] = a.seg_offsets[ub + i];
    for (int i = lane; i < nruns; i += kWave)
        s_key[i] = a.unique_keys[ub + i];
    for (int i = lane; i < q1 - q0; i += kWave)
        s_val[i] = vals[q0 + i];
    __threadfence_block();
    __builtin_amdgcn_wave_barrier();

    float acc[2][4];
    float w[2][4];
    int t = -1;
    uint32_t t_lo = 1u, t_hi = 0u;  // empty range: first key always seeks
    TableMeta m;
    m.woff = 0; m.rbase = 0; m.dim = 4; m.col = 0; m.lpr_fwd = 0; m.lpr_bwd = 0; m.pad = 0;
    auto seek_table = [&](uint32_t key) {
        if (key < t_lo || key >= t_hi) {
            t = find_table(a.row_base, a.T, key);
            m = a.meta[t];
            t_lo = a.row_base[t];
            t_hi = a.row_base[t + 1];
        }
    };
    auto payload = [&](int p) { return p < q1 ? s_val[p - q0] : vals[p]; };

    // the run that is already open at q0: only its long form leaves work here
    const bool incoming = (ub >= U) || (a.seg_offsets[ub] > q0);
    if (incoming) {
        const int u0 = ub - 1;
        const int s0 = a.seg_offsets[u0];
        const int e0 = a.seg_offsets[u0 + 1];
        if (e0 - s0 > kLongRun) {
            seek_table(a.unique_keys[u0]);
            const float* gb = a.grad_out + m.col;
            wave_gather_sum([&](int i) { return gb + (int64_t)payload(i) * sumD; }, q0, min(e0, q1), m.dim,
                            m.lpr_bwd, lane, acc);
            store_partial(a.partials + ((int64_t)k * 2 + 0) * a.dpad, acc, m.dim, m.lpr_bwd, lane);
        }
    }

    int r = 0;
    while (r < nruns) {
        const uint32_t key0 = (uint32_t)uniform((int)s_key[r]);
        seek_table(key0);
        const int D = m.dim;
        const int lprl = m.lpr_bwd;
        const int s0 = uniform(s_seg[r]);
        const int len0 = uniform(s_seg[r + 1]) - s0;
        const float* gb = a.grad_out + m.col;
        WT* wtab = weights + m.woff;
        if (len0 > kShortRun) {
            // ---- one run, whole wavefront
            WT* wrow = wtab + (int64_t)(key0 - m.rbase) * D;
            const bool is_long = len0 > kLongRun;
            const bool writer = (lane >> lprl) == 0;
            float m_old = 0.f;
            if (!is_long) {
                load_row<WT>(wrow, D, lprl, lane, writer, w);
                m_old = a.moments[key0];
            }
            const int e = is_long ? q1 : s0 + len0;
            wave_gather_sum([&](int i) { return gb + (int64_t)payload(i) * sumD; }, s0, e, D, lprl, lane, acc);
            if (!is_long) {
                adagrad_epilogue<WT>(wrow, a.moments + key0, m_old, w, acc, D, lprl, lane, writer, a.lr, a.eps);
            } else {
                store_partial(a.partials + ((int64_t)k * 2 + 1) * a.dpad, acc, D, lprl, lane);
                if (lane == 0) {
                    const uint32_t slot = atomicAdd(&a.counters->long_count, 1u);
                    a.long_list[slot] = (uint32_t)(ub + r);
                }
            }
            r += 1;
        } else {
            // ---- up to G short runs of this table at once, one per lane group
            const int LPR = 1 << lprl;
            const int sub = lane & (LPR - 1);
            const int grp = lane >> lprl;
            const int rr = r + grp;
            const bool in_chunk = rr < nruns;
            const uint32_t key = in_chunk ? s_key[rr] : 0u;
            const int s = in_chunk ? s_seg[rr] : 0;
            const int len = in_chunk ? s_seg[rr + 1] - s : 0;
            const bool fits = in_chunk && key < t_hi && len <= kShortRun;
            const uint64_t bad = __ballot(!fits);
            const int first_bad = bad ? (int)__builtin_ctzll(bad) : kWave;
            const int nb = first_bad >> lprl;  // >= 1: run r itself fits
            const bool active = grp < nb;

            WT* wrow = wtab + (int64_t)(key - m.rbase) * D;
            load_row<WT>(wrow, D, lprl, lane, active, w);
            const float m_old = active ? a.moments[key] : 0.f;
            const int e0 = sub * 4, e1 = (sub + LPR) * 4;
            const bool c0 = e0 < D, c1 = e1 < D;
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            float4 v[kShortRun][2];
#pragma unroll
            for (int u = 0; u < kShortRun; ++u) {
                const bool ok = active && u < len;
                const float* rp = gb + (int64_t)(ok ? payload(s + u) : 0) * sumD;
                v[u][0] = (ok && c0) ? ld4(rp + e0) : z;
                v[u][1] = (ok && c1) ? ld4(rp + e1) : z;
            }
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc[kk][e] = 0.f;
#pragma unroll
            for (int u = 0; u < kShortRun; ++u) {
                acc4(acc[0], v[u][0]);
                acc4(acc[1], v[u][1]);
            }
            adagrad_epilogue<WT>(wrow, a.moments + key, m_old, w, acc, D, lprl, lane, active, a.lr, a.eps);
            r += nb;
        }
    }
}

// One wavefront per queued long run: adds the per-chunk partial rows in chunk order (first the
// piece written by the chunk where the run starts, then one piece per following chunk) and applies
// the run's single AdaGrad step.
template <typename WT>
__global__ __launch_bounds__(kBwdThreads) void long_run_fixup_kernel(BwdArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_global = uniform(blockIdx.x * (kBwdThreads / kWave) + (threadIdx.x >> 6));
    const int wave_total = gridDim.x * (kBwdThreads / kWave);
    const int cnt = (int)a.counters->long_count;
    WT* __restrict__ weights = static_cast<WT*>(a.weights);
    float acc[2][4];
    float w[2][4];
    for (int i = wave_global; i < cnt; i += wave_total) {
        const int u = (int)a.long_list[i];
        const int s = a.seg_offsets[u];
        const int e = a.seg_offsets[u + 1];
        const uint32_t key = a.unique_keys[u];
        const int t = find_table(a.row_base, a.T, key);
        const TableMeta m = a.meta[t];
        const int k0 = s / kChunk;
        const int k1 = (e - 1) / kChunk;
        const float* pbase = a.partials;
        const int64_t dpad = a.dpad;
        WT* wrow = weights + m.woff + (int64_t)(key - m.rbase) * m.dim;
        const bool writer = (lane >> m.lpr_bwd) == 0;
        load_row<WT>(wrow, m.dim, m.lpr_bwd, lane, writer, w);
        const float m_old = a.moments[key];
        wave_gather_sum([&](int c) { return pbase + ((int64_t)(k0 + c) * 2 + (c == 0 ? 1 : 0)) * dpad; }, 0,
                        k1 - k0 + 1, m.dim, m.lpr_bwd, lane, acc);
        adagrad_epilogue<WT>(wrow, a.moments + key, m_old, w, acc, m.dim, m.lpr_bwd, lane, writer, a.lr, a.eps);
    }
}

// ---------------------------------------------------------------- input validation (slow path)

__global__ __launch_bounds__(256) void check_inputs_kernel(
    const TableMeta* __restrict__ meta, const uint32_t* __restrict__ row_base,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets, int64_t num_indices,
    int32_t B, int32_t num_bags, Counters* __restrict__ counters)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= num_bags)
        return;
    uint32_t flags = 0;
    const int64_t lo = offsets[j], hi = offsets[j + 1];
    if ((j == 0 && lo != 0) || (j == num_bags - 1 && hi != num_indices) || lo > hi || lo < 0 ||
        hi > num_indices) {
        flags |= 1u;
    } else {
        const int t = j / B;
        const int64_t H = (int64_t)row_base[t + 1] - (int64_t)row_base[t];
        for (int64_t p = lo; p < hi; ++p) {
            const int64_t r = indices[p];
            if (r < 0 || r >= H)
                flags |= 2u;
        }
    }
    (void)meta;
    if (flags)
        atomicOr(&counters->check_flags, flags);
}

__global__ void clear_counters_kernel(Counters* counters)
{
    counters->num_unique = 0;
    counters->long_count = 0;
    counters->check_flags = 0;
}

}  // namespace tbe
