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

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbe {

constexpr int kWave = 64;

// ---- geometry constants shared by host and device ----
constexpr int kFwdThreads = 256;          // 4 wavefronts per workgroup, each with its own block of bags
constexpr int kFwdUnroll = 4;             // row loads in flight per lane group (8 costs occupancy and is slower)
constexpr int kFwdMaxBagsPerWave = 8;     // measured best on configs 2-4 (4..32 tried)
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
constexpr int kLongRun = 512;             // runs longer than this are summed in pieces by other kernels (window / dense path)
constexpr int kWinMax = 16;               // most bag windows a long run is cut into
constexpr int kWinBatch = 8;               // pieces a workgroup of window_runs_kernel claims at a time
constexpr int kBwdThreads = 256;          // 4 wavefronts = 4 chunks per workgroup
constexpr int kBwdUnroll = 4;             // gradient rows in flight per lane group (long runs)
constexpr int kShortRun = 4;              // runs up to this length are handled one per lane group
constexpr int kMaxDim = 512;
// dense hot rows: runs longer than the call's dense threshold are summed as (count matrix) x (gradient block)
constexpr int kDenseRows = 32;            // most runs per group: they share one pass over the table's gradient block
constexpr int kDenseSlice = 1024;         // bags per work unit = per count table in LDS = per partial row of a dense run
constexpr int kDenseThreads = 256;
constexpr int kDenseMinRun = 1024;        // no run of this length or less is ever treated as dense (> kLongRun)
constexpr int kZeroRowBytes = 4096;        // a row of zeros in the workspace (largest row: 512 x fp32 = 2 KiB)

struct TableMeta {      // 32 bytes, one per table, in the workspace head
    int64_t woff;       // first element of the table in the flat weight array
    uint32_t rbase;     // linear id of the table's row 0
    int32_t dim;        // D_t
    int32_t col;        // first output column
    int32_t lpr_fwd;    // log2 lanes per row, forward (EPL elements per lane)
    int32_t lpr_bwd;    // log2 lanes per row, backward (2 x 4 floats per lane)
    int32_t key_bits;   // ceil(log2 rows) (at least 1): the bits of the table's row index that the sort orders
};

struct Counters {       // workspace scalars
    int64_t num_unique;         // written by the run-length pass of every sort
    // Number of long runs queued by the update kernel for the fix-up kernel.  Zero between update
    // launches: the last workgroup of the fix-up kernel to finish clears it (and fixup_done), so every
    // update starts from an empty queue -- also a second update after one sort, and every replay of a
    // captured graph.
    uint32_t long_count;
    uint32_t fixup_done;        // workgroups of the running fix-up kernel that have finished
    uint32_t check_flags;       // written only by tbe_check_inputs
    uint32_t dense_runs;        // written by the plan kernels: dense runs / groups, windowed runs of this update
    uint32_t dense_groups;
    uint32_t win_runs;          // windowed runs / their pieces of this update (written by window_plan_kernel)
    uint32_t win_pieces;
    uint32_t pad1[23];          // (the claim counters below start a 128-byte line of their own)
    // window_runs_kernel: next unclaimed piece of each L2 domain, one counter per 128-byte line
    // (cleared by the kernel's plan kernel)
    uint32_t win_next[8][32];
};

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// fp16 -> fp32 accumulate as one mixed-precision FMA: x*1 + a is exactly a + x
__device__ __forceinline__ float acc_half(float a, __half h) { return __builtin_fmaf(__half2float(h), 1.0f, a); }

// Row access in the storage type: Vec is the raw vector one lane loads (EPL elements); `add`
// converts to fp32 and accumulates.  Loads are kept raw until they are consumed so that many can
// be in flight with few registers.
template <typename WT, int EPL>
struct RowIO;

template <>
struct RowIO<float, 4> {
    using Vec = float4;
    __device__ static __forceinline__ Vec ldv(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ static __forceinline__ void add(float (&a)[4], const Vec v)
    {
        a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w;
    }
    __device__ static __forceinline__ void unpack(const Vec v, float (&f)[4])
    {
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ static __forceinline__ void store(float* p, const float (&f)[4])
    {
        *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
    }
};

template <>
struct RowIO<__half, 4> {
    using Vec = uint2;
    __device__ static __forceinline__ Vec ldv(const __half* p) { return *reinterpret_cast<const uint2*>(p); }
    __device__ static __forceinline__ void unpack(Vec v, float (&f)[4])
    {
        const float2 a = __half22float2(*reinterpret_cast<__half2*>(&v.x));
        const float2 b = __half22float2(*reinterpret_cast<__half2*>(&v.y));
        f[0] = a.x; f[1] = a.y; f[2] = b.x; f[3] = b.y;
    }
    __device__ static __forceinline__ void add(float (&a)[4], Vec v)
    {
        const __half2 x = *reinterpret_cast<__half2*>(&v.x);
        const __half2 y = *reinterpret_cast<__half2*>(&v.y);
        a[0] = acc_half(a[0], __low2half(x)); a[1] = acc_half(a[1], __high2half(x));
        a[2] = acc_half(a[2], __low2half(y)); a[3] = acc_half(a[3], __high2half(y));
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
    using Vec = uint4;
    __device__ static __forceinline__ Vec ldv(const __half* p) { return *reinterpret_cast<const uint4*>(p); }
    __device__ static __forceinline__ void add(float (&a)[8], Vec v)
    {
        const __half2 x = *reinterpret_cast<__half2*>(&v.x);
        const __half2 y = *reinterpret_cast<__half2*>(&v.y);
        const __half2 z = *reinterpret_cast<__half2*>(&v.z);
        const __half2 w = *reinterpret_cast<__half2*>(&v.w);
        a[0] = acc_half(a[0], __low2half(x)); a[1] = acc_half(a[1], __high2half(x));
        a[2] = acc_half(a[2], __low2half(y)); a[3] = acc_half(a[3], __high2half(y));
        a[4] = acc_half(a[4], __low2half(z)); a[5] = acc_half(a[5], __high2half(z));
        a[6] = acc_half(a[6], __low2half(w)); a[7] = acc_half(a[7], __high2half(w));
    }
};

// ---------------------------------------------------------------- read-rate probe
//
// Streams n16 16-byte words through the chip `passes` times and discards them: the denominator for the
// gather kernels (what plain coalesced reads reach on the machine at hand, from HBM or, for a buffer that fits
// the memory-side cache, from there).  Four loads in flight per thread; an opaque copy of the pointer per pass
// keeps the passes from being merged; the sink is written only for one xor value in 2^32 (a vector store).
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* p, size_t n16, int passes, uint32_t* sink)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    for (int ps = 0; ps < passes; ++ps) {
        // every pass gives a workgroup another part of the buffer (and another L2): a buffer larger than the
        // L2s is read from the level behind them in every pass, not from the workgroup's own lines
        const unsigned vb = (blockIdx.x + (unsigned)ps * 2731u) % gridDim.x;
        size_t i = (size_t)vb * 256 + threadIdx.x;
        for (; i + 3 * stride < n16; i += 4 * stride) {
            const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
            acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
        }
        for (; i < n16; i += stride) {
            const uint4 a = p[i];
            acc ^= a.x ^ a.y ^ a.z ^ a.w;
        }
        asm volatile("" : "+s"(p)::"memory");      // the next pass reads through a pointer the compiler cannot relate to this one
    }
    if (acc == 0x9e3779b9u)
        *sink = acc;
}

// ---------------------------------------------------------------- forward (Section 2, Section 5.1)
//
// One launch for all tables.  A wavefront takes a block of consecutive bags (bag id = t*B + b) and
// reads their offsets with one coalesced load.  The bags are pooled G at a time, one bag per lane
// group (LPR = pow2ceil(D/EPL) lanes x EPL-element vector loads cover a row): every group streams
// its own bag's rows with kFwdUnroll row loads in flight, accumulates in fp32 registers and writes
// its D_t pooled values with one coalesced store -- no cross-group reduction is needed.  Bags of one
// batch always belong to one table, so the lane mapping is uniform inside a batch.
//
// The inner loop is branch-free so that all loads of a step are issued back to back: slots past the
// end of a bag read a row of zeros kept in the workspace (pointer select instead of a predicated
// load), column offsets past D are clamped (those lanes never store), and the indices of the next
// step are requested before the rows of the current step are consumed.
// 4 pooled values in the output type OT (float, or __half rounded to nearest even)
__device__ __forceinline__ void store_out4(float* p, float a, float b, float c, float d)
{
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store_out4(__half* p, float a, float b, float c, float d)
{
    uint2 v;
    *reinterpret_cast<__half2*>(&v.x) = __floats2half2_rn(a, b);
    *reinterpret_cast<__half2*>(&v.y) = __floats2half2_rn(c, d);
    *reinterpret_cast<uint2*>(p) = v;
}

template <typename WT, int EPL, int KMAX, typename OT>
__global__ __launch_bounds__(kFwdThreads) void forward_kernel(
    const TableMeta* __restrict__ meta, const WT* __restrict__ weights,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    OT* __restrict__ out, const void* __restrict__ zero_row, int32_t B, int32_t num_bags,
    int32_t sumD, int32_t n_total, int32_t bags_per_wave, int32_t table_major)
{
    using IO = RowIO<WT, EPL>;
    using Vec = typename IO::Vec;
    constexpr int kWaves = kFwdThreads / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    const int j0 = uniform((blockIdx.x * kWaves + wv) * bags_per_wave);
    if (j0 >= num_bags)
        return;
    const int nbags = min(bags_per_wave, num_bags - j0);  // <= 63

    const int my_o = (int)offsets[j0 + min(lane, nbags)];
    const uint32_t last = (uint32_t)(n_total - 1);
    const WT* __restrict__ zrow = static_cast<const WT*>(zero_row);

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

        int eoff[KMAX];
        bool evalid[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int e0 = (sub + k * LPR) * EPL;
            evalid[k] = e0 < D;
            eoff[k] = min(e0, D - EPL);
        }
        // fp32 tables: one accumulator per load slot, added pairwise at the end -- the rounding error of a
        // long bag grows with the number of terms each accumulator sees.  (Sums of fp16 values in fp32 are
        // exact for thousands of terms: one accumulator.)
        static_assert(kFwdUnroll == 4, "the four accumulators of an fp32 table are added pairwise below");
        constexpr int NACC = sizeof(WT) == 4 ? kFwdUnroll : 1;
        float accs[NACC][KMAX][EPL];
#pragma unroll
        for (int q = 0; q < NACC; ++q)
#pragma unroll
            for (int k = 0; k < KMAX; ++k)
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    accs[q][k][e] = 0.f;

        if (__ballot(len > 0) != 0ull && LPR >= kFwdUnroll) {
            // The address unit spends as long on a 4-byte load as on a 16-byte one, so the indices are not
            // loaded once per row: the LPR lanes of a group load the bag's next LPR indices with ONE
            // instruction (lane `sub` the sub-th of them) a block ahead of their use, and every row load
            // takes its index from the group's lanes by a shuffle.
            const int gbase = lane & ~(LPR - 1);
            int cur = 0;
            int nxt = indices[min((uint32_t)(start + sub), last)];
            for (int it = 0; __ballot(it < len) != 0ull; it += kFwdUnroll) {
                if ((it & (LPR - 1)) == 0) {
                    cur = nxt;
                    nxt = indices[min((uint32_t)(start + it + LPR + sub), last)];
                }
                Vec raw[kFwdUnroll][KMAX];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) {
                    const int idx = __shfl(cur, gbase | ((it + u) & (LPR - 1)));
                    const WT* rp = (it + u < len) ? wbase + (int64_t)idx * D : zrow;
#pragma unroll
                    for (int k = 0; k < KMAX; ++k)
                        raw[u][k] = IO::ldv(rp + eoff[k]);
                }
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u)
#pragma unroll
                    for (int k = 0; k < KMAX; ++k)
                        IO::add(accs[u % NACC][k], raw[u][k]);
            }
        } else if (__ballot(len > 0) != 0ull) {
            // rows of one or two lanes: every lane loads its own indices
            int idx[kFwdUnroll];
#pragma unroll
            for (int u = 0; u < kFwdUnroll; ++u)
                idx[u] = indices[min((uint32_t)(start + u), last)];
            for (int it = 0; __ballot(it < len) != 0ull; it += kFwdUnroll) {
                Vec raw[kFwdUnroll][KMAX];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u) {
                    const WT* rp = (it + u < len) ? wbase + (int64_t)idx[u] * D : zrow;
#pragma unroll
                    for (int k = 0; k < KMAX; ++k)
                        raw[u][k] = IO::ldv(rp + eoff[k]);
                }
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u)
                    idx[u] = indices[min((uint32_t)(start + it + kFwdUnroll + u), last)];
#pragma unroll
                for (int u = 0; u < kFwdUnroll; ++u)
#pragma unroll
                    for (int k = 0; k < KMAX; ++k)
                        IO::add(accs[u % NACC][k], raw[u][k]);
            }
        }
        float acc[KMAX][EPL];
#pragma unroll
        for (int k = 0; k < KMAX; ++k)
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                if (NACC == 4)
                    acc[k][e] = (accs[0][k][e] + accs[1 % NACC][k][e]) + (accs[2 % NACC][k][e] + accs[3 % NACC][k][e]);
                else
                    acc[k][e] = accs[0][k][e];
            }

        if (active) {
            const int b = j - t * B + grp;
            // batch-major: row b of [B, sumD] at column col; table-major: row b of the table's own [B, D] block
            OT* op = table_major ? out + (int64_t)B * m.col + (int64_t)b * D : out + (int64_t)b * sumD + m.col;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                if (evalid[k]) {
#pragma unroll
                    for (int q = 0; q < EPL; q += 4)
                        store_out4(op + eoff[k] + q, acc[k][q], acc[k][q + 1], acc[k][q + 2], acc[k][q + 3]);
                }
            }
        }
        r += nb;
    }
}

// ---------------------------------------------------------------- workgroup scan helper (256 threads)

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

// ---------------------------------------------------------------- sort by (table, row)  (Section 5.1, "sorting by rows")
//
// The input is table-major, so the lookups of table t already occupy one contiguous range of
// positions: sorting by (table, row) is a SEGMENTED sort in which every table is sorted by its own
// row index.  That needs only ceil(log2 max_t H_t) key bits instead of ceil(log2 sum_t H_t), the first
// pass can read the caller's indices directly as keys (the payload b, the bag's position inside its
// table's batch, is derived from the offsets on the fly), and the last pass adds the table's row base
// so that the result is sorted by the linear row id.
//
// Tiles of kSortTile positions never cross a table border.  A small plan (two launches) turns the
// table borders offsets[t*B] into: the first tile of every table, the first position of every
// table, and the table of every tile.  The per-tile digit histograms are laid out table by table,
// digit-major inside a table: hist[tile_base[t]*nd + d*ntiles_t + local_tile].  One exclusive scan
// over the whole array then yields global output positions, because every table's counts add up to
// exactly its number of lookups.
//
// Every table is sorted over its own ceil(log2 H_t) index bits in ceil(bits / 8) passes of equal-as-possible
// digit widths.  A launch serves all tables; a table that needs fewer passes than the tallest one sits out
// the first launches (its tiles report all their keys under digit 0, so the scan still yields global
// positions, and move nothing) and makes its first pass -- the one that reads the caller's indices -- later,
// so that every table finishes in the same launch and in the same buffer.
//
// Per pass: (1) per-tile digit histogram, (2) the scan, (3) scatter: every wavefront ranks its
// 16 x 64 keys with ballot-based digit matching into per-wave LDS counters, the tile is reordered by
// digit inside LDS and then written out in runs that are contiguous in global memory.  Order inside
// a tile is (wavefront, round, lane) = ascending position, so equal digits keep their input order
// and the whole sort is stable.

struct TileDesc {        // 32 bytes: everything a workgroup needs to know about its tile, in one load
    int32_t t;           // table, -1 past the last tile
    int32_t first;       // first position of the tile
    int32_t cnt;         // positions in the tile (1..kSortTile)
    int32_t hstride;     // tiles of the table = distance between consecutive digits in the histogram
    int32_t tbase;       // first tile of the table
    int32_t local;       // index of the tile inside its table
    int32_t bag_lo;      // bag (inside the table's batch) of the tile's first position ...
    int32_t bag_hi;      // ... and of its last one
};

struct SortPlan {
    const int32_t* tile_base;    // [T+1] first tile of table t; [T] = number of tiles
    const int32_t* tstart;       // [T+1] first position of table t; [T] = n
    const TileDesc* tiles;       // [max_tiles]
};

// one workgroup: table borders -> tile_base / tstart; also clears the per-call counters
__global__ __launch_bounds__(256) void sort_plan_tables_kernel(const int64_t* __restrict__ offsets, int32_t B,
                                                               int32_t T, int32_t* __restrict__ tile_base,
                                                               int32_t* __restrict__ tstart,
                                                               Counters* __restrict__ counters)
{
    __shared__ uint32_t s_wave[4];
    if (threadIdx.x == 0)
        counters->num_unique = 0;
    uint32_t carry = 0;
    for (int base = 0; base < T; base += 256) {
        const int t = base + threadIdx.x;
        int32_t lo = 0, cnt = 0;
        if (t < T) {
            lo = (int32_t)offsets[(int64_t)t * B];
            cnt = (int32_t)offsets[(int64_t)(t + 1) * B] - lo;
        }
        const uint32_t tiles = (uint32_t)((cnt + kSortTile - 1) / kSortTile);
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan_256(tiles, s_wave, tot);
        if (t < T) {
            tile_base[t] = (int32_t)(carry + ex);
            tstart[t] = lo;
        }
        carry += tot;
    }
    if (threadIdx.x == 0) {
        tile_base[T] = (int32_t)carry;
        tstart[T] = (int32_t)offsets[(int64_t)T * B];
    }
}

// last bag b in [0, B) of table t with offsets[t*B + b] <= q
__device__ __forceinline__ int bag_of_position(const int64_t* __restrict__ offsets, int64_t j0, int B, int64_t q)
{
    int a = 0, c = B;
    while (c - a > 1) {
        const int mid = (a + c) >> 1;
        if (offsets[j0 + mid] <= q)
            a = mid;
        else
            c = mid;
    }
    return a;
}

__global__ __launch_bounds__(256) void sort_plan_tiles_kernel(const int32_t* __restrict__ tile_base,
                                                              const int32_t* __restrict__ tstart,
                                                              const int64_t* __restrict__ offsets, int32_t B,
                                                              int32_t T, TileDesc* __restrict__ tiles,
                                                              int32_t max_tiles)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= max_tiles)
        return;
    TileDesc d;
    d.t = -1; d.first = 0; d.cnt = 0; d.hstride = 0; d.tbase = 0; d.local = 0; d.bag_lo = d.bag_hi = 0;
    if (g < tile_base[T]) {
        int a = 0, c = T;  // last a in [0, T) with tile_base[a] <= g
        while (c - a > 1) {
            const int mid = (a + c) >> 1;
            if (tile_base[mid] <= g)
                a = mid;
            else
                c = mid;
        }
        const int tb = tile_base[a];
        d.t = a;
        d.tbase = tb;
        d.local = g - tb;
        d.first = tstart[a] + d.local * kSortTile;
        d.cnt = min(kSortTile, tstart[a + 1] - d.first);
        d.hstride = tile_base[a + 1] - tb;
        d.bag_lo = bag_of_position(offsets, (int64_t)a * B, B, d.first);
        d.bag_hi = bag_of_position(offsets, (int64_t)a * B, B, d.first + d.cnt - 1);
    }
    tiles[g] = d;
}

struct TileGeom {
    int t;          // table
    int first;      // first position of the tile
    int cnt;        // positions in the tile (1..kSortTile)
    int64_t hbase;  // index of this tile's digit-0 histogram entry
    int hstride;    // distance between consecutive digits (tiles of the table)
};

__device__ __forceinline__ bool tile_geom(const SortPlan& pl, int g, int nd, TileGeom& tg)
{
    const int4 a = *reinterpret_cast<const int4*>(&pl.tiles[g]);            // t, first, cnt, hstride
    const int2 b = *reinterpret_cast<const int2*>(&pl.tiles[g].tbase);      // tbase, local
    if (a.x < 0)
        return false;
    tg.t = a.x;
    tg.first = a.y;
    tg.cnt = a.z;
    tg.hstride = a.w;
    tg.hbase = (int64_t)b.x * nd + b.y;
    return true;
}

// Where table t stands in launch p of P: P_t = ceil(bits / 8) passes, the last P_t launches; pass lp orders
// `width` bits starting at `shift` (the bits are split as evenly as possible, wider digits first).
struct PassGeom {
    bool active;     // the table takes part in this launch
    bool first;      // this is the table's first pass: keys come from the caller's indices
    int shift, width;
};

__device__ __forceinline__ PassGeom pass_geom(int key_bits, int p, int P)
{
    const int pt = (key_bits + 7) >> 3;
    const int lp = p - (P - pt);
    PassGeom g;
    g.active = lp >= 0;
    g.first = lp == 0;
    const int q = key_bits / pt, rem = key_bits - q * pt;
    const int l = max(lp, 0);
    g.width = q + (l < rem ? 1 : 0);
    g.shift = l * q + min(l, rem);
    return g;
}

// Lanes of the wavefront whose digit equals this lane's (valid lanes only).  Bit b of every lane is
// broadcast by a ballot; a lane keeps the lanes whose bit agrees with its own.  The loop is unrolled
// for the largest digit width with a uniform guard, so no bit position costs a loop iteration.
__device__ __forceinline__ uint64_t match_digit(uint32_t dg, bool valid, int bits)
{
    uint32_t lo, hi;
    {
        const uint64_t v = __ballot(valid);
        lo = (uint32_t)v;
        hi = (uint32_t)(v >> 32);
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        if (b < bits) {
            const uint32_t m = (uint32_t)(((int32_t)(dg << (31 - b))) >> 31);   // all ones if bit b is set
            const uint64_t bal = __ballot(m != 0u);
            // lanes whose bit differs from mine drop out: peers &= ~(bal ^ m)
            lo &= ~((uint32_t)bal ^ m);
            hi &= ~((uint32_t)(bal >> 32) ^ m);
        }
    }
    return ((uint64_t)hi << 32) | lo;
}

__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(
    SortPlan pl, const TableMeta* __restrict__ meta, const uint32_t* __restrict__ keys_cur,
    const uint32_t* __restrict__ indices, uint32_t* __restrict__ hist, int p, int P, int nd_bits)
{
    __shared__ uint32_t s_hist[256];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int nd = 1 << nd_bits;
    TileGeom tg;
    if (!tile_geom(pl, blockIdx.x, nd, tg))
        return;
    const PassGeom pg = pass_geom(meta[tg.t].key_bits, p, P);
    if (!pg.active) {
        // the table sits this launch out: all its keys count under digit 0
        if ((int)threadIdx.x < nd)
            hist[tg.hbase + (int64_t)threadIdx.x * tg.hstride] = threadIdx.x == 0 ? (uint32_t)tg.cnt : 0u;
        return;
    }
    const uint32_t* __restrict__ keys = pg.first ? indices : keys_cur;
    const int shift = pg.shift;
    const uint32_t mask = (1u << pg.width) - 1u;
    const int base = tg.first + wave * (kSortTile / (kSortThreads / kWave));
    const int end = tg.first + tg.cnt;
    // all 16 key loads are issued before the first one is used (positions past the tile are clamped);
    // 16-byte loads of four keys per lane were measured and are not faster
    uint32_t key[kSortKeysPerThread];
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r)
        key[r] = keys[min(base + r * kWave + lane, end - 1)];
    if ((int)threadIdx.x < nd)
        s_hist[threadIdx.x] = 0;
    __syncthreads();
    // Counting needs no ranks: when the 64 keys of a round share one digit (identical rows are adjacent
    // from the second pass on) one lane adds the whole count, otherwise every lane adds 1; LDS integer
    // atomics, so the totals do not depend on the order.
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        const bool valid = q < end;                   // valid lanes are a prefix of the wavefront
        const uint32_t dg = (key[r] >> shift) & mask;
        const uint64_t vm = __ballot(valid);
        const uint32_t d0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)dg);
        const uint64_t same = __ballot(dg == d0);
        if ((same & vm) == vm) {
            if (lane == 0 && vm != 0ull)
                atomicAdd(&s_hist[d0], (uint32_t)__popcll(vm));
        } else if (valid) {
            atomicAdd(&s_hist[dg], 1u);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < nd)
        hist[tg.hbase + (int64_t)threadIdx.x * tg.hstride] = s_hist[threadIdx.x];
}

// A table's first pass reads the caller's index array as keys and computes the payload from the offsets;
// LAST (the launch in which every table makes its last pass): the table's row base is added to the keys
// that are written out.  V16 (batch <= 65536): between the passes the payload, a bag number below 2^16,
// travels as 16 bits (in the same buffers); the last launch writes the int32 payloads the update reads.
template <bool LAST, bool V16>
__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(
    SortPlan pl, const TableMeta* __restrict__ meta, const uint32_t* __restrict__ keys_cur,
    const int32_t* __restrict__ vals_in, const uint32_t* __restrict__ indices,
    uint32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out,
    const uint32_t* __restrict__ hist_scanned, const int64_t* __restrict__ offsets,
    const uint32_t* __restrict__ row_base, int32_t B, int p, int P, int nd_bits)
{
    constexpr int kWaves = kSortThreads / kWave;
    __shared__ uint32_t s_keys[kSortTile];
    __shared__ int32_t s_vals[kSortTile];
    __shared__ uint32_t s_whist[kWaves][256];
    __shared__ uint32_t s_dstart[256];
    __shared__ uint32_t s_goff[256];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int nd = 1 << nd_bits;
    TileGeom tg;
    if (!tile_geom(pl, blockIdx.x, nd, tg))
        return;
    const PassGeom pg = pass_geom(meta[tg.t].key_bits, p, P);
    if (!pg.active)
        return;                                  // the table sits this launch out: nothing moves
    const bool FIRST = pg.first;
    const int shift = pg.shift, bits = pg.width;
    const uint32_t mask = (1u << bits) - 1u;
    const uint32_t* __restrict__ keys_in = FIRST ? indices : keys_cur;
    const int tile_cnt = tg.cnt;
    const int end = tg.first + tile_cnt;

    for (int i = threadIdx.x; i < kWaves * 256; i += kSortThreads)
        (&s_whist[0][0])[i] = 0;
    __syncthreads();

    uint32_t key[kSortKeysPerThread];
    int32_t val[kSortKeysPerThread];
    uint32_t rank[kSortKeysPerThread];
    const int base = tg.first + wave * (kSortTile / kWaves);
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = min(base + r * kWave + lane, end - 1);
        key[r] = keys_in[q];
        if (!FIRST)
            val[r] = V16 ? (int32_t)reinterpret_cast<const uint16_t*>(vals_in)[q] : vals_in[q];
    }
    if (FIRST) {
        // payload = bag of the position: the borders of the bags the tile touches are staged in
        // LDS (in the space the reordered payloads use later) and searched there
        const int2 bags = *reinterpret_cast<const int2*>(&pl.tiles[blockIdx.x].bag_lo);
        const int b_lo = bags.x, b_hi = bags.y;
        const int nb = b_hi - b_lo + 1;
        const int64_t j0 = (int64_t)tg.t * B + b_lo;
        if (nb <= kSortTile) {
            for (int i = threadIdx.x; i < nb; i += kSortThreads)
                s_vals[i] = (int32_t)offsets[j0 + i];
            __syncthreads();
            int steps = 0;
            while ((1 << steps) < nb)
                ++steps;
#pragma unroll
            for (int r = 0; r < kSortKeysPerThread; ++r) {
                const int q = min(base + r * kWave + lane, end - 1);
                int a = 0, c = nb;  // last a with s_vals[a] <= q
                for (int st = 0; st < steps; ++st) {
                    const int mid = (a + c) >> 1;
                    const bool up = s_vals[mid] <= q;
                    a = up ? mid : a;
                    c = up ? c : max(mid, a + 1);
                }
                val[r] = b_lo + a;
            }
        } else {
#pragma unroll 1
            for (int r = 0; r < kSortKeysPerThread; ++r) {
                const int q = min(base + r * kWave + lane, end - 1);
                int a = 0, c = nb;
                while (c - a > 1) {
                    const int mid = (a + c) >> 1;
                    if (offsets[j0 + mid] <= q)
                        a = mid;
                    else
                        c = mid;
                }
                val[r] = b_lo + a;
            }
        }
    }
    // The wavefront's private counters are indexed as the LDS array they are (a pointer to the row would be
    // a generic pointer: flat loads and stores, each waited for).  LDS operations of one wavefront execute
    // in order and the compiler keeps a load behind a store that may alias it, so a round sees the counts
    // of the rounds before it.
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        const bool valid = q < end;
        const uint32_t dg = (key[r] >> shift) & mask;
        const uint64_t peers = match_digit(dg, valid, bits);
        const uint32_t pre = s_whist[wave][dg];
        const uint32_t below = (uint32_t)__popcll(peers & lt);
        if (valid && below == 0)
            s_whist[wave][dg] = pre + (uint32_t)__popcll(peers);
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
                s_goff[d] = hist_scanned[tg.hbase + (int64_t)d * tg.hstride] - ex;
            }
            ex += c[i];
        }
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < kSortKeysPerThread; ++r) {
        const int q = base + r * kWave + lane;
        if (q < end) {
            const uint32_t dg = (key[r] >> shift) & mask;
            const uint32_t pos = s_dstart[dg] + s_whist[wave][dg] + rank[r];
            s_keys[pos] = key[r];
            s_vals[pos] = val[r];
        }
    }
    __syncthreads();
    const uint32_t add = LAST ? row_base[tg.t] : 0u;
#pragma unroll
    for (int i = 0; i < kSortKeysPerThread; ++i) {
        const int p = threadIdx.x + i * kSortThreads;
        if (p < tile_cnt) {
            const uint32_t k = s_keys[p];
            const uint32_t g = s_goff[(k >> shift) & mask] + (uint32_t)p;
            keys_out[g] = k + add;
            if (V16 && !LAST)
                reinterpret_cast<uint16_t*>(vals_out)[g] = (uint16_t)s_vals[p];
            else
                vals_out[g] = s_vals[p];
        }
    }
}

// ---------------------------------------------------------------- device-wide exclusive scan (uint32)

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
// Each wavefront owns a span of kSpan consecutive sorted positions and every run that STARTS inside it.
// The span's run descriptors and payloads are staged in LDS once.  Lane mapping: a row of D floats
// is covered by LPR = pow2ceil(D/8) lanes, two float4 blocks per lane, so G = 64/LPR rows are
// fetched per load instruction.  The runs of the span are sorted by length class (a counting sort with
// ballots into a byte list in LDS) and handled class by class, so that every step is full:
//   * runs of one or two lookups: several per lane group and step (as many as the registers hold);
//   * runs of up to kShortRun lookups: one per lane group; all gradient rows, weight rows and moments
//     of a step are requested before anything is consumed, and all groups apply their update together;
//   * runs of up to 4 x 2^j lookups, 2^j <= G: teams of 2^j lane groups, G / 2^j runs per step, the
//     members' sums combined with an xor butterfly;
//   * longer runs use the whole wavefront in several steps (groups take alternate lookups); up to
//     kLongRun lookups the owner follows the run past its span and finishes it;
//   * a run longer than kLongRun is not summed here: it is queued, per table, for window_runs_kernel
//     (pieces by bag window) or, beyond the call's dense threshold, for dense_rows_kernel (counts x
//     gradient block); those write fp32 partial rows to the workspace, and the fix-up kernel adds a
//     run's partial rows in a fixed order and applies the single update.
// The single-lookup rows of the tail of the index distribution move a row, its moment and one gradient row
// each and run at the rate of the memory system; the steps of the longer runs are bound by how fast gradient
// rows come out of the caches, so nothing here is arranged around instruction counts.
// Either way each touched row is read, updated and written exactly once, nothing is accumulated
// with atomics, and the summation order is fixed: results are bit-identical run to run.
//
// All gathers are branch-free (slots past the end of a run read a row of zeros kept in the
// workspace, column offsets past D are clamped) so that the loads of a step are issued back to
// back and waited for once.

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

// Optimizer of the fused epilogue (Section 5.1 names AdaGrad and Adam next to the row-wise AdaGrad of
// Section 5.2).  state0: row-wise AdaGrad -> one moment per row (indexed by linear row id);
// AdaGrad -> sum of squares per element; Adam -> first moment per element, state1 -> second moment.
// Per-element states are indexed like the flat weight array.
constexpr int kOptRowwiseAdagrad = 0;
constexpr int kOptAdagrad = 1;
constexpr int kOptAdam = 2;

struct OptParams {
    float* state0;
    float* state1;
    float lr;
    float eps;
    float beta1;
    float beta2;
    float inv_bc1;   // 1 / (1 - beta1^step)
    float inv_bc2;   // 1 / (1 - beta2^step)
};

struct BwdArgs {
    const TableMeta* meta;
    const uint32_t* row_base;
    const uint32_t* sorted_keys;
    const int32_t* sorted_vals;
    const uint32_t* unique_keys;
    const int32_t* seg_offsets;
    const int32_t* chunk_first_run;
    Counters* counters;
    const void* grad_out;   // [B, sumD] in the gradient type (float, __half or __hip_bfloat16)
    void* weights;
    float* partials;      // [num_chunks][2][dpad]
    uint32_t* long_list;
    const float* zero_row;  // >= 2 KiB of zeros
    int32_t n;
    int32_t num_chunks;
    int32_t T;
    int32_t sumD;
    int32_t dpad;
    int32_t batch;
    int32_t table_major;   // gradient layout: 0 = [B, sumD] rows, 1 = one [B, D_t] block per table
    // dense hot rows (runs longer than dense_thr): queued per table by the update kernel, summed by dense_rows_kernel
    int32_t dense_thr;     // >= kDenseMinRun; INT32_MAX switches the dense path off
    int32_t dense_slices;  // ceil(batch / kDenseSlice): partial rows per dense run
    const int32_t* tstart; // [T+1] first sorted position of every table
    uint32_t* dense_cnt;   // [T] dense runs queued per table (zero between updates)
    uint32_t* dense_list;  // table t's queue starts at entry tstart[t] / dense_thr + t
    uint32_t* dense_dirty; // [T] set by dense_rows_kernel when a table's gradient block holds Inf / NaN
    // long runs (kLongRun < length <= dense_thr): queued per table, summed window by window by window_runs_kernel
    uint32_t* win_cnt;     // [T] (zero between updates)
    uint32_t* win_list;    // table t's queue starts at entry tstart[t] / kLongRun + t
    int32_t grad_bytes;    // bytes per gradient element (sizes the bag windows)
    OptParams opt;
};

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void acc4(float (&a)[4], const float4 v)
{
    a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w;
}

// Gradient rows in their storage type: Vec is what one lane loads for a block of 4 elements.
template <typename GT>
struct GradIO;

template <>
struct GradIO<float> {
    using Vec = float4;
    __device__ static __forceinline__ Vec ldv(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ static __forceinline__ void add(float (&a)[4], const Vec v) { acc4(a, v); }
};

template <>
struct GradIO<__half> {
    using Vec = uint2;
    __device__ static __forceinline__ Vec ldv(const __half* p) { return *reinterpret_cast<const uint2*>(p); }
    __device__ static __forceinline__ void add(float (&a)[4], const Vec v) { RowIO<__half, 4>::add(a, v); }
};

template <>
struct GradIO<__hip_bfloat16> {
    using Vec = uint2;
    __device__ static __forceinline__ Vec ldv(const __hip_bfloat16* p) { return *reinterpret_cast<const uint2*>(p); }
    // bfloat16 is the upper half of a float: widening is a 16-bit shift
    __device__ static __forceinline__ void add(float (&a)[4], const Vec v)
    {
        a[0] += __uint_as_float(v.x << 16); a[1] += __uint_as_float(v.x & 0xffff0000u);
        a[2] += __uint_as_float(v.y << 16); a[3] += __uint_as_float(v.y & 0xffff0000u);
    }
};

// Per-lane column geometry of a D-element row covered by LPR lanes with two 4-element blocks each.
struct Cols {
    int e0, e1;      // clamped element offsets of the two blocks (always loadable)
    bool c0, c1;     // whether the block really belongs to the row
    int sub, grp, lprl;
    __device__ __forceinline__ Cols(int D, int lprl_, int lane) : lprl(lprl_)
    {
        const int LPR = 1 << lprl;
        sub = lane & (LPR - 1);
        grp = lane >> lprl;
        const int a = sub * 4, b = (sub + LPR) * 4;
        c0 = a < D;
        c1 = b < D;
        e0 = min(a, D - 4);
        e1 = min(b, D - 4);
    }
};

// Whole-wavefront fp32 sum of the rows rowptr(i) (element type GT), i in [p0, p1), p1 > p0; rowptr must
// be valid for every i in the range.  Afterwards every lane group holds the complete sums.
template <typename GT, typename RowPtr>
__device__ __forceinline__ void wave_gather_sum(RowPtr rowptr, int p0, int p1, const float* __restrict__ zero_row_f,
                                                const Cols& c, float (&acc)[2][4])
{
    using GIO = GradIO<GT>;
    const GT* zero_row = reinterpret_cast<const GT*>(zero_row_f);
    const int G = kWave >> c.lprl;
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc[k][e] = 0.f;
    for (int i0 = p0; i0 < p1; i0 += G * kBwdUnroll) {
        typename GIO::Vec v[kBwdUnroll][2];
        const GT* rp[kBwdUnroll];
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            const int i = i0 + u * G + c.grp;
            const GT* p = rowptr(min(i, p1 - 1));
            rp[u] = i < p1 ? p : zero_row;
        }
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            v[u][0] = GIO::ldv(rp[u] + c.e0);
            v[u][1] = GIO::ldv(rp[u] + c.e1);
        }
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            GIO::add(acc[0], v[u][0]);
            GIO::add(acc[1], v[u][1]);
        }
    }
    for (int s = 1 << c.lprl; s < kWave; s <<= 1) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[k][e] += __shfl_xor(acc[k][e], s);
    }
}

// The optimizer state of the row held by this lane's group, requested together with the row itself.
template <int OPT>
struct OptRow {
    float m_old;         // row-wise AdaGrad
    float4 s0[2];        // AdaGrad sum of squares / Adam first moment, this lane's two blocks
    float4 s1[2];        // Adam second moment
    // key: linear row id; wel: index of the row's first element in the flat weight array
    __device__ __forceinline__ void load(const OptParams& p, uint32_t key, int64_t wel, const Cols& c)
    {
        if (OPT == kOptRowwiseAdagrad)
            m_old = p.state0[key];
        if (OPT == kOptAdagrad || OPT == kOptAdam) {
            s0[0] = ld4(p.state0 + wel + c.e0);
            s0[1] = ld4(p.state0 + wel + c.e1);
        }
        if (OPT == kOptAdam) {
            s1[0] = ld4(p.state1 + wel + c.e0);
            s1[1] = ld4(p.state1 + wel + c.e1);
        }
    }
};

__device__ __forceinline__ void st4(float* p, const float (&f)[4])
{
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
}
__device__ __forceinline__ void un4(const float4 v, float (&f)[4]) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }

// One block (4 elements) of the element-wise rules; g: aggregated gradient, w: weights (updated in place).
// Hardware reciprocal / square root (1 ulp each): far inside the 1e-5 tolerance of the result.
template <int OPT>
__device__ __forceinline__ void elementwise_block(const OptParams& p, const float (&g)[4], float (&w)[4],
                                                  const float4 s0v, const float4 s1v, float* s0p, float* s1p)
{
    float a[4], b[4];
    un4(s0v, a);
    if (OPT == kOptAdagrad) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] += g[e] * g[e];
            w[e] -= p.lr * g[e] * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(a[e]) + p.eps);
        }
        st4(s0p, a);
    } else {
        un4(s1v, b);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = p.beta1 * a[e] + (1.0f - p.beta1) * g[e];
            b[e] = p.beta2 * b[e] + (1.0f - p.beta2) * g[e] * g[e];
            w[e] -= p.lr * (a[e] * p.inv_bc1) *
                    __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(b[e] * p.inv_bc2) + p.eps);
        }
        st4(s0p, a);
        st4(s1p, b);
    }
}

// The optimizer epilogue for the row held by this lane's group (wv: the row's old values, raw).
//   row-wise AdaGrad (Section 5.2): m += mean_d(G_d^2); w -= lr * G / (sqrt(m) + eps)
//   AdaGrad: S_d += G_d^2; w_d -= lr * G_d / (sqrt(S_d) + eps)
//   Adam (lazy, bias-corrected): m = b1 m + (1-b1) G; v = b2 v + (1-b2) G^2;
//                                w -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
template <typename WT, int OPT>
__device__ __forceinline__ void optimizer_epilogue(WT* __restrict__ wrow, const typename RowIO<WT, 4>::Vec (&wv)[2],
                                                   const float (&acc)[2][4], int D, const Cols& c, bool writer,
                                                   const OptParams& p, uint32_t key, int64_t wel,
                                                   const OptRow<OPT>& st)
{
    if (OPT == kOptRowwiseAdagrad) {
        float ss0 = acc[0][0] * acc[0][0] + acc[0][1] * acc[0][1] + acc[0][2] * acc[0][2] + acc[0][3] * acc[0][3];
        float ss1 = acc[1][0] * acc[1][0] + acc[1][1] * acc[1][1] + acc[1][2] * acc[1][2] + acc[1][3] * acc[1][3];
        float ss = (c.c0 ? ss0 : 0.f) + (c.c1 ? ss1 : 0.f);
        for (int s = 1; s < (1 << c.lprl); s <<= 1)
            ss += __shfl_xor(ss, s);
        // hardware reciprocal / square root (1 ulp each): far inside the 1e-5 tolerance of the result
        const float m_new = st.m_old + ss * __builtin_amdgcn_rcpf((float)D);
        const float scale = p.lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(m_new) + p.eps);
        if (writer) {
            float w[4];
            if (c.c0) {
                RowIO<WT, 4>::unpack(wv[0], w);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] -= scale * acc[0][e];
                RowIO<WT, 4>::store(wrow + c.e0, w);
            }
            if (c.c1) {
                RowIO<WT, 4>::unpack(wv[1], w);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] -= scale * acc[1][e];
                RowIO<WT, 4>::store(wrow + c.e1, w);
            }
            if (c.sub == 0)
                p.state0[key] = m_new;
        }
    } else if (writer) {
        float w[4];
        if (c.c0) {
            RowIO<WT, 4>::unpack(wv[0], w);
            elementwise_block<OPT>(p, acc[0], w, st.s0[0], st.s1[0], p.state0 + wel + c.e0, p.state1 + wel + c.e0);
            RowIO<WT, 4>::store(wrow + c.e0, w);
        }
        if (c.c1) {
            RowIO<WT, 4>::unpack(wv[1], w);
            elementwise_block<OPT>(p, acc[1], w, st.s0[1], st.s1[1], p.state0 + wel + c.e1, p.state1 + wel + c.e1);
            RowIO<WT, 4>::store(wrow + c.e1, w);
        }
    }
}

__device__ __forceinline__ void store_partial(float* __restrict__ dst, const float (&acc)[2][4], const Cols& c)
{
    if (c.grp == 0) {
        if (c.c0)
            *reinterpret_cast<float4*>(dst + c.e0) = make_float4(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
        if (c.c1)
            *reinterpret_cast<float4*>(dst + c.e1) = make_float4(acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
    }
}

// One step of the update kernel: up to NB * (G >> tsl) runs of one table at once.  The G lane groups of the
// wavefront form teams of 1 << tsl groups; a team takes NB runs from the class list (entries i0 .. i0 + cnt - 1,
// run indices of the wavefront's span), every member group fetches up to ML gradient rows of each (member m takes
// the lookups m, m + team size, ...), the members' sums are combined with an xor butterfly, and member 0 applies
// the update.  All weight rows, moments and gradient rows of the step are requested before anything is consumed:
// the number of rows in flight per wavefront, not the instruction count, bounds this kernel.
template <typename WT, typename GT, int OPT, int ML, int NB>
__device__ __forceinline__ void run_batch(const BwdArgs& a, WT* __restrict__ wtab, int64_t woff,
                                          const GT* __restrict__ gb, int sumD,
                                          const int32_t* __restrict__ s_seg, const uint32_t* __restrict__ s_key,
                                          const int32_t* __restrict__ s_val, const uint8_t* __restrict__ s_list,
                                          int q0, int i0, int cnt, int tsl, uint32_t rbase, int D, const Cols& c)
{
    using IO = RowIO<WT, 4>;
    using GIO = GradIO<GT>;
    const int teams = (kWave >> c.lprl) >> tsl;
    const int team = c.grp >> tsl;
    const int member = c.grp & ((1 << tsl) - 1);
    typename IO::Vec wv[NB][2];
    OptRow<OPT> st[NB];
    uint32_t key[NB];
    int vbase[NB], len[NB], run[NB];
    bool act[NB];
    // all LDS reads of a level are issued together: the row requests below start one LDS round trip
    // after the other, not one per run
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int li = j * teams + team;
        act[j] = li < cnt;
        run[j] = s_list[i0 + (act[j] ? li : 0)];     // idle teams shadow the first run: loads stay valid
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        key[j] = s_key[run[j]];
        vbase[j] = s_seg[run[j]];
        len[j] = s_seg[run[j] + 1];
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        len[j] = act[j] ? len[j] - vbase[j] : 0;
        vbase[j] -= q0;
        const uint64_t rel = (uint64_t)(key[j] - rbase) * (uint32_t)D;
        wv[j][0] = IO::ldv(wtab + rel + c.e0);
        wv[j][1] = IO::ldv(wtab + rel + c.e1);
        st[j].load(a.opt, key[j], woff + (int64_t)rel, c);
    }
    typename GIO::Vec v[NB][ML][2];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const GT* rp[ML];
#pragma unroll
        for (int u = 0; u < ML; ++u) {
            const int pos = member + (u << tsl);
            const bool ok = pos < len[j];
            const int b = s_val[vbase[j] + (ok ? pos : 0)];
            rp[u] = ok ? gb + (uint64_t)(uint32_t)b * (uint32_t)sumD : reinterpret_cast<const GT*>(a.zero_row);
        }
#pragma unroll
        for (int u = 0; u < ML; ++u) {
            v[j][u][0] = GIO::ldv(rp[u] + c.e0);
            v[j][u][1] = GIO::ldv(rp[u] + c.e1);
        }
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        float acc[2][4];
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[k][e] = 0.f;
#pragma unroll
        for (int u = 0; u < ML; ++u) {
            GIO::add(acc[0], v[j][u][0]);
            GIO::add(acc[1], v[j][u][1]);
        }
        for (int sh = 1 << c.lprl; sh < (1 << (c.lprl + tsl)); sh <<= 1) {
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc[k][e] += __shfl_xor(acc[k][e], sh);
        }
        uint32_t kj = key[j];
        asm volatile("" : "+v"(kj));    // the store addresses are formed again here, not kept in registers meanwhile
        const uint64_t rel = (uint64_t)(kj - rbase) * (uint32_t)D;
        optimizer_epilogue<WT, OPT>(wtab + rel, wv[j], acc, D, c, act[j] && member == 0, a.opt, kj,
                                    woff + (int64_t)rel, st[j]);
    }
}

constexpr int kSpanChunks = 2;                  // chunks owned by one wavefront of the update kernel
constexpr int kSpan = kSpanChunks * kChunk;     // 256 sorted positions

template <typename WT, typename GT, int OPT>
__global__ __launch_bounds__(kBwdThreads) void reduce_update_kernel(BwdArgs a)
{
    using IO = RowIO<WT, 4>;
    const GT* __restrict__ grad_out = static_cast<const GT*>(a.grad_out);
    constexpr int kWaves = kBwdThreads / kWave;
    constexpr int kRounds = kSpan / kWave;         // staging rounds of one entry per lane
    constexpr int kSegCap = (kRounds + 1) * kWave; // >= kSpan + 1
    constexpr int kValCap = kSpan + kLongRun;      // a run owned by the span ends within this window
    // row-wise AdaGrad keeps one moment per row, so several runs per lane group fit in registers; the
    // element-wise optimizers carry whole state rows and take one run per group
    constexpr int kNB1 = OPT != kOptRowwiseAdagrad ? 1 : sizeof(WT) == 2 ? 4 : 2;   // runs of one lookup per group
    constexpr int kNB2 = OPT != kOptRowwiseAdagrad ? 1 : 2;                          // runs of two lookups per group
    static_assert(kSpan <= 256, "run indices of a span are kept in bytes");
    static_assert(kShortRun == 4, "run_batch is instantiated for 1..4 lookups");
    __shared__ int32_t s_seg_all[kWaves][kSegCap];
    __shared__ uint32_t s_key_all[kWaves][kSpan];
    __shared__ int32_t s_val_all[kWaves][kValCap];
    __shared__ uint8_t s_list_all[kWaves][kSpan];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    const int k = uniform(blockIdx.x * kWaves + wv);
    const int ch0 = k * kSpanChunks;
    if (ch0 >= a.num_chunks)
        return;
    const int ch1 = min(ch0 + kSpanChunks, a.num_chunks);
    int32_t* s_seg = s_seg_all[wv];
    uint32_t* s_key = s_key_all[wv];
    int32_t* s_val = s_val_all[wv];
    uint8_t* s_list = s_list_all[wv];

    const int q0 = ch0 * kChunk;
    const int q1 = min(a.n, q0 + kSpan);
    const int ub = a.chunk_first_run[ch0];
    const int ue = a.chunk_first_run[ch1];
    const int nruns = ue - ub;  // runs that start in [q0, q1): at most kSpan
    if (nruns == 0)
        return;     // the span lies inside one run: its owner, or (long runs) another kernel, sums all of it
    WT* __restrict__ weights = static_cast<WT*>(a.weights);
    const int32_t* __restrict__ vals = a.sorted_vals;

    // ---- stage run descriptors and payloads (wavefront-private LDS); straight-line clamped loads
    {
        int sg[kRounds + 1];
        uint32_t ky[kRounds];
        int vl[kRounds];
#pragma unroll
        for (int i = 0; i < kRounds + 1; ++i)
            sg[i] = a.seg_offsets[ub + min(i * kWave + lane, nruns)];
#pragma unroll
        for (int i = 0; i < kRounds; ++i)
            ky[i] = a.unique_keys[ub + min(i * kWave + lane, nruns - 1)];
#pragma unroll
        for (int i = 0; i < kRounds; ++i)
            vl[i] = vals[min(q0 + i * kWave + lane, a.n - 1)];
#pragma unroll
        for (int i = 0; i < kRounds + 1; ++i)
            s_seg[i * kWave + lane] = sg[i];
#pragma unroll
        for (int i = 0; i < kRounds; ++i) {
            s_key[i * kWave + lane] = ky[i];
            s_val[i * kWave + lane] = vl[i];
        }
    }
    __threadfence_block();
    __builtin_amdgcn_wave_barrier();
    // the last run that starts here may continue past the span: stage its payloads too, unless it is
    // a long run (those are not summed here)
    {
        const int e_last = uniform(s_seg[nruns]);
        const int s_last = uniform(s_seg[nruns - 1]);
        if (e_last > q1 && e_last - s_last <= kLongRun) {
            for (int p = q1 + lane; p < e_last; p += kWave)
                s_val[p - q0] = vals[p];
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
        }
    }

    const uint64_t lt = (1ull << lane) - 1ull;
    // entries [0, count) of s_list <- the span's runs of class cl, in run order
    auto build_list = [&](const int (&cls)[kRounds], int cl, int first) {
        int n = first;
#pragma unroll
        for (int i = 0; i < kRounds; ++i) {
            const uint64_t mk = __ballot(cls[i] == cl);
            if (cls[i] == cl)
                s_list[n + __popcll(mk & lt)] = (uint8_t)(i * kWave + lane);
            n += __popcll(mk);
        }
        return n;
    };
    auto run_len = [&](int li) {
        const int run = s_list[li];
        return uniform(s_seg[run + 1] - s_seg[run]);
    };

    int ra = 0;
    while (ra < nruns) {
        // ---- the runs [ra, rb) of the table of run ra (a span rarely touches more than one table)
        const uint32_t key0 = (uint32_t)uniform((int)s_key[ra]);
        const int t = uniform(find_table(a.row_base, a.T, key0));
        TableMeta m = a.meta[t];            // wavefront-uniform: kept in scalar registers
        m.woff = ((int64_t)uniform((int)(m.woff >> 32)) << 32) | (uint32_t)uniform((int)m.woff);
        m.rbase = (uint32_t)uniform((int)m.rbase);
        m.dim = uniform(m.dim);
        m.col = uniform(m.col);
        m.lpr_bwd = uniform(m.lpr_bwd);
        const uint32_t t_hi = (uint32_t)uniform((int)a.row_base[t + 1]);
        int rb = 0;
#pragma unroll
        for (int i = 0; i < kRounds; ++i) {
            const int run = i * kWave + lane;
            rb += __popcll(__ballot(run < nruns && s_key[min(run, nruns - 1)] < t_hi));
        }
        const int D = m.dim;
        const int lprl = m.lpr_bwd;
        const int lgG = 6 - lprl;
        const int G = 1 << lgG;
        const GT* gb = a.table_major ? grad_out + (int64_t)a.batch * m.col : grad_out + m.col;
        const int sumD = a.table_major ? m.dim : (int)a.sumD;   // distance between the gradient rows of consecutive bags
        WT* wtab = weights + m.woff;
        const Cols c(D, lprl, lane);

        // ---- classes by length: 0 .. 3: one .. four lookups; 3 + j: up to 4 << j lookups, summed by a team of
        // 1 << j lane groups (while that is at most a wavefront); 14: whole wavefront, several steps;
        // 15: long, queued for the fix-up kernel and, per table, for the kernel that sums it
        int cls[kRounds];
#pragma unroll
        for (int i = 0; i < kRounds; ++i) {
            const int run = i * kWave + lane;
            const bool valid = run >= ra && run < rb;
            const int rc = valid ? run : ra;
            const int len = s_seg[rc + 1] - s_seg[rc];
            int cl;
            if (len <= kShortRun) {
                cl = len - 1;
            } else if (len > kLongRun) {
                cl = 15;
            } else {
                const int tl = 32 - __clz((len - 1) >> 2);     // smallest tl with (4 << tl) >= len
                cl = tl <= lgG ? 3 + tl : 14;
            }
            cls[i] = valid ? cl : -1;
            if (valid && cl == 15) {
                if (len > a.dense_thr) {
                    const uint32_t dslot = atomicAdd(&a.dense_cnt[t], 1u);
                    a.dense_list[a.tstart[t] / a.dense_thr + t + (int)dslot] = (uint32_t)(ub + run);
                } else {
                    const uint32_t wslot = atomicAdd(&a.win_cnt[t], 1u);
                    a.win_list[a.tstart[t] / kLongRun + t + (int)wslot] = (uint32_t)(ub + run);
                }
                const uint32_t slot = atomicAdd(&a.counters->long_count, 1u);
                a.long_list[slot] = (uint32_t)(ub + run);
            }
        }

        // ---- runs of up to four lookups, shortest first: as many per step as the registers hold
        {
            int nshort = build_list(cls, 0, 0);
            nshort = build_list(cls, 1, nshort);
            nshort = build_list(cls, 2, nshort);
            nshort = build_list(cls, 3, nshort);
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
            int i = 0;
            while (i < nshort) {
                const int rem = nshort - i;
                if (kNB1 > 1 && rem > G) {
                    const int cand = min(kNB1 * G, rem);
                    if (run_len(i + cand - 1) == 1) {
                        if (kNB1 > 2 && cand > 2 * G)
                            run_batch<WT, GT, OPT, 1, kNB1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c);
                        else
                            run_batch<WT, GT, OPT, 1, 2>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c);
                        i += cand;
                        continue;
                    }
                }
                if (kNB2 > 1 && rem > G) {
                    const int cand = min(2 * G, rem);
                    const int ml = run_len(i + cand - 1);
                    if (ml <= 2) {
                        if (ml == 1)
                            run_batch<WT, GT, OPT, 1, 2>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c);
                        else
                            run_batch<WT, GT, OPT, 2, 2>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c);
                        i += cand;
                        continue;
                    }
                }
                const int cand = min(G, rem);
                switch (run_len(i + cand - 1)) {
                    case 1: run_batch<WT, GT, OPT, 1, 1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c); break;
                    case 2: run_batch<WT, GT, OPT, 2, 1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c); break;
                    case 3: run_batch<WT, GT, OPT, 3, 1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c); break;
                    default: run_batch<WT, GT, OPT, 4, 1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, cand, 0, m.rbase, D, c); break;
                }
                i += cand;
            }
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
        }

        // ---- teams of 2, 4, ... lane groups: runs of up to 4 lookups per member group, one step each
        for (int tl = 1; tl <= lgG; ++tl) {
            const int cnt = build_list(cls, 3 + tl, 0);
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
            const int teams = G >> tl;
            for (int i = 0; i < cnt; i += teams)
                run_batch<WT, GT, OPT, 4, 1>(a, wtab, m.woff, gb, sumD, s_seg, s_key, s_val, s_list, q0, i, min(teams, cnt - i), tl, m.rbase, D, c);
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
        }

        // ---- longer runs: the whole wavefront, several steps
        {
            const int cnt = build_list(cls, 14, 0);
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
            for (int i = 0; i < cnt; ++i) {
                const int run = uniform((int)s_list[i]);
                const uint32_t key = (uint32_t)uniform((int)s_key[run]);
                const int s0 = uniform(s_seg[run]);
                const int len0 = uniform(s_seg[run + 1]) - s0;
                const int64_t rel = (int64_t)(key - m.rbase) * D;
                WT* wrow = wtab + rel;
                typename IO::Vec wvv[2];
                OptRow<OPT> st;
                wvv[0] = IO::ldv(wrow + c.e0);
                wvv[1] = IO::ldv(wrow + c.e1);
                st.load(a.opt, key, m.woff + rel, c);
                float acc[2][4];
                wave_gather_sum<GT>([&](int p) { return gb + (int64_t)s_val[p - q0] * sumD; }, s0, s0 + len0, a.zero_row,
                                    c, acc);
                optimizer_epilogue<WT, OPT>(wrow, wvv, acc, D, c, c.grp == 0, a.opt, key, m.woff + rel, st);
            }
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
        }
        ra = rb;
    }
}

// ---------------------------------------------------------------- dense hot rows
//
// Under a skewed index distribution a few rows per table are looked up by a large share of the bags
// (Section 5.1 aggregates all of their gradients before the one optimizer step).  Gathering one gradient
// row per lookup re-reads the table's [B, D_t] gradient block once per such row.  For a run longer than
// the call's dense threshold (about one lookup per 8 bags) the sum is formed the other way round:
//     G[r, :] = sum_b count[r, b] * grad[b, :]
// with count[r, b] = how often bag b looks row r up.  kDenseRows runs of one table form a group and share
// ONE pass over the gradient block; a work unit is (group, slice of kDenseSlice bags) and writes one fp32
// partial row per run into the slots of the chunks that run covers completely (the update kernel leaves
// them unused); the fix-up kernel adds a run's partial rows in slice order and applies the single step.
// Counts are exact integers built with LDS integer atomics from the run's sorted payloads; the float sum of
// a (run, slice) has a fixed order that does not depend on which other runs share the group, so results
// are bit-identical run to run.  A bag with a non-finite gradient must only reach the rows it looks up:
// such a bag takes a select-based path instead of multiplying by a zero count.

struct DenseGroup {      // 32 bytes
    int32_t t;           // table
    int32_t first;       // index of the group's first run in the compact run list
    int32_t nrows;       // runs in the group (1..kDenseRows)
    int32_t gbase;       // first group of the table
    int32_t ng;          // groups of the table
    int32_t pad[3];
};

struct DenseArgs {              // also used for the windowed runs (groups of one run, slices = windows)
    BwdArgs b;
    const uint32_t* drun;       // compact list of runs (run index u), grouped by table
    const DenseGroup* dgroup;
    int32_t* dbounds;           // [run][nsub + 1] first sorted position of the run whose bag is >= c * slice_bags
    const uint32_t* nruns;      // number of runs in drun (device counter)
    int32_t nsub;               // number of slices = ceil(batch / slice_bags)
    int32_t slice_bags;
};

// one workgroup: per-table queues -> compact run list + groups of at most rpg runs; clears the per-table
// counters.  cnt / list: the queues (table t's starts at entry tstart[t] / base_div + t).
__global__ __launch_bounds__(256) void run_plan_kernel(BwdArgs a, uint32_t* __restrict__ cnt,
                                                       const uint32_t* __restrict__ list, int base_div, int rpg,
                                                       uint32_t* __restrict__ drun, DenseGroup* __restrict__ dgroup,
                                                       uint32_t* __restrict__ out_runs, uint32_t* __restrict__ out_groups,
                                                       uint32_t* __restrict__ clear_flags)
{
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_c[256], s_rfirst[256], s_gfirst[256];
    uint32_t carry_r = 0, carry_g = 0;
    for (int base = 0; base < a.T; base += 256) {
        const int t = base + threadIdx.x;
        const uint32_t c = t < a.T ? cnt[t] : 0u;
        const uint32_t g = (c + rpg - 1) / rpg;
        if (t < a.T && clear_flags)
            clear_flags[t] = 0;
        uint32_t tot_r, tot_g;
        const uint32_t ex_r = block_exclusive_scan_256(c, s_wave, tot_r);
        const uint32_t ex_g = block_exclusive_scan_256(g, s_wave, tot_g);
        s_c[threadIdx.x] = c;
        s_rfirst[threadIdx.x] = carry_r + ex_r;
        s_gfirst[threadIdx.x] = carry_g + ex_g;
        if (c > 0)
            cnt[t] = 0;
        __syncthreads();
        // short queues (the usual case) are copied by their own thread, all tables at once ...
        if (c > 0 && c <= 64) {
            const uint32_t rfirst = carry_r + ex_r, gfirst = carry_g + ex_g;
            const uint32_t* q = list + (a.tstart[t] / base_div + t);
            for (uint32_t i = 0; i < c; ++i)
                drun[rfirst + i] = q[i];
            for (uint32_t gi = 0; gi < g; ++gi) {
                DenseGroup d;
                d.t = t;
                d.first = (int32_t)(rfirst + gi * rpg);
                d.nrows = (int32_t)min((uint32_t)rpg, c - gi * rpg);
                d.gbase = (int32_t)gfirst;
                d.ng = (int32_t)g;
                d.pad[0] = d.pad[1] = d.pad[2] = 0;
                dgroup[gfirst + gi] = d;
            }
        }
        // ... long ones (a queue can be long when the batch is small) by the whole workgroup, one table after the other
        const int nt = min(256, a.T - base);
        for (int tt = 0; tt < nt; ++tt) {
            const uint32_t ct = s_c[tt];
            if (ct <= 64)
                continue;
            const uint32_t rfirst = s_rfirst[tt], gfirst = s_gfirst[tt];
            const uint32_t gt = (ct + rpg - 1) / rpg;
            const uint32_t* q = list + (a.tstart[base + tt] / base_div + base + tt);
            for (uint32_t i = threadIdx.x; i < ct; i += 256)
                drun[rfirst + i] = q[i];
            for (uint32_t gi = threadIdx.x; gi < gt; gi += 256) {
                DenseGroup d;
                d.t = base + tt;
                d.first = (int32_t)(rfirst + gi * rpg);
                d.nrows = (int32_t)min((uint32_t)rpg, ct - gi * rpg);
                d.gbase = (int32_t)gfirst;
                d.ng = (int32_t)gt;
                d.pad[0] = d.pad[1] = d.pad[2] = 0;
                dgroup[gfirst + gi] = d;
            }
        }
        __syncthreads();
        carry_r += tot_r;
        carry_g += tot_g;
    }
    if (threadIdx.x == 0) {
        *out_runs = carry_r;
        if (out_groups)
            *out_groups = carry_g;
    }
}

// one wavefront per listed run: where the run's payloads (ascending bags) cross every multiple of slice_bags
__global__ __launch_bounds__(256) void run_bounds_kernel(DenseArgs d)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_global = uniform(blockIdx.x * 4 + (threadIdx.x >> 6));
    const int wave_total = gridDim.x * 4;
    const int nruns = (int)*d.nruns;
    const int nb = d.nsub + 1;
    const int32_t* __restrict__ vals = d.b.sorted_vals;
    for (int i = wave_global; i < nruns; i += wave_total) {
        const int u = (int)d.drun[i];
        const int s = d.b.seg_offsets[u];
        const int e = d.b.seg_offsets[u + 1];
        for (int c = lane; c < nb; c += kWave) {
            const int target = c * d.slice_bags;
            int lo = s, hi = e;              // first p in [s, e) with vals[p] >= target
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (vals[mid] < target)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            d.dbounds[(int64_t)i * nb + c] = c == d.nsub ? e : lo;
        }
    }
}

typedef float mfma_f4 __attribute__((ext_vector_type(4)));

// the four gradient values of one 16-byte (fp32) / 8-byte (16-bit) load as floats
__device__ __forceinline__ void grad_floats(const float4 v, float (&g)[4]) { g[0] = v.x; g[1] = v.y; g[2] = v.z; g[3] = v.w; }
__device__ __forceinline__ void grad_floats_half(const uint2 v, float (&g)[4])
{
    const float2 x = __half22float2(*reinterpret_cast<const __half2*>(&v.x));
    const float2 y = __half22float2(*reinterpret_cast<const __half2*>(&v.y));
    g[0] = x.x; g[1] = x.y; g[2] = y.x; g[3] = y.y;
}
__device__ __forceinline__ void grad_floats_bf16(const uint2 v, float (&g)[4])
{
    g[0] = __uint_as_float(v.x << 16); g[1] = __uint_as_float(v.x & 0xffff0000u);
    g[2] = __uint_as_float(v.y << 16); g[3] = __uint_as_float(v.y & 0xffff0000u);
}
template <typename GT> struct GradFloats;
template <> struct GradFloats<float> { __device__ static __forceinline__ void get(const float4 v, float (&g)[4]) { grad_floats(v, g); } };
template <> struct GradFloats<__half> { __device__ static __forceinline__ void get(const uint2 v, float (&g)[4]) { grad_floats_half(v, g); } };
template <> struct GradFloats<__hip_bfloat16> { __device__ static __forceinline__ void get(const uint2 v, float (&g)[4]) { grad_floats_bf16(v, g); } };

// One (group, slice) unit for a table of D columns: RT tiles of 16 runs, CL loads of 64 columns per bag.
// The contraction runs on the matrix cores in fp32 (v_mfma_f32_16x16x4_f32: 16 runs x 16 columns x 4 bags;
// operand A = counts, lane l holds run l%16 of bag l/16; operand B = gradient, lane l holds one column of
// bag l/16; a lane's gradient load covers columns 4*(l%16)..+3, so tile q of a load takes component q and
// holds columns 4*(l%16)+q; result tile: lane l holds runs 4*(l/16)+i, i = 0..3).  Counts are exact small
// integers, products and sums are fp32: the same arithmetic as adding the gradient row count times.
//
// The count table of the whole slice is one byte per (bag, run), built with LDS integer atomics on the
// containing words.  A bag that holds one row 256 times or more would overflow its byte, and 0 x Inf / NaN of
// a bag's gradient would reach runs the bag does not look up: both cases only set the table's dirty flag;
// the fix-up kernel then ignores the partial rows of that table's dense runs and sums those runs by gathering.
template <typename GT, int RT, int CL>
__device__ __forceinline__ void dense_unit(const DenseArgs& d, const DenseGroup& grp, const TableMeta& m, int j,
                                           uint32_t* __restrict__ s_cnt, int32_t* __restrict__ s_p0,
                                           int32_t* __restrict__ s_pre, int32_t* __restrict__ s_slot,
                                           uint32_t& dirty_bits)
{
    using GIO = GradIO<GT>;
    constexpr int kWaves = kDenseThreads / kWave;
    constexpr int kBagsPerWave = kDenseSlice / kWaves;        // 256 bags = 64 steps of 4
    constexpr int kSteps = kBagsPerWave / 4;
    constexpr int kUnroll = CL == 2 ? 2 : 4;                  // steps whose gradient loads are issued together
    constexpr int kLoads = 8;                                 // payload loads in flight per thread while counting
    const BwdArgs& a = d.b;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x >> 6;
    const int l16 = lane & 15, kq = lane >> 4;
    const int D = m.dim;
    const int nb = a.dense_slices + 1;
    const int64_t stride = a.table_major ? D : a.sumD;
    const GT* __restrict__ grad_out = static_cast<const GT*>(a.grad_out);
    const GT* gb = a.table_major ? grad_out + (int64_t)a.batch * m.col : grad_out + m.col;
    const int32_t* __restrict__ vals = a.sorted_vals;
    const uint8_t* s_cnt8 = reinterpret_cast<const uint8_t*>(s_cnt);
    const int sl_lo = j * kDenseSlice;
    const int sl_n = min(kDenseSlice, a.batch - sl_lo);       // >= 1

    // ---- count table of the slice
    __syncthreads();
    for (int i = threadIdx.x; i < kDenseSlice * kDenseRows / 16; i += kDenseThreads)
        reinterpret_cast<uint4*>(s_cnt)[i] = make_uint4(0u, 0u, 0u, 0u);
    if (threadIdx.x < kDenseRows) {
        int p0 = 0, cntr = 0, slot = 0;
        if ((int)threadIdx.x < grp.nrows) {
            const int64_t bi = (int64_t)(grp.first + threadIdx.x) * nb + j;
            p0 = d.dbounds[bi];
            cntr = d.dbounds[bi + 1] - p0;
            const int u = (int)d.drun[grp.first + threadIdx.x];
            slot = (a.seg_offsets[u] / kChunk + 1) * 2 + j;
        }
        s_p0[threadIdx.x] = p0;
        s_slot[threadIdx.x] = slot;
        int incl = cntr;   // inclusive prefix over the group's runs inside the first wavefront
#pragma unroll
        for (int o = 1; o < kDenseRows; o <<= 1) {
            const int up = __shfl_up(incl, o);
            if ((int)threadIdx.x >= o)
                incl += up;
        }
        s_pre[threadIdx.x + 1] = incl;
        if (threadIdx.x == 0)
            s_pre[0] = 0;
    }
    __syncthreads();
    const int tot = s_pre[kDenseRows];
    for (int f0 = 0; f0 < tot; f0 += kDenseThreads * kLoads) {
        int rr[kLoads], bb[kLoads];
#pragma unroll
        for (int x = 0; x < kLoads; ++x) {       // all loads are issued before the first atomic
            const int f = f0 + x * kDenseThreads + threadIdx.x;
            int lo = 0, hi = kDenseRows;         // last r with s_pre[r] <= f
#pragma unroll
            for (int st = 0; st < 5; ++st) {
                const int mid = (lo + hi) >> 1;
                if (s_pre[mid] <= f)
                    lo = mid;
                else
                    hi = mid;
            }
            rr[x] = f < tot ? lo : -1;
            bb[x] = f < tot ? vals[s_p0[lo] + (f - s_pre[lo])] : 0;
        }
#pragma unroll
        for (int x = 0; x < kLoads; ++x) {
            if (rr[x] >= 0) {
                const int sh = 8 * (rr[x] & 3);
                const uint32_t old = atomicAdd(&s_cnt[(bb[x] - sl_lo) * (kDenseRows / 4) + (rr[x] >> 2)], 1u << sh);
                if (((old >> sh) & 0xffu) == 0xffu)
                    dirty_bits = 0x7f800000u;    // the byte wrapped around
            }
        }
    }
    __syncthreads();

    for (int cbase = 0; cbase < D; cbase += CL * 64) {
        int coff[CL];
#pragma unroll
        for (int cl = 0; cl < CL; ++cl)
            coff[cl] = min(cbase + cl * 64 + 4 * l16, D - 4);   // columns past D are computed and dropped
        mfma_f4 acc[RT][CL][4];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int cl = 0; cl < CL; ++cl)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    acc[rt][cl][q] = mfma_f4{0.f, 0.f, 0.f, 0.f};

        // ---- counts x gradient rows on the matrix cores; a wavefront takes kBagsPerWave consecutive bags.
        // Bags past the end of the batch have all-zero counts; their gradient operand is the batch's last row.
        const int wbase = wv * kBagsPerWave;
        const uint8_t* ap = s_cnt8 + (wbase + kq) * kDenseRows + l16;
        if (wbase < sl_n) {
            for (int s0 = 0; s0 < kSteps; s0 += kUnroll) {
                typename GIO::Vec raw[kUnroll][CL];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int x = min(wbase + (s0 + u) * 4 + kq, sl_n - 1);
                    const GT* rp = gb + (int64_t)(sl_lo + x) * stride;
#pragma unroll
                    for (int cl = 0; cl < CL; ++cl)
                        raw[u][cl] = GIO::ldv(rp + coff[cl]);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    float av[RT];
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        av[rt] = (float)ap[((s0 + u) * 4) * kDenseRows + rt * 16];
#pragma unroll
                    for (int cl = 0; cl < CL; ++cl) {
                        float g[4];
                        GradFloats<GT>::get(raw[u][cl], g);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            dirty_bits = max(dirty_bits, __float_as_uint(g[q]) & 0x7f800000u);   // Inf / NaN: all ones
#pragma unroll
                            for (int rt = 0; rt < RT; ++rt)
                                acc[rt][cl][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[rt], g[q], acc[rt][cl][q], 0, 0, 0);
                        }
                    }
                }
            }
        }
        // ---- wavefronts of the workgroup, in wavefront order, one tile of 16 runs at a time through LDS.
        // The count table is overwritten: a further column pass (rows wider than CL * 64) builds it again.
        constexpr int kCH = CL < 2 ? CL : 2;                // 64-column loads per pass through LDS
        constexpr int kW = kCH * 64;                        // columns per pass
        float* s_red = reinterpret_cast<float*>(s_cnt);     // [kWaves][16][kW] floats <= 32 KiB
        for (int rt = 0; rt < RT; ++rt) {
            for (int ch = 0; ch < CL; ch += kCH) {
                __syncthreads();
#pragma unroll
                for (int cl = 0; cl < CL; ++cl) {
                    if (cl >= ch && cl < ch + kCH) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            *reinterpret_cast<float4*>(&s_red[(wv * 16 + 4 * kq + i) * kW + (cl - ch) * 64 + 4 * l16]) =
                                make_float4(acc[rt][cl][0][i], acc[rt][cl][1][i], acc[rt][cl][2][i], acc[rt][cl][3][i]);
                    }
                }
                __syncthreads();
                for (int idx = threadIdx.x; idx < 16 * (kW / 4); idx += kDenseThreads) {
                    const int r = idx / (kW / 4);
                    const int c4 = (idx - r * (kW / 4)) * 4;
                    const int row = rt * 16 + r;
                    const int col = cbase + ch * 64 + c4;
                    if (row < grp.nrows && col < D) {
                        float4 sum = *reinterpret_cast<const float4*>(&s_red[r * kW + c4]);
#pragma unroll
                        for (int w2 = 1; w2 < kWaves; ++w2) {
                            const float4 v = *reinterpret_cast<const float4*>(&s_red[(w2 * 16 + r) * kW + c4]);
                            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
                        }
                        *reinterpret_cast<float4*>(a.partials + (int64_t)s_slot[row] * a.dpad + col) = sum;
                    }
                }
            }
        }
        if (cbase + CL * 64 < D) {
            // rebuild the count table for the next column pass (only rows wider than 128 columns get here)
            __syncthreads();
            for (int i = threadIdx.x; i < kDenseSlice * kDenseRows / 16; i += kDenseThreads)
                reinterpret_cast<uint4*>(s_cnt)[i] = make_uint4(0u, 0u, 0u, 0u);
            __syncthreads();
            for (int f = threadIdx.x; f < tot; f += kDenseThreads) {
                int lo = 0, hi = kDenseRows;
#pragma unroll
                for (int st = 0; st < 5; ++st) {
                    const int mid = (lo + hi) >> 1;
                    if (s_pre[mid] <= f)
                        lo = mid;
                    else
                        hi = mid;
                }
                const int b = vals[s_p0[lo] + (f - s_pre[lo])];
                atomicAdd(&s_cnt[(b - sl_lo) * (kDenseRows / 4) + (lo >> 2)], 1u << (8 * (lo & 3)));
            }
            __syncthreads();
        }
    }
}

template <typename GT>
__global__ __launch_bounds__(kDenseThreads, 4) void dense_rows_kernel(DenseArgs d)
{
    __shared__ __align__(16) uint32_t s_cnt[kDenseSlice * kDenseRows / 4];   // 32 KiB; reused for the cross-wave sums
    __shared__ int32_t s_p0[kDenseRows], s_pre[kDenseRows + 1], s_slot[kDenseRows];
    const BwdArgs& a = d.b;
    const int ngroups = (int)a.counters->dense_groups;
    const int nslices = a.dense_slices;
    const int total = ngroups * nslices;
    // Work units in an order that keeps the groups of one (table, slice) next to each other, and the
    // workgroups that share an L2 (every 8th one) on neighbouring units: they then read the same piece of
    // the gradient block at about the same time.
    const int xcd = blockIdx.x & 7, nper = gridDim.x >> 3, within = blockIdx.x >> 3;
    const int per_xcd = (total + 7) / 8;
    for (int w = within; w < per_xcd; w += nper) {
        const int unit = xcd * per_xcd + w;
        if (unit >= total)
            break;
        // unit -> (group, slice): the units of table t are [gbase * nslices, (gbase + ng) * nslices), slice-major
        const DenseGroup any = d.dgroup[unit / nslices];
        const int local = unit - any.gbase * nslices;
        const int j = local / any.ng;
        const DenseGroup grp = d.dgroup[any.gbase + (local - j * any.ng)];
        const TableMeta m = a.meta[grp.t];
        uint32_t dirty_bits = 0;
        // 128 columns per pass (64 for narrow tables); wider rows take further passes over the same bags
        if (grp.nrows > 16) {
            if (m.dim > 64)
                dense_unit<GT, 2, 2>(d, grp, m, j, s_cnt, s_p0, s_pre, s_slot, dirty_bits);
            else
                dense_unit<GT, 2, 1>(d, grp, m, j, s_cnt, s_p0, s_pre, s_slot, dirty_bits);
        } else {
            if (m.dim > 64)
                dense_unit<GT, 1, 2>(d, grp, m, j, s_cnt, s_p0, s_pre, s_slot, dirty_bits);
            else
                dense_unit<GT, 1, 1>(d, grp, m, j, s_cnt, s_p0, s_pre, s_slot, dirty_bits);
        }
        if (__ballot(dirty_bits == 0x7f800000u) != 0ull && (threadIdx.x & (kWave - 1)) == 0)
            atomicOr(&a.dense_dirty[grp.t], 1u);
    }
}

// ---------------------------------------------------------------- long runs, window by window
//
// A run of kLongRun < L <= dense threshold lookups is cut into pieces by bag window (the batch is divided
// into at most kWinMax windows of win_bags bags); the payloads of a run ascend by bag, so a piece is a
// contiguous part of the run.  One wavefront sums one piece (one gathered gradient row per lookup) and
// writes one fp32 partial row; the fix-up kernel adds a run's partial rows in window order.  Pieces are
// processed table by table, window by window, run by run, and the wavefronts that share an L2 work on
// neighbouring pieces: the gradient rows they gather then come from one window of one table's gradient
// block (2 MiB for 128 fp32 columns) instead of from all of it, and are mostly found in L2.
// The partial rows of a run live in the slots of the chunks it covers completely (two per chunk).  A run
// too short to own kWinMax slots merges neighbouring windows in pairs or fours (8 or 4 pieces).

// Bag windows of a table with D columns: about 2 MiB of its gradient block each (a power of two of at least
// 1024 bags), at most kWinMax windows per batch.
struct WinGeom {
    int bags, nwin;
};

__device__ __forceinline__ WinGeom window_geom(int batch, int D, int grad_bytes)
{
    WinGeom g;
    g.bags = 1024;
    while (g.bags * 2 * D * grad_bytes <= (2 << 20))
        g.bags <<= 1;
    g.nwin = (batch + g.bags - 1) / g.bags;
    if (g.nwin > kWinMax) {
        g.bags = ((batch + kWinMax - 1) / kWinMax + 1023) / 1024 * 1024;
        g.nwin = (batch + g.bags - 1) / g.bags;
    }
    g.nwin = max(g.nwin, 1);
    return g;
}

// pieces a run of sorted positions [s, e) is cut into: as many windows as it has slots for, as a power of two
__device__ __forceinline__ int window_step(int s, int e, int nwin)
{
    const int slots = 2 * ((e - 1) / kChunk - s / kChunk - 1);     // >= 6 for a run longer than kLongRun
    int step = 1;                                                  // windows per piece
    while ((nwin + step - 1) / step > slots)
        step <<= 1;
    return step;
}

struct WinPiece {        // 16 bytes: what a wavefront needs to sum one piece, in one load
    int32_t p0, p1;      // sorted positions of the piece
    int32_t slot;        // partial row it writes; < 0: merged into the piece that starts at an earlier window
    int32_t t;           // table
};

// one workgroup: exclusive prefixes of the per-table queue lengths (wpre[T] = number of windowed runs) and of
// the per-table piece counts, runs x windows (ppre[T] = number of pieces); clears the queue lengths and the
// piece-claim counters for this update
__global__ __launch_bounds__(256) void window_plan_kernel(BwdArgs a, uint32_t* __restrict__ wpre,
                                                          uint32_t* __restrict__ ppre)
{
    __shared__ uint32_t s_wave[4];
    uint32_t carry = 0, carry_p = 0;
    for (int base = 0; base < a.T; base += 256) {
        const int t = base + threadIdx.x;
        const uint32_t c = t < a.T ? a.win_cnt[t] : 0u;
        const uint32_t np = t < a.T ? c * (uint32_t)window_geom(a.batch, a.meta[t].dim, a.grad_bytes).nwin : 0u;
        uint32_t tot, tot_p;
        const uint32_t ex = block_exclusive_scan_256(c, s_wave, tot);
        const uint32_t ex_p = block_exclusive_scan_256(np, s_wave, tot_p);
        if (t < a.T) {
            wpre[t] = carry + ex;
            ppre[t] = carry_p + ex_p;
            if (c > 0)
                a.win_cnt[t] = 0;
        }
        carry += tot;
        carry_p += tot_p;
    }
    if (threadIdx.x == 0) {
        wpre[a.T] = carry;
        ppre[a.T] = carry_p;
        a.counters->win_runs = carry;
        a.counters->win_pieces = carry_p;
    }
    if (threadIdx.x < 8)
        a.counters->win_next[threadIdx.x][0] = 0;
}

// Sixteen lanes per windowed run (four runs per wavefront): where the run's payloads (ascending bags) cross the
// window borders, written as the run's piece records.  Run ri belongs to the table t with wpre[t] <= ri <
// wpre[t + 1] and is entry ri - wpre[t] of that table's queue; the pieces of table t are
// [ppre[t], ppre[t + 1]), window-major, run-minor.
__global__ __launch_bounds__(256) void window_pieces_kernel(BwdArgs a, const uint32_t* __restrict__ wpre,
                                                            const uint32_t* __restrict__ ppre,
                                                            WinPiece* __restrict__ pieces)
{
    static_assert(kWinMax == 16, "one 16-lane group per run");
    const int lane = threadIdx.x & (kWave - 1);
    const int sub = lane & 15;
    const int nruns = (int)wpre[a.T];
    const int32_t* __restrict__ vals = a.sorted_vals;
    const int groups_total = gridDim.x * (256 / 16);
    for (int ri0 = (blockIdx.x * 256 + (int)threadIdx.x) >> 4; ri0 - (ri0 & 3) < nruns; ri0 += groups_total) {
        const bool live = ri0 < nruns;               // the four groups of a wavefront stay together for the shuffle
        const int ri = live ? ri0 : nruns - 1;
        int t0 = 0, t1 = a.T;                        // wpre[t0] <= ri < wpre[t1]
        while (t1 - t0 > 1) {
            const int mid = (t0 + t1) >> 1;
            if ((int)wpre[mid] <= ri)
                t0 = mid;
            else
                t1 = mid;
        }
        const int gbase = (int)wpre[t0], ng = (int)wpre[t0 + 1] - gbase;
        const WinGeom wg = window_geom(a.batch, a.meta[t0].dim, a.grad_bytes);
        const int nwin = wg.nwin;
        const int u = (int)a.win_list[a.tstart[t0] / kLongRun + t0 + (ri - gbase)];
        const int s = a.seg_offsets[u];
        const int e = a.seg_offsets[u + 1];
        const int step = window_step(s, e, nwin);
        int bound = e;                               // first p in [s, e) with vals[p] >= sub * win_bags
        if (sub < nwin) {
            const int target = sub * wg.bags;
            int lo = s, hi = e;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (vals[mid] < target)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            bound = lo;
        }
        const int up = __shfl(bound, (lane & ~15) | min(sub + step, 15));
        if (live && sub < nwin) {
            WinPiece p;
            p.p0 = bound;
            p.p1 = sub + step >= nwin ? e : up;
            p.slot = sub % step == 0 ? (s / kChunk + 1) * 2 + sub / step : -1;
            p.t = t0;
            pieces[(int64_t)ppre[t0] + (int64_t)sub * ng + (ri - gbase)] = p;
        }
    }
}

template <typename GT>
__global__ __launch_bounds__(kBwdThreads) void window_runs_kernel(BwdArgs a, const WinPiece* __restrict__ pieces)
{
    using GIO = GradIO<GT>;
    const int lane = threadIdx.x & (kWave - 1);
    const int total = (int)a.counters->win_pieces;
    const GT* __restrict__ grad_out = static_cast<const GT*>(a.grad_out);
    const GT* zero_row = reinterpret_cast<const GT*>(a.zero_row);
    const int32_t* __restrict__ vals = a.sorted_vals;
    // The workgroups that share an L2 (every 8th block) take the pieces of one eighth of the list, kWinBatch
    // consecutive unclaimed ones at a time (one integer atomic per batch; the wavefronts of the workgroup then
    // share the batch out through LDS): whatever the pieces' lengths, the wavefronts of an L2 domain are always
    // at work on neighbouring pieces.  Which wavefront sums a piece has no influence on the result.
    __shared__ int s_batch, s_taken;
    const int xcd = blockIdx.x & 7;
    const int per_xcd = (total + 7) / 8;
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) {
            s_batch = (int)atomicAdd(&a.counters->win_next[xcd][0], (uint32_t)kWinBatch);
            s_taken = 0;
        }
        __syncthreads();
        const int batch0 = s_batch;
        if (batch0 >= per_xcd)
            break;
      for (;;) {
        int w = 0;
        if (lane == 0)
            w = atomicAdd(&s_taken, 1);
        w = uniform(w);
        if (w >= kWinBatch || batch0 + w >= per_xcd)
            break;
        const int piece = xcd * per_xcd + batch0 + w;
        if (piece >= total)
            break;
        const int4 rec = *reinterpret_cast<const int4*>(&pieces[piece]);   // p0, p1, slot, t
        if (rec.z < 0)
            continue;                                           // merged into the piece that starts earlier
        const int p0 = rec.x, p1 = rec.y;
        const TableMeta m = a.meta[rec.w];
        const int64_t stride = a.table_major ? m.dim : a.sumD;
        const GT* gb = a.table_major ? grad_out + (int64_t)a.batch * m.col : grad_out + m.col;
        const Cols c(m.dim, m.lpr_bwd, lane);
        const int G = kWave >> c.lprl;
        float acc[2][4];
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc[k][x] = 0.f;
        for (int base = p0; base < p1; base += kWave) {
            const int cnt = min(kWave, p1 - base);
            const int myv = vals[min(base + lane, p1 - 1)];     // 64 payloads with one coalesced load
            for (int i0 = 0; i0 < cnt; i0 += G * kBwdUnroll) {
                typename GIO::Vec v[kBwdUnroll][2];
                const GT* rp[kBwdUnroll];
#pragma unroll
                for (int x = 0; x < kBwdUnroll; ++x) {
                    const int i = i0 + x * G + c.grp;
                    const int b = __shfl(myv, min(i, cnt - 1));
                    rp[x] = i < cnt ? gb + (int64_t)b * stride : zero_row;
                }
#pragma unroll
                for (int x = 0; x < kBwdUnroll; ++x) {
                    v[x][0] = GIO::ldv(rp[x] + c.e0);
                    v[x][1] = GIO::ldv(rp[x] + c.e1);
                }
#pragma unroll
                for (int x = 0; x < kBwdUnroll; ++x) {
                    GIO::add(acc[0], v[x][0]);
                    GIO::add(acc[1], v[x][1]);
                }
            }
        }
        for (int sft = 1 << c.lprl; sft < kWave; sft <<= 1) {
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    acc[k][x] += __shfl_xor(acc[k][x], sft);
        }
        store_partial(a.partials + (int64_t)rec.z * a.dpad, acc, c);
      }
    }
}

// One wavefront per queued long run: adds the run's partial rows in order (one per bag slice of a dense
// run, one per window piece otherwise) and applies the run's single optimizer step.
template <typename WT, typename GT, int OPT>
__global__ __launch_bounds__(kBwdThreads) void long_run_fixup_kernel(BwdArgs a)
{
    using IO = RowIO<WT, 4>;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_global = uniform(blockIdx.x * (kBwdThreads / kWave) + (threadIdx.x >> 6));
    const int wave_total = gridDim.x * (kBwdThreads / kWave);
    const int cnt = (int)a.counters->long_count;
    WT* __restrict__ weights = static_cast<WT*>(a.weights);
    float acc[2][4];
    for (int i = wave_global; i < cnt; i += wave_total) {
        const int u = (int)a.long_list[i];
        const int s = a.seg_offsets[u];
        const int e = a.seg_offsets[u + 1];
        const bool dense = e - s > a.dense_thr;
        const uint32_t key = a.unique_keys[u];
        const int t = find_table(a.row_base, a.T, key);
        const TableMeta m = a.meta[t];
        const Cols c(m.dim, m.lpr_bwd, lane);
        const int k0 = s / kChunk;
        const float* pbase = a.partials;
        const int64_t dpad = a.dpad;
        const int64_t wel = m.woff + (int64_t)(key - m.rbase) * m.dim;
        WT* wrow = weights + wel;
        typename IO::Vec wvv[2];
        wvv[0] = IO::ldv(wrow + c.e0);
        wvv[1] = IO::ldv(wrow + c.e1);
        OptRow<OPT> st;
        st.load(a.opt, key, wel, c);
        if (dense && a.dense_dirty[t] != 0u) {
            // the table's gradient block holds Inf / NaN, which the dense sums leave out: this run is
            // summed the plain way, one gathered gradient row per lookup (a rare, slow path)
            const GT* gb = a.table_major ? static_cast<const GT*>(a.grad_out) + (int64_t)a.batch * m.col
                                         : static_cast<const GT*>(a.grad_out) + m.col;
            const int64_t gstride = a.table_major ? m.dim : a.sumD;
            const int32_t* __restrict__ vals = a.sorted_vals;
            wave_gather_sum<GT>([&](int i) { return gb + (int64_t)vals[i] * gstride; }, s, e, a.zero_row, c, acc);
        } else if (dense) {
            // one partial row per slice of bags, kept in the slots of the chunks the run covers completely
            wave_gather_sum<float>([&](int cc) { return pbase + ((int64_t)(k0 + 1) * 2 + cc) * dpad; }, 0,
                                   a.dense_slices, a.zero_row, c, acc);
        } else {
            const int nwin = window_geom(a.batch, m.dim, a.grad_bytes).nwin;
            const int step = window_step(s, e, nwin);
            wave_gather_sum<float>([&](int cc) { return pbase + ((int64_t)(k0 + 1) * 2 + cc) * dpad; }, 0,
                                   (nwin + step - 1) / step, a.zero_row, c, acc);
        }
        optimizer_epilogue<WT, OPT>(wrow, wvv, acc, m.dim, c, c.grp == 0, a.opt, key, wel, st);
    }
    // Leave the queue empty for the next update launch.  Every wavefront read the count before its
    // loop (the loop bound depends on it), the barrier orders those reads before this workgroup's
    // arrival, and only the workgroup that arrives last -- after all others have arrived -- clears.
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t arrived = atomicAdd(&a.counters->fixup_done, 1u);
        if (arrived == gridDim.x - 1) {
            a.counters->long_count = 0;
            a.counters->fixup_done = 0;
        }
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

__global__ void clear_num_unique_kernel(Counters* counters) { counters->num_unique = 0; }

__global__ void clear_check_flags_kernel(Counters* counters) { counters->check_flags = 0; }

}  // namespace tbe
