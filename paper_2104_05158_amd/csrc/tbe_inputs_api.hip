// Host side of the input-side entry points declared in include/tbe_inputs.h: argument checks,
// scratch carve-up and launch sequences (arxiv 2104.05158, Section 7.1 and Section 4 "Row-wise
// parallelism").  Everything is enqueued on the caller's stream; nothing allocates or synchronises.
#include "tbe_inputs.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "tbe_inputs_kernels.hip.h"

using namespace tbe_in;

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

constexpr int64_t kMaxCount = ((int64_t)1 << 31) - 1;

struct Scratch {
    int64_t* offsets_in;   // int64[num_bags + 1]
    int64_t* block_sums;   // int64[tiles + 1]
};

size_t scratch_bytes(int64_t num_bags)
{
    const int64_t n = std::max<int64_t>(num_bags, 0);
    return align_up(8 * (size_t)(n + 1), 256) + align_up(8 * (size_t)(ceil_div(n, kScanTile) + 1), 256);
}

Scratch carve(void* d_scratch, int64_t num_bags)
{
    char* p = static_cast<char*>(d_scratch);
    Scratch s;
    s.offsets_in = reinterpret_cast<int64_t*>(p);
    s.block_sums = reinterpret_cast<int64_t*>(p + align_up(8 * (size_t)(std::max<int64_t>(num_bags, 0) + 1), 256));
    return s;
}

tbe_status_t check_scratch(const void* d_scratch, size_t bytes, int64_t num_bags)
{
    if (!d_scratch || misaligned(d_scratch, 256) || bytes < scratch_bytes(num_bags))
        return TBE_ERR_INVALID_ARG;
    return TBE_OK;
}

// Scratch of tbe_lengths_to_offsets_noalloc: the per-tile block sums of the scan live in this array
// instead of a caller-provided buffer.  Every GPU the library runs on holds its own copy at its own
// address; host code never uses the array's name as an address, only the pointer that
// hipGetSymbolAddress returned for the current device.
constexpr int64_t kNoAllocMaxTiles = 131071;                         // (1 MiB / 8) - 1 block sums
constexpr int64_t kNoAllocMaxBags = kNoAllocMaxTiles * kScanTile;    // 536,866,816 bags
static __device__ __align__(256) unsigned char scratch[(kNoAllocMaxTiles + 1) * 8];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of `scratch` on the current device (looked up once per device)
tbe_status_t noalloc_scratch(int64_t** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return TBE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return TBE_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<int64_t*>(g_scratch_ptr[dev]);
    return TBE_OK;
}

tbe_status_t launch_status()
{
    return hipGetLastError() == hipSuccess ? TBE_OK : TBE_ERR_HIP;
}

// offsets[0..n] = exclusive prefix sum of lengths[0..n)
tbe_status_t enqueue_scan(const int32_t* lengths, int64_t n, int64_t* offsets, int64_t* block_sums, hipStream_t st)
{
    if (n == 0) {
        hipLaunchKernelGGL(write_zero_offset_kernel, dim3(1), dim3(1), 0, st, offsets);
        return launch_status();
    }
    const int nb = (int)ceil_div(n, kScanTile);
    hipLaunchKernelGGL(scan64_reduce_kernel, dim3(nb), dim3(kThreads), 0, st, lengths, block_sums, n);
    hipLaunchKernelGGL(scan64_top_kernel, dim3(1), dim3(kThreads), 0, st, block_sums, nb);
    hipLaunchKernelGGL(scan64_apply_kernel, dim3(nb), dim3(kThreads), 0, st, lengths, block_sums, offsets, n);
    return launch_status();
}

}  // namespace

extern "C" {

size_t tbe_inputs_scratch_bytes(int64_t num_bags) { return scratch_bytes(num_bags); }

tbe_status_t tbe_lengths_to_offsets(const int32_t* d_lengths, int64_t num_bags, int64_t* d_offsets, void* d_scratch,
                                    size_t scratch_bytes_given, void* stream)
{
    if (num_bags < 0 || !d_offsets || (num_bags > 0 && !d_lengths) || misaligned(d_lengths, 16) ||
        misaligned(d_offsets, 16))
        return TBE_ERR_INVALID_ARG;
    if (num_bags > kMaxCount)
        return TBE_ERR_UNSUPPORTED;
    tbe_status_t rc = check_scratch(d_scratch, scratch_bytes_given, num_bags);
    if (rc != TBE_OK)
        return rc;
    const Scratch s = carve(d_scratch, num_bags);
    return enqueue_scan(d_lengths, num_bags, d_offsets, s.block_sums, static_cast<hipStream_t>(stream));
}

int64_t tbe_lengths_to_offsets_noalloc_max_bags(void) { return kNoAllocMaxBags; }

tbe_status_t tbe_lengths_to_offsets_noalloc(const int32_t* d_lengths, int64_t num_bags, int64_t* d_offsets,
                                            void* stream)
{
    if (num_bags < 0 || !d_offsets || (num_bags > 0 && !d_lengths) || misaligned(d_lengths, 16) ||
        misaligned(d_offsets, 16))
        return TBE_ERR_INVALID_ARG;
    if (num_bags > kNoAllocMaxBags)
        return TBE_ERR_UNSUPPORTED;
    int64_t* block_sums = nullptr;
    tbe_status_t rc = noalloc_scratch(&block_sums);
    if (rc != TBE_OK)
        return rc;
    // every block sum the scan reads is written by its first kernel in the same call: nothing has to be cleared
    return enqueue_scan(d_lengths, num_bags, d_offsets, block_sums, static_cast<hipStream_t>(stream));
}

tbe_status_t tbe_permute_wtb_to_twb(int32_t W, int32_t T, int32_t B, const int32_t* d_lengths_in,
                                    const int32_t* d_indices_in, int64_t num_indices, int32_t* d_lengths_out,
                                    int64_t* d_offsets_out, int32_t* d_indices_out, void* d_scratch,
                                    size_t scratch_bytes_given, void* stream)
{
    if (W < 1 || T < 1 || B < 0 || num_indices < 0 || !d_offsets_out)
        return TBE_ERR_INVALID_ARG;
    const int64_t n = (int64_t)W * T * B;
    if (n > kMaxCount || num_indices > kMaxCount || (int64_t)W * T > kMaxCount)
        return TBE_ERR_UNSUPPORTED;
    if ((n > 0 && (!d_lengths_in || !d_lengths_out)) || (num_indices > 0 && (!d_indices_in || !d_indices_out)) ||
        misaligned(d_lengths_in, 16) || misaligned(d_lengths_out, 16) || misaligned(d_offsets_out, 16))
        return TBE_ERR_INVALID_ARG;
    tbe_status_t rc = check_scratch(d_scratch, scratch_bytes_given, n);
    if (rc != TBE_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Scratch s = carve(d_scratch, n);
    if (n == 0)
        return enqueue_scan(d_lengths_out, 0, d_offsets_out, s.block_sums, st);
    rc = enqueue_scan(d_lengths_in, n, s.offsets_in, s.block_sums, st);
    if (rc != TBE_OK)
        return rc;
    const int vec = B % 4 == 0 ? 4 : 1;
    const int blocks_per_row = (int)ceil_div(B, kThreads * vec);
    const int64_t grid = (int64_t)W * T * blocks_per_row;
    if (grid > kMaxCount)
        return TBE_ERR_UNSUPPORTED;
    if (vec == 4)
        hipLaunchKernelGGL(permute_lengths_kernel<4>, dim3((unsigned)grid), dim3(kThreads), 0, st, d_lengths_in,
                           d_lengths_out, W, T, B, blocks_per_row);
    else
        hipLaunchKernelGGL(permute_lengths_kernel<1>, dim3((unsigned)grid), dim3(kThreads), 0, st, d_lengths_in,
                           d_lengths_out, W, T, B, blocks_per_row);
    rc = enqueue_scan(d_lengths_out, n, d_offsets_out, s.block_sums, st);
    if (rc != TBE_OK)
        return rc;
    if (num_indices > 0) {
        hipLaunchKernelGGL(permute_indices_kernel, dim3((unsigned)ceil_div(num_indices, kCopyTile)), dim3(kThreads),
                           0, st, d_indices_in, s.offsets_in, d_offsets_out, d_indices_out, W, T, B, num_indices);
    }
    return launch_status();
}

tbe_status_t tbe_bucketize_rowwise(int32_t T, int32_t B, int32_t W, const int64_t* d_rows, const int32_t* d_indices,
                                   const int64_t* d_offsets, int64_t num_indices, int32_t* d_lengths_out,
                                   int64_t* d_offsets_out, int32_t* d_indices_out, void* d_scratch,
                                   size_t scratch_bytes_given, void* stream)
{
    if (T < 1 || B < 0 || W < 1 || num_indices < 0 || !d_rows || !d_offsets || !d_offsets_out)
        return TBE_ERR_INVALID_ARG;
    const int64_t n_in = (int64_t)T * B;
    const int64_t n_out = n_in * W;
    if (W > kMaxShards || n_out > kMaxCount || num_indices > kMaxCount)
        return TBE_ERR_UNSUPPORTED;
    if ((n_out > 0 && !d_lengths_out) || (num_indices > 0 && (!d_indices || !d_indices_out)) ||
        misaligned(d_lengths_out, 16) || misaligned(d_offsets_out, 16))
        return TBE_ERR_INVALID_ARG;
    tbe_status_t rc = check_scratch(d_scratch, scratch_bytes_given, n_out);
    if (rc != TBE_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Scratch s = carve(d_scratch, n_out);
    if (n_out == 0)
        return enqueue_scan(d_lengths_out, 0, d_offsets_out, s.block_sums, st);
    int wbits = 0;
    while ((1 << wbits) < W)
        ++wbits;
    // bags per workgroup: the LDS count table holds W * nbags <= 8192 entries; small batches get
    // fewer bags per workgroup so that the grid still fills the chip
    int nbags = std::min<int>(kBuckMaxBags, 8192 / W);
    while (nbags > 8 && n_in / nbags < 2048)
        nbags >>= 1;
    const unsigned grid = (unsigned)ceil_div(n_in, nbags);
    hipLaunchKernelGGL(bucketize_count_kernel, dim3(grid), dim3(kThreads), 0, st, d_rows, d_indices, d_offsets,
                       d_lengths_out, T, B, W, (int32_t)n_in, nbags);
    rc = enqueue_scan(d_lengths_out, n_out, d_offsets_out, s.block_sums, st);
    if (rc != TBE_OK)
        return rc;
    if (num_indices > 0) {
        if (W <= 32)
            hipLaunchKernelGGL(bucketize_place_kernel<32>, dim3(grid), dim3(kThreads), 0, st, d_rows, d_indices,
                               d_offsets, d_offsets_out, d_indices_out, T, B, W, wbits, (int32_t)n_in, nbags);
        else
            hipLaunchKernelGGL(bucketize_place_kernel<kMaxShards>, dim3(grid), dim3(kThreads), 0, st, d_rows,
                               d_indices, d_offsets, d_offsets_out, d_indices_out, T, B, W, wbits, (int32_t)n_in,
                               nbags);
    }
    return launch_status();
}

}  // extern "C"
