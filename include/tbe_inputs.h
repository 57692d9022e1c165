/*
 * tbe_inputs.h -- C ABI of the input-side kernels that sit next to the embedding operator
 * (same shared library as tbe.h; gfx950 only).
 *
 * arxiv 2104.05158, Section 7.1: sparse inputs travel in a combined format (per-bag LENGTHS, all
 * tables concatenated); after the all-to-alls of table-wise sharding they arrive in (W, T, B) order
 * and must be permuted to (T, W, B) for the embedding kernel; for row-wise sharding (Section 4,
 * "Row-wise parallelism") the indices of every bag are bucketized by the trainer that owns the row.
 * The paper names custom GPU kernels for permute and bucketize; these are their single-GPU parts.
 *
 * Conventions: d_* are DEVICE pointers, everything else is HOST memory.  The functions only
 * enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = default stream), never
 * allocate and never synchronise.  Temporary storage is a caller-provided device scratch buffer of
 * at least tbe_inputs_scratch_bytes(n) bytes, 256-byte aligned, where n is the number of bags the
 * call handles (stated per function).  Every lengths and offsets array must be 16-byte aligned.
 * Integer results are exact and do not depend on scheduling.
 * Errors: TBE_ERR_INVALID_ARG (null pointer, negative size, scratch too small or misaligned),
 * TBE_ERR_UNSUPPORTED (sizes beyond the stated limits), TBE_ERR_HIP (launch failure).
 * Lengths must be >= 0 and indices valid rows; like the hot path these kernels do not validate
 * device data.
 */
#ifndef TBE_INPUTS_H_
#define TBE_INPUTS_H_

#include "tbe.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Scratch bytes needed by any function below when it handles num_bags bags. */
TBE_API size_t tbe_inputs_scratch_bytes(int64_t num_bags);

/*
 * Section 7.1, combined format: offsets are the exclusive prefix sum of the lengths.
 *   d_offsets[0] = 0, d_offsets[i+1] = d_offsets[i] + d_lengths[i],   i < num_bags
 * d_lengths int32[num_bags], d_offsets int64[num_bags+1].  num_bags < 2^31.
 */
TBE_API tbe_status_t tbe_lengths_to_offsets(const int32_t* d_lengths, int64_t num_bags, int64_t* d_offsets,
                                            void* d_scratch, size_t scratch_bytes, void* stream);

/*
 * tbe_lengths_to_offsets for callers that can neither allocate nor pass a scratch buffer: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * tbe_lengths_to_offsets, same kernels; the per-tile block sums of the scan live in a fixed 1 MiB
 * array inside the library's device image (one copy per GPU, held until the process ends), so the
 * call allocates nothing and takes no scratch argument.
 * Limit: num_bags <= tbe_lengths_to_offsets_noalloc_max_bags() (536,866,816); larger -> TBE_ERR_UNSUPPORTED.
 * All calls on one GPU share that array: two calls that overlap in time on the same GPU (different
 * streams, or different host threads) race and give wrong offsets; order them on one stream.
 * Nothing in the array has to start at zero (every entry that is read is written first by the same call).
 * Errors: TBE_ERR_INVALID_ARG as tbe_lengths_to_offsets, TBE_ERR_HIP if the array's address cannot be obtained.
 */
TBE_API tbe_status_t tbe_lengths_to_offsets_noalloc(const int32_t* d_lengths, int64_t num_bags,
                                                    int64_t* d_offsets, void* stream);
TBE_API int64_t tbe_lengths_to_offsets_noalloc_max_bags(void);

/*
 * Section 7.1: (W, T, B) -> (T, W, B).  Input bag (w,t,b) has id (w*T + t)*B + b, output bag
 * (t,w,b) has id (t*W + w)*B + b; every bag moves with its indices as a block, order kept:
 *   d_lengths_out[(t,w,b)] = d_lengths_in[(w,t,b)];  d_offsets_out = prefix sum of d_lengths_out;
 *   d_indices_out[d_offsets_out[(t,w,b)] + i] = d_indices_in[in_offset[(w,t,b)] + i].
 * d_lengths_in/out int32[W*T*B], d_offsets_out int64[W*T*B+1], d_indices_in/out int32[num_indices]
 * (num_indices = sum of the lengths, < 2^31).  Scratch for num_bags = W*T*B.
 */
TBE_API tbe_status_t tbe_permute_wtb_to_twb(int32_t W, int32_t T, int32_t B, const int32_t* d_lengths_in,
                                            const int32_t* d_indices_in, int64_t num_indices,
                                            int32_t* d_lengths_out, int64_t* d_offsets_out,
                                            int32_t* d_indices_out, void* d_scratch, size_t scratch_bytes,
                                            void* stream);

/*
 * Section 4 "Row-wise parallelism" / Section 7.1 bucketize.  Input: T tables x B bags, table-major
 * (bag id t*B + b), d_indices int32[num_indices], d_offsets int64[T*B+1] as for tbe_forward;
 * d_rows int64[T] (device) holds the table heights.  Table t is split over W shards in contiguous
 * row blocks of blk_t = ceil(rows[t] / W) (the paper gives no formula; this is the reading taken).
 * Output bag (w,t,b) has id (w*T + t)*B + b and receives, in input order, the LOCAL row ids
 * (row - w*blk_t) of the bag's indices owned by shard w:
 *   d_lengths_out int32[W*T*B], d_offsets_out int64[W*T*B+1], d_indices_out int32[num_indices].
 * The slice of shard w is a valid table-major (indices, offsets) input for that shard's operator.
 * Limits: 1 <= W <= 1024.  Scratch for num_bags = W*T*B.
 */
TBE_API tbe_status_t tbe_bucketize_rowwise(int32_t T, int32_t B, int32_t W, const int64_t* d_rows,
                                           const int32_t* d_indices, const int64_t* d_offsets,
                                           int64_t num_indices, int32_t* d_lengths_out,
                                           int64_t* d_offsets_out, int32_t* d_indices_out, void* d_scratch,
                                           size_t scratch_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TBE_INPUTS_H_ */
