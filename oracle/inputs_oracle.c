/*
 * CPU oracle for the input-side kernels that sit next to the embedding operator.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT: plain single-threaded loops written from the definitions
 * in arxiv 2104.05158, called only by tests; it shares no code with the HIP library.
 *
 *   - Section 7.1, combined input format: per-bag LENGTHS are shipped instead of offsets and the
 *     inputs of all tables are concatenated; the embedding kernel consumes offsets, i.e. the
 *     exclusive prefix sum of the lengths.
 *   - Section 7.1, table-wise sharding: after the two all-to-alls a worker holds lengths and
 *     indices in (W, T, B) order (source worker, local table, local batch) and must permute them
 *     to (T, W, B) so that each table sees its whole global batch contiguously.
 *   - Section 4 "Row-wise parallelism" + Section 7.1: a table is split by rows over W trainers and
 *     the indices of every bag are bucketized by owner.  Reading (the paper gives no formula): shard
 *     w of table t owns the contiguous rows [w*blk_t, (w+1)*blk_t) with blk_t = ceil(H_t / W);
 *     bucketized indices are LOCAL row ids (row - w*blk_t), keep their order inside the bag, and are
 *     emitted in (W, T, B) order -- exactly the order the next all-to-all ships and the permute
 *     above consumes.
 */
#include <stdint.h>
#include <stdlib.h>

/* offsets[0] = 0, offsets[i+1] = offsets[i] + lengths[i].  Returns -1 on a negative length. */
int oracle_lengths_to_offsets(const int32_t* lengths, int64_t n, int64_t* offsets)
{
    offsets[0] = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (lengths[i] < 0)
            return -1;
        offsets[i + 1] = offsets[i] + lengths[i];
    }
    return 0;
}

/*
 * Input bag (w,t,b) has id (w*T + t)*B + b; output bag (t,w,b) has id (t*W + w)*B + b.
 * lengths_out[(t,w,b)] = lengths_in[(w,t,b)], offsets_out = prefix sum, and the indices of each bag
 * move as a block, order kept.
 */
int oracle_permute_wtb_to_twb(int W, int T, int B, const int32_t* lengths_in, const int32_t* indices_in,
                              int32_t* lengths_out, int64_t* offsets_out, int32_t* indices_out)
{
    int64_t n = (int64_t)W * T * B;
    int64_t* in_off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (oracle_lengths_to_offsets(lengths_in, n, in_off)) {
        free(in_off);
        return -1;
    }
    for (int t = 0; t < T; ++t)
        for (int w = 0; w < W; ++w)
            for (int b = 0; b < B; ++b)
                lengths_out[((int64_t)t * W + w) * B + b] = lengths_in[((int64_t)w * T + t) * B + b];
    oracle_lengths_to_offsets(lengths_out, n, offsets_out);
    for (int t = 0; t < T; ++t)
        for (int w = 0; w < W; ++w)
            for (int b = 0; b < B; ++b) {
                int64_t src = ((int64_t)w * T + t) * B + b, dst = ((int64_t)t * W + w) * B + b;
                for (int64_t i = 0; i < lengths_in[src]; ++i)
                    indices_out[offsets_out[dst] + i] = indices_in[in_off[src] + i];
            }
    free(in_off);
    return 0;
}

/*
 * Input: T tables x B bags in table-major order (bag id t*B + b), indices/offsets as for the
 * embedding operator.  Output bag (w,t,b) has id (w*T + t)*B + b and holds, in input order, the
 * local row ids of the bag's indices owned by shard w.  Returns -2 on an index outside its table.
 */
int oracle_bucketize_rowwise(int T, int B, int W, const int64_t* rows, const int32_t* indices,
                             const int64_t* offsets, int32_t* lengths_out, int64_t* offsets_out,
                             int32_t* indices_out)
{
    int64_t n_out = (int64_t)W * T * B;
    for (int64_t i = 0; i < n_out; ++i)
        lengths_out[i] = 0;
    for (int t = 0; t < T; ++t) {
        int64_t blk = (rows[t] + W - 1) / W;
        for (int b = 0; b < B; ++b)
            for (int64_t p = offsets[(int64_t)t * B + b]; p < offsets[(int64_t)t * B + b + 1]; ++p) {
                int64_t r = indices[p];
                if (r < 0 || r >= rows[t])
                    return -2;
                lengths_out[((int64_t)(r / blk) * T + t) * B + b] += 1;
            }
    }
    oracle_lengths_to_offsets(lengths_out, n_out, offsets_out);
    int64_t* cursor = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_out > 0 ? n_out : 1));
    for (int64_t i = 0; i < n_out; ++i)
        cursor[i] = offsets_out[i];
    for (int t = 0; t < T; ++t) {
        int64_t blk = (rows[t] + W - 1) / W;
        for (int b = 0; b < B; ++b)
            for (int64_t p = offsets[(int64_t)t * B + b]; p < offsets[(int64_t)t * B + b + 1]; ++p) {
                int64_t r = indices[p];
                int64_t w = r / blk;
                indices_out[cursor[(w * T + t) * B + b]++] = (int32_t)(r - w * blk);
            }
    }
    free(cursor);
    return 0;
}
