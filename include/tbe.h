/*
 * tbe.h -- C ABI of the MI355X (gfx950) table-batched embedding-bag library.
 *
 * The operator is the embedding part of DLRM training as arxiv 2104.05158 states it:
 *   - Section 2 "Embedding operators" (Fig. 2): each index of a multi-hot input fetches a full
 *     table row; the rows of one input ("bag") are combined by element-wise pooling (sum here).
 *   - Section 5.1 (Fig. 6a): the lookups of ALL tables placed on a GPU run as one fused kernel.
 *   - Section 5.1 (Fig. 6b): the backward pass is fused with the sparse optimizer; gradients are
 *     sorted by row so that every gradient of one embedding row meets in one place, is aggregated
 *     on chip, and the (non-linear) optimizer is applied once per touched row.  No gradient
 *     tensor of the tables is ever materialised.
 *   - Section 5.2: row-wise sparse AdaGrad, one moment scalar per table row.
 *   - Section 7.1: input is the nn.EmbeddingBag (indices, offsets) pair, all tables concatenated
 *     in table-major order (the "(T, W, B)" order the embedding kernel consumes).
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (HIP global memory); every other pointer is HOST memory.
 *   - The library owns only its host-side handle.  Weights, optimizer state, workspace, inputs and
 *     outputs are allocated by the caller and merely borrowed between tbe_bind and tbe_destroy.
 *     The library never allocates or frees device memory.
 *   - tbe_forward / tbe_backward_rowwise_adagrad only enqueue kernels on the given stream and
 *     return; they never synchronise.  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  tbe_bind, tbe_check_inputs and tbe_profile_read synchronise.
 *   - A handle is used from one host thread at a time; distinct handles are independent.  Two calls
 *     that use the same handle (hence the same workspace) must be ordered on one stream.
 *   - Every function returns a tbe_status_t; nothing throws, nothing aborts.  Errors detectable
 *     on the host (null pointers, sizes beyond what tbe_create was told, unbound handle) are
 *     reported before anything is enqueued.
 *
 * Data layout
 *   bag id            j = t * batch + b          (table-major)
 *   d_indices         int32[num_indices]; the lookups of bag j are positions
 *                     [d_offsets[j], d_offsets[j+1]); each value is a row of table t, 0 <= row < rows[t]
 *   d_offsets         int64[num_tables*batch + 1], non-decreasing, first 0, last num_indices
 *   weights           one flat array in the storage type; table t is the row-major block of
 *                     rows[t] x dims[t] elements starting at element weight_offsets[t]
 *   state             float32; row-wise AdaGrad: the moment of row r of table t is element
 *                     state_offsets[t] + r (other optimizers: see tbe_config_t)
 *   output / grad     [batch, sum_t dims[t]] row-major, float32 unless configured otherwise; table t owns columns
 *                     [out_col_offsets[t], out_col_offsets[t] + dims[t]).  TBE_LAYOUT_TABLE_MAJOR stores the
 *                     same values as one [batch, dims[t]] block per table instead.
 *   linear row id     key = state_offsets[t] + row  (uint32; the sort key of the backward pass)
 */
#ifndef TBE_H_
#define TBE_H_

#include <stddef.h>
#include <stdint.h>

#if defined(TBE_BUILDING)
#define TBE_API __attribute__((visibility("default")))
#else
#define TBE_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tbe_s* tbe_handle_t;

typedef enum {
    TBE_OK = 0,
    TBE_ERR_INVALID_ARG = 1,
    TBE_ERR_UNSUPPORTED = 2,
    TBE_ERR_NOT_BOUND = 3,
    TBE_ERR_WORKSPACE_TOO_SMALL = 4,
    TBE_ERR_INDEX_OUT_OF_RANGE = 5,
    TBE_ERR_HIP = 6
} tbe_status_t;

enum { TBE_DTYPE_FP32 = 0, TBE_DTYPE_FP16 = 1, TBE_DTYPE_BF16 = 2 };
enum { TBE_POOLING_SUM = 0 };
/* Sparse optimizer fused into the backward pass.  Section 5.2 describes the row-wise AdaGrad;
 * Section 5.1 names (element-wise) AdaGrad and Adam as further non-linear optimizers it serves. */
enum { TBE_OPT_ROWWISE_ADAGRAD = 0, TBE_OPT_ADAGRAD = 1, TBE_OPT_ADAM = 2 };
/* Layout of d_out and d_grad_out.  BATCH_MAJOR: one row of sumD values per sample, table t in columns
 * [c_t, c_t + D_t) -- what a sample's feature interaction consumes.  TABLE_MAJOR: one contiguous
 * [batch, D_t] block per table, table t's block starting at element batch * c_t (batch = the call's
 * batch, not max_batch) -- what a table-wise all-to-all ships per table.  The values are the same. */
enum { TBE_LAYOUT_BATCH_MAJOR = 0, TBE_LAYOUT_TABLE_MAJOR = 1 };

typedef struct {
    int32_t num_tables;     /* T >= 1 */
    const int64_t* rows;    /* host int64[T], each in [1, 2^31), sum < 2^32 - 1 */
    const int32_t* dims;    /* host int32[T], each a multiple of 4 in [4, 512] (Table 3 reports 4..384) */
    int32_t weight_dtype;   /* TBE_DTYPE_FP32, or TBE_DTYPE_FP16 storage with fp32 accumulation */
    int32_t pooling;        /* TBE_POOLING_SUM is the only mode */
    int32_t max_batch;      /* largest `batch` any later call will pass; T*max_batch < 2^31 */
    int64_t max_indices;    /* largest `num_indices` any later call will pass; < 2^31 - 2^24 */
    int32_t optimizer;      /* TBE_OPT_*: fixes the size of the state buffer and which backward entry points apply */
    int32_t output_dtype;   /* type of d_out: TBE_DTYPE_FP32, or TBE_DTYPE_FP16 (fp32 sums rounded to nearest even) */
    int32_t grad_dtype;     /* type of d_grad_out: TBE_DTYPE_FP32, TBE_DTYPE_FP16 or TBE_DTYPE_BF16; sums stay fp32 */
    int32_t layout;         /* TBE_LAYOUT_*: layout of d_out and d_grad_out */
} tbe_config_t;
/* The 16-bit output / gradient types follow Section 8.4: the pooled embeddings leave the operator
 * through an FP16 all-to-all and their gradients come back through a BF16 one, so that precision is
 * all that is there to consume.  Optimizer state (float32, zero-filled by the caller before step 1):
 *   TBE_OPT_ROWWISE_ADAGRAD  one moment per table row (linear row id)                 4 * sum_t rows[t]
 *   TBE_OPT_ADAGRAD          one sum of squares per weight element (weight layout)     4 * sum_t rows[t]*dims[t]
 *   TBE_OPT_ADAM             first moments of all elements, then all second moments    8 * sum_t rows[t]*dims[t] */

/*
 * Creates a handle (host only; copies the config arrays).  Section 5.1: one handle stands for all
 * tables that are fused into one operator on this GPU.
 * Errors: INVALID_ARG (null, T < 1, rows/dims not positive, negative sizes),
 *         UNSUPPORTED (dim not a multiple of 4 or > 512, a table of 2^31 rows or more (indices are int32),
 *         sum of rows >= 2^32 - 1, sizes too large,
 *         unknown dtype/pooling/optimizer/layout, BF16 tables or BF16 output).
 */
TBE_API tbe_status_t tbe_create(const tbe_config_t* cfg, tbe_handle_t* out_handle);

/* Frees the host handle.  Device buffers stay with the caller.  NULL is accepted. */
TBE_API tbe_status_t tbe_destroy(tbe_handle_t h);

/*
 * Sizes (bytes) of the three device buffers the caller must provide, and the layout tables
 * described above.  Any output pointer may be NULL.  weight_offsets / state_offsets are host
 * int64[T+1] in ELEMENTS, out_col_offsets is host int32[T+1].  state_offsets are the linear row
 * ids of the tables' first rows (the index of the row-wise moments and the base of the sort keys);
 * per-element optimizer states are indexed by weight_offsets.
 */
TBE_API tbe_status_t tbe_query_sizes(tbe_handle_t h, size_t* weight_bytes, size_t* state_bytes,
                             size_t* workspace_bytes, int64_t* weight_offsets,
                             int64_t* state_offsets, int32_t* out_col_offsets);

/*
 * Lends the device buffers to the handle and uploads the table metadata into the head of the
 * workspace (synchronous copy).  d_weights: storage type, weight_bytes; d_state: float32 optimizer
 * state, state_bytes, zero-filled by the caller before the first step (Section 5.2 keeps one moment
 * per row; its start value is not given, 0 is used); d_workspace: at least workspace_bytes,
 * 256-byte aligned.  Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, HIP.
 */
TBE_API tbe_status_t tbe_bind(tbe_handle_t h, void* d_weights, float* d_state, void* d_workspace,
                      size_t workspace_bytes);

/*
 * Forward (Section 2 "Embedding operators", fused over tables per Section 5.1):
 *   d_out[b, c_t + d] = sum_{p in bag (t,b)} W_t[d_indices[p], d]      accumulated in fp32
 * One kernel launch for all tables.  An empty bag pools to 0.  Indices are assumed valid
 * (see tbe_check_inputs).  d_out holds batch * sumD elements of the configured output type in the
 * configured layout and is written completely.
 * Errors: NOT_BOUND, INVALID_ARG (null, batch < 0 or > max_batch, num_indices < 0 or > max_indices), HIP.
 */
TBE_API tbe_status_t tbe_forward(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                         int64_t num_indices, int32_t batch, void* d_out, void* stream);

/*
 * Backward fused with row-wise AdaGrad, in place (Sections 5.1 and 5.2).  With
 *   G[t,r,:] = sum over every lookup p of the batch with d_indices[p] == r in table t of
 *              d_grad_out[b(p), c_t : c_t + D_t]
 * each touched row gets exactly one optimizer step
 *   m[t,r]  += (1/D_t) * sum_d G[t,r,d]^2
 *   W_t[r,:] -= lr * G[t,r,:] / (sqrt(m[t,r]) + eps)
 * computed in fp32 and rounded to the storage type (nearest even).  Rows not looked up are not
 * written.  Implementation: the lookups are radix-sorted by (table, row) (stable; the sort is
 * segmented by table and reads the caller's indices directly) and run-length segmented in the
 * workspace, then every run is reduced on chip and its row updated once.
 * The integer artefacts stay in the workspace until the next backward call (tbe_backward_artifacts).
 * d_grad_out holds batch * sumD elements of the configured gradient type, laid out like d_out.
 * Errors: as tbe_forward; INVALID_ARG if the handle was created for another optimizer.
 */
TBE_API tbe_status_t tbe_backward_rowwise_adagrad(tbe_handle_t h, const int32_t* d_indices,
                                          const int64_t* d_offsets, int64_t num_indices,
                                          int32_t batch, const void* d_grad_out, float lr,
                                          float eps, void* stream);

/*
 * The same fused backward with the other optimizers Section 5.1 names; G is aggregated exactly as
 * above and every touched row gets one step, element by element (d over the row's columns):
 *   AdaGrad   S[t,r,d] += G_d^2;   W_t[r,d] -= lr * G_d / (sqrt(S[t,r,d]) + eps)
 *   Adam      m = beta1*m + (1-beta1)*G_d;   v = beta2*v + (1-beta2)*G_d^2;
 *             W_t[r,d] -= lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps)
 * Adam is the lazy sparse form: rows that the batch does not look up keep weights and moments;
 * `step` >= 1 is the caller's global iteration count (bias correction).  The paper gives no
 * formulas for these; they are the textbook rules with the conventions of the row-wise form
 * (updated state scales the step, eps outside the root, states start at 0).
 * Errors: as above; Adam with step < 1 or beta outside [0,1) returns INVALID_ARG.
 */
TBE_API tbe_status_t tbe_backward_adagrad(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                          int64_t num_indices, int32_t batch, const void* d_grad_out, float lr,
                                          float eps, void* stream);
TBE_API tbe_status_t tbe_backward_adam(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                       int64_t num_indices, int32_t batch, const void* d_grad_out, float lr,
                                       float beta1, float beta2, float eps, int64_t step, void* stream);

/*
 * The same backward pass in two calls, for callers that overlap work (Section 4.2 pipelines
 * independent stages on separate streams).  tbe_backward_sort enqueues the part that needs only the
 * batch's (indices, offsets): sort plan, radix sort, run-length segmentation (Section 5.1 "gradient
 * sorting by rows"); it may run on another stream, concurrently with tbe_forward or with dense
 * layers.  tbe_backward_update_<optimizer> enqueues the aggregation + optimizer step
 * (Sections 5.1, 5.2) for the batch sorted last; the caller must order it after that sort (same
 * stream, or an event) and must not start the next sort of this handle before it has finished:
 * both use the handle's workspace.  tbe_backward_<optimizer> is exactly these two in a row.
 * An update may be repeated for the same sort (each call applies one more optimizer step for that
 * batch with the gradient it is given); the sort's artefacts are not consumed.
 * Errors: as tbe_forward; update without a preceding sort returns INVALID_ARG.
 */
TBE_API tbe_status_t tbe_backward_sort(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                       int64_t num_indices, int32_t batch, void* stream);
TBE_API tbe_status_t tbe_backward_update_rowwise_adagrad(tbe_handle_t h, const void* d_grad_out, float lr,
                                                         float eps, void* stream);
TBE_API tbe_status_t tbe_backward_update_adagrad(tbe_handle_t h, const void* d_grad_out, float lr, float eps,
                                                 void* stream);
TBE_API tbe_status_t tbe_backward_update_adam(tbe_handle_t h, const void* d_grad_out, float lr, float beta1,
                                              float beta2, float eps, int64_t step, void* stream);

/*
 * Device pointers (into the workspace) of the last backward call's integer artefacts
 * (Section 5.1 "gradient sorting by rows"), valid once that call's stream work has completed:
 *   d_sorted_keys  uint32[num_indices]  linear row ids, ascending
 *   d_sorted_vals  int32[num_indices]   bag position b of each sorted lookup; equal keys keep input order
 *   d_unique_keys  uint32[U]            distinct keys, ascending
 *   d_seg_offsets  int32[U+1]           run u = sorted positions [seg_offsets[u], seg_offsets[u+1])
 *   d_num_unique   int64[1]             U
 * Any output pointer may be NULL.  Errors: NOT_BOUND, INVALID_ARG (no backward call yet).
 */
TBE_API tbe_status_t tbe_backward_artifacts(tbe_handle_t h, const uint32_t** d_sorted_keys,
                                    const int32_t** d_sorted_vals, const uint32_t** d_unique_keys,
                                    const int32_t** d_seg_offsets, const int64_t** d_num_unique);

/*
 * Slow, synchronising validator of a batch: offsets start at 0, never decrease and end at
 * num_indices; every index lies inside its table.  Returns INDEX_OUT_OF_RANGE or INVALID_ARG
 * (bad offsets) instead of letting the hot path read out of bounds.  It keeps its result flag in a
 * workspace word of its own and touches nothing else there, so it may be called between
 * tbe_backward_sort and the update; like every call on a handle it must be ordered on the stream
 * with the handle's other work.
 */
TBE_API tbe_status_t tbe_check_inputs(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                              int64_t num_indices, int32_t batch, void* stream);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream around every kernel the
 * entry points enqueue.  max_calls > 0 enables it and sizes the event pool (calls beyond it are
 * not timed); 0 disables it and drops the pool.
 */
TBE_API tbe_status_t tbe_profile_enable(tbe_handle_t h, int32_t max_calls);

/*
 * Synchronises the recorded events and returns, per kernel slot, the number of timed launches and
 * their total duration in milliseconds since the last read; then resets the pool.  names receives
 * pointers to static strings.  capacity = length of the three host arrays; *num_slots = entries filled.
 */
TBE_API tbe_status_t tbe_profile_read(tbe_handle_t h, int32_t capacity, const char** names,
                              int64_t* launches, double* total_ms, int32_t* num_slots);

/*
 * Measurement aid (Appendix A measures its kernels against the bandwidth the machine reaches): enqueues one
 * kernel that reads the first bytes / 16 * 16 bytes of d_src `passes` times with coalesced 16-byte loads and
 * discards them.  d_src: device memory, 16-byte aligned, at least 16 bytes; d_sink: 4 bytes of device memory
 * (practically never written); both stay the caller's.  Timed by the caller (events on `stream`): bytes x
 * passes / duration is the read rate of the memory level the buffer fits in.  No handle, no allocation.
 * Errors: TBE_ERR_INVALID_ARG (null or misaligned pointer, bytes < 16, passes < 1), TBE_ERR_HIP.
 */
TBE_API tbe_status_t tbe_probe_read(const void* d_src, size_t bytes, int32_t passes, void* d_sink, void* stream);

TBE_API const char* tbe_status_string(tbe_status_t s);

/* Text of the last HIP error seen by this handle ("" if none); valid until the next call. */
TBE_API const char* tbe_last_hip_error(tbe_handle_t h);

#ifdef __cplusplus
}
#endif
#endif /* TBE_H_ */
