// Host side of the table-batched embedding-bag library: handle, workspace carve-up, launch
// geometry and the extern "C" entry points declared in include/tbe.h.
//
// Section 5.1 of arxiv 2104.05158 asks for one forward launch and one fused backward+optimizer
// step for all tables of a GPU; here the forward is literally one kernel and the backward is a
// fixed sequence (sort plan, radix sort passes, run-length, fused reduce+optimizer, long-run fix-up)
// enqueued on the caller's stream without any host synchronisation.
#include "tbe.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "tbe_kernels.hip.h"

using namespace tbe;

namespace {

enum Slot {
    SLOT_FORWARD = 0,
    SLOT_SORT_PLAN,
    SLOT_RADIX_HIST,
    SLOT_RADIX_SCAN,
    SLOT_RADIX_SCATTER,
    SLOT_RUNLENGTH,
    SLOT_REDUCE_UPDATE,
    SLOT_WINDOW_RUNS,
    SLOT_DENSE_ROWS,
    SLOT_LONG_FIXUP,
    SLOT_COUNT
};
const char* const kSlotNames[SLOT_COUNT] = {"forward",       "sort_plan",  "radix_hist",    "radix_scan",
                                            "radix_scatter", "runlength",  "reduce_update", "window_runs", "dense_rows", "long_fixup"};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
constexpr int kDenseGrid = 1024;
constexpr int kWindowGrid = 1024;  // persistent workgroups of window_runs_kernel: 8 wavefronts per CU, a multiple of 8
constexpr int kDenseBagsPerLookup = 8;   // persistent workgroups of dense_rows_kernel: 4 per CU, a multiple of 8

inline int pow2ceil_log2(int x)
{
    int l = 0;
    while ((1 << l) < x)
        ++l;
    return l;
}

struct ProfRec {
    int slot;
    hipEvent_t start, stop;
};

}  // namespace

struct tbe_s {
    int T = 0;
    std::vector<int64_t> rows;
    std::vector<int32_t> dims;
    int dtype = 0;
    int optimizer = 0;
    int out_dtype = 0;
    int grad_dtype = 0;
    int layout = 0;
    int64_t weight_elems = 0;
    int max_batch = 0;
    int64_t max_indices = 0;
    int64_t sumD = 0;
    int dmax = 0;
    int fwd_epl = 4;
    int fwd_kmax = 1;
    int key_bits = 1;                   // bits of the tallest table's row index
    std::vector<int> pass_digit_bits;   // per sort launch: the widest digit any table sorts in it
    std::vector<int64_t> woff;      // T+1, elements
    std::vector<int64_t> soff;      // T+1, rows
    std::vector<int32_t> coloff;    // T+1
    std::vector<TableMeta> meta;

    // workspace layout (byte offsets)
    size_t off_meta = 0, off_rowbase = 0, off_counters = 0, off_keys[2] = {0, 0}, off_vals[2] = {0, 0};
    size_t off_tile_base = 0, off_tstart = 0, off_tile_table = 0;
    int64_t max_tiles = 1;
    size_t off_hist = 0, off_scan_tmp = 0, off_rl_counts = 0, off_chunk_first = 0, off_partials = 0;
    size_t off_long_list = 0, off_zero = 0, workspace_bytes = 0;
    size_t off_win_cnt = 0, off_win_list = 0, off_wrun = 0, off_wbounds = 0;
    size_t off_dense_dirty = 0, off_dense_cnt = 0, off_dense_list = 0, off_drun = 0, off_dgroup = 0, off_dbounds = 0;
    int64_t dbounds_cap = 0;   // entries
    size_t weight_bytes = 0, state_bytes = 0;

    // bound buffers
    void* d_weights = nullptr;
    float* d_state = nullptr;
    char* d_ws = nullptr;
    bool bound = false;
    int final_buf = -1;  // which (keys, vals) pair holds the sorted result of the last backward
    int32_t sorted_n = -1, sorted_batch = 0;  // size of the batch that was sorted last

    // profiling
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    std::vector<ProfRec> recs;
    bool profiling = false;

    std::string last_hip_error;

    template <typename P>
    P* ws(size_t off) const
    {
        return reinterpret_cast<P*>(d_ws + off);
    }
};

namespace {

struct ScopedTimer {
    tbe_s* h;
    hipStream_t st;
    ProfRec rec;
    bool on = false;
    ScopedTimer(tbe_s* h_, int slot, hipStream_t st_) : h(h_), st(st_)
    {
        if (h->profiling && h->ev_used + 2 <= h->ev_pool.size()) {
            rec.slot = slot;
            rec.start = h->ev_pool[h->ev_used++];
            rec.stop = h->ev_pool[h->ev_used++];
            on = hipEventRecord(rec.start, st) == hipSuccess;
        }
    }
    ~ScopedTimer()
    {
        if (on && hipEventRecord(rec.stop, st) == hipSuccess)
            h->recs.push_back(rec);
    }
};

tbe_status_t hip_fail(tbe_s* h, hipError_t e, const char* what)
{
    if (h)
        h->last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return TBE_ERR_HIP;
}

#define TBE_HIP_CHECK(h, expr)                     \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess)                      \
            return hip_fail((h), e_, #expr);       \
    } while (0)

#define TBE_LAUNCH_CHECK(h, what)                  \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess)                      \
            return hip_fail((h), e_, what);        \
    } while (0)

// Dense hot rows: the run-length threshold for a call with `batch` bags per table.  One lookup per
// kDenseBagsPerLookup bags is where summing counts x gradient block pays (measured on configurations 2-4:
// with 8 a table's first group of 32 runs saves twice what it costs, a second group costs more than it
// saves); the third term keeps the partial rows of a dense run (one per kDenseSlice bags) inside the slots
// of the chunks that run covers completely (two per chunk).
int dense_threshold(int64_t batch)
{
    const int64_t nslices = ceil_div(std::max<int64_t>(batch, 1), kDenseSlice);
    return (int)std::max<int64_t>({kDenseMinRun, batch / kDenseBagsPerLookup, (int64_t)kChunk * ((nslices + 1) / 2 + 3)});
}

// entries of the bounds table a call with n lookups and `batch` bags per table can need
int64_t dense_bounds_entries(int64_t n, int64_t batch, int T)
{
    if (batch <= 0)
        return 0;
    const int64_t runs = n / dense_threshold(batch) + 1;
    return runs * (ceil_div(batch, kDenseSlice) + 1);
}

void plan_workspace(tbe_s* h)
{
    const int64_t nmax = h->max_indices;
    const int64_t bags = (int64_t)h->T * h->max_batch;
    (void)bags;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    h->off_meta = take(sizeof(TableMeta) * (size_t)h->T);
    h->off_rowbase = take(sizeof(uint32_t) * (size_t)(h->T + 1));
    h->off_counters = take(sizeof(Counters));
    h->off_zero = take(kZeroRowBytes);
    const size_t nelem = (size_t)nmax + 64;  // +1 for seg_offsets' sentinel, rounded
    for (int i = 0; i < 2; ++i) {
        h->off_keys[i] = take(4 * nelem);
        h->off_vals[i] = take(4 * nelem);
    }
    // tiles never cross a table border: at most one partly filled tile per table on top of nmax / tile
    h->max_tiles = ceil_div(nmax, kSortTile) + h->T;
    h->off_tile_base = take(4 * (size_t)(h->T + 1));
    h->off_tstart = take(4 * (size_t)(h->T + 1));
    h->off_tile_table = take(sizeof(TileDesc) * (size_t)h->max_tiles);
    const int64_t hist_len = 256 * h->max_tiles;
    h->off_hist = take(4 * (size_t)hist_len);
    const int64_t rl_tiles = std::max<int64_t>(1, ceil_div(nmax, kRlTile));
    const int64_t scan_blocks = std::max(ceil_div(hist_len, kScanTile), ceil_div(rl_tiles, kScanTile));
    h->off_scan_tmp = take(4 * (size_t)(scan_blocks + 1));
    h->off_rl_counts = take(4 * (size_t)(rl_tiles + 16));
    const int64_t chunks = std::max<int64_t>(1, ceil_div(nmax, kChunk));
    h->off_chunk_first = take(4 * (size_t)(chunks + 1));
    const int dpad = (int)align_up((size_t)h->dmax, 4);
    h->off_partials = take(4 * (size_t)chunks * 2 * (size_t)dpad);
    h->off_long_list = take(4 * (size_t)(nmax / kLongRun + 2));
    // dense hot rows: per-table queues, compact run list, groups, and the runs' positions at every
    // kDenseSlice-th bag.  The threshold is never below kDenseMinRun, which bounds the number of dense runs.
    const int64_t dense_runs_max = nmax / kDenseMinRun + h->T + 2;
    h->off_dense_cnt = take(4 * (size_t)h->T);
    h->off_dense_dirty = take(4 * (size_t)h->T);
    h->off_dense_list = take(4 * (size_t)dense_runs_max);
    h->off_drun = take(4 * (size_t)dense_runs_max);
    h->off_dgroup = take(sizeof(DenseGroup) * (size_t)(dense_runs_max / kDenseRows + h->T + 1));
    h->dbounds_cap = 0;
    for (int64_t b = 1;; b *= 2) {     // the need is largest at one end of a range of batch sizes: probe them all
        const int64_t bb = std::min<int64_t>(b, h->max_batch);
        for (int64_t cand : {bb, std::min<int64_t>(h->max_batch, 12288), std::min<int64_t>(h->max_batch, 3 * bb / 2)})
            h->dbounds_cap = std::max(h->dbounds_cap, dense_bounds_entries(nmax, cand, h->T));
        if (b >= h->max_batch)
            break;
    }
    h->off_dbounds = take(4 * (size_t)h->dbounds_cap);
    // long runs below the dense threshold: per-table queues, the prefix of their lengths, and the runs' piece records
    const int64_t win_runs_max = nmax / kLongRun + h->T + 2;
    h->off_win_cnt = take(4 * (size_t)h->T);
    h->off_win_list = take(4 * (size_t)win_runs_max);
    h->off_wrun = take(4 * 2 * (size_t)(h->T + 1));   // prefixes of the per-table queue lengths and piece counts
    h->off_wbounds = take(sizeof(WinPiece) * (size_t)win_runs_max * kWinMax);   // the runs' piece records
    h->workspace_bytes = off;
}

// exclusive scan of a uint32 device array in place (three launches)
tbe_status_t device_scan(tbe_s* h, uint32_t* data, int64_t n, int64_t* total_out, hipStream_t st)
{
    if (n <= 0)
        return TBE_OK;
    const int nb = (int)ceil_div(n, kScanTile);
    uint32_t* tmp = h->ws<uint32_t>(h->off_scan_tmp);
    hipLaunchKernelGGL(scan_reduce_kernel, dim3(nb), dim3(kScanThreads), 0, st, data, tmp, n);
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(kScanThreads), 0, st, tmp, nb, total_out);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(nb), dim3(kScanThreads), 0, st, data, tmp, n);
    TBE_LAUNCH_CHECK(h, "device_scan");
    return TBE_OK;
}

tbe_status_t check_call(tbe_s* h, const void* d_indices, const void* d_offsets, int64_t num_indices,
                        int32_t batch)
{
    if (!h)
        return TBE_ERR_INVALID_ARG;
    if (!h->bound)
        return TBE_ERR_NOT_BOUND;
    if (!d_offsets || batch < 0 || batch > h->max_batch || num_indices < 0 ||
        num_indices > h->max_indices || (num_indices > 0 && !d_indices))
        return TBE_ERR_INVALID_ARG;
    return TBE_OK;
}

template <typename WT, typename OT>
tbe_status_t launch_forward(tbe_s* h, const int32_t* idx, const int64_t* off, int32_t n_total, int32_t batch,
                            OT* out, hipStream_t st)
{
    const int num_bags = h->T * batch;
    // bags per wavefront: enough to amortise the per-block prologue, few enough to keep >= ~16k
    // wavefronts in the grid when the batch is small
    const int bpw = (int)std::min<int64_t>(kFwdMaxBagsPerWave, std::max<int64_t>(1, num_bags / 16384));
    const int per_block = (kFwdThreads / kWave) * bpw;
    const dim3 grid((unsigned)ceil_div(num_bags, per_block)), block(kFwdThreads);
    const TableMeta* meta = h->ws<TableMeta>(h->off_meta);
    const WT* w = static_cast<const WT*>(h->d_weights);
    const int sumD = (int)h->sumD;
    const void* zero = h->ws<void>(h->off_zero);
#define FWD(EPL, KMAX)                                                                              \
    hipLaunchKernelGGL((forward_kernel<WT, EPL, KMAX, OT>), grid, block, 0, st, meta, w, idx, off, out, \
                       zero, batch, num_bags, sumD, n_total, bpw, h->layout)
    if constexpr (sizeof(WT) == 4) {
        if (h->fwd_kmax == 1)
            FWD(4, 1);
        else
            FWD(4, 2);
    } else {
        if (h->fwd_epl == 8)
            FWD(8, 1);
        else if (h->fwd_kmax == 1)
            FWD(4, 1);
        else
            FWD(4, 2);
    }
#undef FWD
    TBE_LAUNCH_CHECK(h, "forward_kernel");
    return TBE_OK;
}

}  // namespace

extern "C" {

const char* tbe_status_string(tbe_status_t s)
{
    switch (s) {
        case TBE_OK: return "ok";
        case TBE_ERR_INVALID_ARG: return "invalid argument";
        case TBE_ERR_UNSUPPORTED: return "unsupported configuration";
        case TBE_ERR_NOT_BOUND: return "device buffers not bound";
        case TBE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case TBE_ERR_INDEX_OUT_OF_RANGE: return "index out of range";
        case TBE_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* tbe_last_hip_error(tbe_handle_t h) { return h ? h->last_hip_error.c_str() : ""; }

tbe_status_t tbe_create(const tbe_config_t* cfg, tbe_handle_t* out_handle)
{
    if (!cfg || !out_handle || !cfg->rows || !cfg->dims || cfg->num_tables < 1 || cfg->max_batch < 0 ||
        cfg->max_indices < 0)
        return TBE_ERR_INVALID_ARG;
    for (int t = 0; t < cfg->num_tables; ++t)
        if (cfg->rows[t] <= 0 || cfg->dims[t] <= 0)
            return TBE_ERR_INVALID_ARG;
    for (int t = 0; t < cfg->num_tables; ++t)
        if (cfg->rows[t] >= ((int64_t)1 << 31))   // indices are int32: such a table could not be addressed
            return TBE_ERR_UNSUPPORTED;
    if ((cfg->weight_dtype != TBE_DTYPE_FP32 && cfg->weight_dtype != TBE_DTYPE_FP16) ||
        cfg->pooling != TBE_POOLING_SUM || (cfg->layout != TBE_LAYOUT_BATCH_MAJOR && cfg->layout != TBE_LAYOUT_TABLE_MAJOR) ||
        (cfg->optimizer != TBE_OPT_ROWWISE_ADAGRAD && cfg->optimizer != TBE_OPT_ADAGRAD &&
         cfg->optimizer != TBE_OPT_ADAM) ||
        (cfg->output_dtype != TBE_DTYPE_FP32 && cfg->output_dtype != TBE_DTYPE_FP16) ||
        (cfg->grad_dtype != TBE_DTYPE_FP32 && cfg->grad_dtype != TBE_DTYPE_FP16 &&
         cfg->grad_dtype != TBE_DTYPE_BF16))
        return TBE_ERR_UNSUPPORTED;
    if (cfg->max_indices >= ((int64_t)1 << 31) - ((int64_t)1 << 24) ||
        (int64_t)cfg->num_tables * cfg->max_batch >= ((int64_t)1 << 31) - 1024)
        return TBE_ERR_UNSUPPORTED;
    int64_t total_rows = 0, sumD = 0;
    bool all8 = true;
    int dmax = 0;
    for (int t = 0; t < cfg->num_tables; ++t) {
        if (cfg->dims[t] % 4 != 0 || cfg->dims[t] > kMaxDim)
            return TBE_ERR_UNSUPPORTED;
        total_rows += cfg->rows[t];
        if (total_rows >= ((int64_t)1 << 32) - 1)
            return TBE_ERR_UNSUPPORTED;
        sumD += cfg->dims[t];
        all8 = all8 && cfg->dims[t] % 8 == 0;
        dmax = std::max(dmax, cfg->dims[t]);
    }
    if (sumD >= ((int64_t)1 << 31))
        return TBE_ERR_UNSUPPORTED;

    tbe_s* h = new (std::nothrow) tbe_s();
    if (!h)
        return TBE_ERR_INVALID_ARG;
    h->T = cfg->num_tables;
    h->rows.assign(cfg->rows, cfg->rows + h->T);
    h->dims.assign(cfg->dims, cfg->dims + h->T);
    h->dtype = cfg->weight_dtype;
    h->optimizer = cfg->optimizer;
    h->out_dtype = cfg->output_dtype;
    h->grad_dtype = cfg->grad_dtype;
    h->layout = cfg->layout;
    h->max_batch = cfg->max_batch;
    h->max_indices = cfg->max_indices;
    h->sumD = sumD;
    h->dmax = dmax;
    h->fwd_epl = (h->dtype == TBE_DTYPE_FP16 && all8) ? 8 : 4;
    h->fwd_kmax = (int)ceil_div(dmax, h->fwd_epl * kWave);
    // the sort is segmented by table, so only the bits of the tallest table's row index are sorted
    int64_t max_rows = 1;
    for (int t = 0; t < cfg->num_tables; ++t)
        max_rows = std::max(max_rows, cfg->rows[t]);
    h->key_bits = 1;
    while (h->key_bits < 32 && ((int64_t)1 << h->key_bits) < max_rows)
        ++h->key_bits;
    // per-table sort geometry: table t orders ceil(log2 H_t) bits in P_t = ceil(bits / 8) passes during the
    // last P_t of the P launches, bits split as evenly as possible (wider digits first)
    const int P = (int)ceil_div(h->key_bits, 8);
    h->pass_digit_bits.assign(P, 1);
    std::vector<int> table_bits(cfg->num_tables, 1);
    for (int t = 0; t < cfg->num_tables; ++t) {
        int b = 1;
        while (b < 32 && ((int64_t)1 << b) < cfg->rows[t])
            ++b;
        table_bits[t] = b;
        const int pt = (b + 7) / 8, q = b / pt, rem = b - q * pt;
        for (int lp = 0; lp < pt; ++lp) {
            int& w = h->pass_digit_bits[P - pt + lp];
            w = std::max(w, q + (lp < rem ? 1 : 0));
        }
    }

    h->woff.resize(h->T + 1);
    h->soff.resize(h->T + 1);
    h->coloff.resize(h->T + 1);
    h->meta.resize(h->T);
    int64_t w = 0, s = 0;
    int32_t c = 0;
    for (int t = 0; t < h->T; ++t) {
        h->woff[t] = w;
        h->soff[t] = s;
        h->coloff[t] = c;
        TableMeta& m = h->meta[t];
        m.woff = w;
        m.rbase = (uint32_t)s;
        m.dim = h->dims[t];
        m.col = c;
        m.lpr_fwd = std::min(6, pow2ceil_log2((int)ceil_div(h->dims[t], h->fwd_epl)));
        m.lpr_bwd = std::min(6, pow2ceil_log2((int)ceil_div(h->dims[t], 8)));
        m.key_bits = table_bits[t];
        w += h->rows[t] * (int64_t)h->dims[t];
        s += h->rows[t];
        c += h->dims[t];
    }
    h->woff[h->T] = w;
    h->soff[h->T] = s;
    h->coloff[h->T] = c;
    h->weight_elems = w;
    h->weight_bytes = (size_t)w * (h->dtype == TBE_DTYPE_FP32 ? 4 : 2);
    h->state_bytes = h->optimizer == TBE_OPT_ROWWISE_ADAGRAD ? (size_t)s * 4
                     : h->optimizer == TBE_OPT_ADAGRAD       ? (size_t)w * 4
                                                             : (size_t)w * 8;
    plan_workspace(h);
    *out_handle = h;
    return TBE_OK;
}

tbe_status_t tbe_destroy(tbe_handle_t h)
{
    if (!h)
        return TBE_OK;
    for (hipEvent_t e : h->ev_pool)
        (void)hipEventDestroy(e);
    delete h;
    return TBE_OK;
}

tbe_status_t tbe_query_sizes(tbe_handle_t h, size_t* weight_bytes, size_t* state_bytes,
                             size_t* workspace_bytes, int64_t* weight_offsets, int64_t* state_offsets,
                             int32_t* out_col_offsets)
{
    if (!h)
        return TBE_ERR_INVALID_ARG;
    if (weight_bytes)
        *weight_bytes = h->weight_bytes;
    if (state_bytes)
        *state_bytes = h->state_bytes;
    if (workspace_bytes)
        *workspace_bytes = h->workspace_bytes;
    if (weight_offsets)
        std::memcpy(weight_offsets, h->woff.data(), sizeof(int64_t) * (h->T + 1));
    if (state_offsets)
        std::memcpy(state_offsets, h->soff.data(), sizeof(int64_t) * (h->T + 1));
    if (out_col_offsets)
        std::memcpy(out_col_offsets, h->coloff.data(), sizeof(int32_t) * (h->T + 1));
    return TBE_OK;
}

tbe_status_t tbe_bind(tbe_handle_t h, void* d_weights, float* d_state, void* d_workspace,
                      size_t workspace_bytes)
{
    if (!h || !d_weights || !d_state || !d_workspace)
        return TBE_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(d_workspace) & 255) || (reinterpret_cast<uintptr_t>(d_weights) & 15) ||
        (reinterpret_cast<uintptr_t>(d_state) & (h->optimizer == TBE_OPT_ROWWISE_ADAGRAD ? 3 : 15)))
        return TBE_ERR_INVALID_ARG;
    if (workspace_bytes < h->workspace_bytes)
        return TBE_ERR_WORKSPACE_TOO_SMALL;
    h->bound = false;
    h->d_weights = d_weights;
    h->d_state = d_state;
    h->d_ws = static_cast<char*>(d_workspace);
    std::vector<uint32_t> rb(h->T + 1);
    for (int t = 0; t <= h->T; ++t)
        rb[t] = (uint32_t)h->soff[t];
    Counters zero;
    std::memset(&zero, 0, sizeof(zero));
    TBE_HIP_CHECK(h, hipMemcpy(h->d_ws + h->off_meta, h->meta.data(), sizeof(TableMeta) * h->T,
                               hipMemcpyHostToDevice));
    TBE_HIP_CHECK(h, hipMemcpy(h->d_ws + h->off_rowbase, rb.data(), sizeof(uint32_t) * (h->T + 1),
                               hipMemcpyHostToDevice));
    TBE_HIP_CHECK(h, hipMemcpy(h->d_ws + h->off_counters, &zero, sizeof(zero), hipMemcpyHostToDevice));
    TBE_HIP_CHECK(h, hipMemset(h->d_ws + h->off_zero, 0, kZeroRowBytes));
    TBE_HIP_CHECK(h, hipMemset(h->d_ws + h->off_dense_cnt, 0, 4 * (size_t)h->T));
    TBE_HIP_CHECK(h, hipMemset(h->d_ws + h->off_dense_dirty, 0, 4 * (size_t)h->T));
    TBE_HIP_CHECK(h, hipMemset(h->d_ws + h->off_win_cnt, 0, 4 * (size_t)h->T));
    TBE_HIP_CHECK(h, hipDeviceSynchronize());
    h->bound = true;
    h->final_buf = -1;
    h->sorted_n = -1;
    return TBE_OK;
}

tbe_status_t tbe_forward(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                         int64_t num_indices, int32_t batch, void* d_out, void* stream)
{
    tbe_status_t rc = check_call(h, d_indices, d_offsets, num_indices, batch);
    if (rc != TBE_OK)
        return rc;
    if (batch == 0)
        return TBE_OK;
    if (!d_out)
        return TBE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ScopedTimer tm(h, SLOT_FORWARD, st);
    const int32_t n = (int32_t)num_indices;
    if (h->out_dtype == TBE_DTYPE_FP32) {
        float* out = static_cast<float*>(d_out);
        if (h->dtype == TBE_DTYPE_FP32)
            return launch_forward<float, float>(h, d_indices, d_offsets, n, batch, out, st);
        return launch_forward<__half, float>(h, d_indices, d_offsets, n, batch, out, st);
    }
    __half* out = static_cast<__half*>(d_out);
    if (h->dtype == TBE_DTYPE_FP32)
        return launch_forward<float, __half>(h, d_indices, d_offsets, n, batch, out, st);
    return launch_forward<__half, __half>(h, d_indices, d_offsets, n, batch, out, st);
}

// a2..a4: needs only the batch's (indices, offsets)
static tbe_status_t enqueue_sort(tbe_s* h, const int32_t* d_indices, const int64_t* d_offsets, int32_t n,
                                 int32_t batch, hipStream_t st)
{
    tbe_status_t rc = TBE_OK;
    Counters* counters = h->ws<Counters>(h->off_counters);
    h->sorted_n = n;
    h->sorted_batch = batch;
    if (batch == 0 || n == 0) {
        hipLaunchKernelGGL(clear_num_unique_kernel, dim3(1), dim3(1), 0, st, counters);
        TBE_LAUNCH_CHECK(h, "clear_num_unique_kernel");
        h->final_buf = 0;
        return TBE_OK;
    }
    const uint32_t* row_base = h->ws<uint32_t>(h->off_rowbase);
    uint32_t* keys[2] = {h->ws<uint32_t>(h->off_keys[0]), h->ws<uint32_t>(h->off_keys[1])};
    int32_t* vals[2] = {h->ws<int32_t>(h->off_vals[0]), h->ws<int32_t>(h->off_vals[1])};

    SortPlan pl;
    pl.tile_base = h->ws<int32_t>(h->off_tile_base);
    pl.tstart = h->ws<int32_t>(h->off_tstart);
    pl.tiles = h->ws<TileDesc>(h->off_tile_table);
    // upper bound of the number of tiles for THIS call (the exact number is only known on the device)
    const int max_tiles = (int)std::min<int64_t>(h->max_tiles, ceil_div(n, kSortTile) + h->T);
    {   // a2: table borders -> tile plan (keys are the caller's indices; payloads are made in the first pass)
        ScopedTimer tm(h, SLOT_SORT_PLAN, st);
        hipLaunchKernelGGL(sort_plan_tables_kernel, dim3(1), dim3(256), 0, st, d_offsets, batch, h->T,
                           h->ws<int32_t>(h->off_tile_base), h->ws<int32_t>(h->off_tstart), counters);
        hipLaunchKernelGGL(sort_plan_tiles_kernel, dim3((unsigned)ceil_div(max_tiles, 256)), dim3(256), 0, st,
                           pl.tile_base, pl.tstart, d_offsets, batch, h->T, h->ws<TileDesc>(h->off_tile_table),
                           max_tiles);
        TBE_LAUNCH_CHECK(h, "sort_plan kernels");
    }

    // a3: stable LSD radix sort, segmented by table; every table over the bits of its own row index, in its own
    // number of passes, all tables finishing in the last launch (tables with fewer passes sit out the first ones)
    const int passes = (int)ceil_div(h->key_bits, 8);
    uint32_t* hist = h->ws<uint32_t>(h->off_hist);
    const TableMeta* meta = h->ws<TableMeta>(h->off_meta);
    const uint32_t* indices = reinterpret_cast<const uint32_t*>(d_indices);
    int cur = -1;  // pair that holds the current order (-1 = nothing sorted yet)
    for (int p = 0; p < passes; ++p) {
        const int nd_bits = h->pass_digit_bits[p];   // widest digit any table sorts in this launch
        const int out = cur < 0 ? 0 : cur ^ 1;
        const uint32_t* keys_cur = cur < 0 ? indices : keys[cur];
        const int32_t* vals_cur = cur < 0 ? nullptr : vals[cur];
        {
            ScopedTimer tm(h, SLOT_RADIX_HIST, st);
            hipLaunchKernelGGL(radix_hist_kernel, dim3(max_tiles), dim3(kSortThreads), 0, st, pl, meta, keys_cur,
                               indices, hist, p, passes, nd_bits);
            TBE_LAUNCH_CHECK(h, "radix_hist_kernel");
        }
        {
            ScopedTimer tm(h, SLOT_RADIX_SCAN, st);
            rc = device_scan(h, hist, (int64_t)max_tiles << nd_bits, nullptr, st);
            if (rc != TBE_OK)
                return rc;
        }
        {
            ScopedTimer tm(h, SLOT_RADIX_SCATTER, st);
            // a bag number below 2^16 travels as 16 bits between the passes
            auto launch = [&](auto kernel) {
                hipLaunchKernelGGL(kernel, dim3(max_tiles), dim3(kSortThreads), 0, st, pl, meta, keys_cur, vals_cur,
                                   indices, keys[out], vals[out], hist, d_offsets, row_base, batch, p, passes, nd_bits);
            };
            const bool last = p == passes - 1, v16 = batch <= 65536;
            if (last && v16)
                launch(radix_scatter_kernel<true, true>);
            else if (last)
                launch(radix_scatter_kernel<true, false>);
            else if (v16)
                launch(radix_scatter_kernel<false, true>);
            else
                launch(radix_scatter_kernel<false, false>);
            TBE_LAUNCH_CHECK(h, "radix_scatter_kernel");
        }
        cur = out;
    }
    h->final_buf = cur;

    // a4: run heads -> unique keys, segment offsets, per-chunk first run (the free ping-pong pair
    // of the sort holds unique_keys / seg_offsets)
    uint32_t* unique_keys = keys[cur ^ 1];
    int32_t* seg_offsets = vals[cur ^ 1];
    int32_t* chunk_first = h->ws<int32_t>(h->off_chunk_first);
    const int num_chunks = (int)ceil_div(n, kChunk);
    {
        ScopedTimer tm(h, SLOT_RUNLENGTH, st);
        const int rl_tiles = (int)ceil_div(n, kRlTile);
        uint32_t* rl_counts = h->ws<uint32_t>(h->off_rl_counts);
        hipLaunchKernelGGL(runlength_count_kernel, dim3(rl_tiles), dim3(kRlThreads), 0, st, keys[cur],
                           rl_counts, n);
        rc = device_scan(h, rl_counts, rl_tiles, nullptr, st);
        if (rc != TBE_OK)
            return rc;
        hipLaunchKernelGGL(runlength_write_kernel, dim3(rl_tiles), dim3(kRlThreads), 0, st, keys[cur],
                           rl_counts, unique_keys, seg_offsets, chunk_first, counters, n, num_chunks);
        TBE_LAUNCH_CHECK(h, "runlength kernels");
    }

    return TBE_OK;
}

// a5 + a6 on the artefacts left by enqueue_sort
extern "C++" {
template <typename WT, typename GT, int OPT>
static void launch_update(const BwdArgs& a, dim3 grid, dim3 grid_fix, hipStream_t st, tbe_s* h)
{
    {
        ScopedTimer tm(h, SLOT_REDUCE_UPDATE, st);
        hipLaunchKernelGGL((reduce_update_kernel<WT, GT, OPT>), grid, dim3(kBwdThreads), 0, st, a);
    }
    Counters* counters = h->ws<Counters>(h->off_counters);
    if (a.n > kLongRun) {
        // the long runs below the dense threshold: plan -> window-border positions -> pieces, window by window
        ScopedTimer tm(h, SLOT_WINDOW_RUNS, st);
        uint32_t* wpre = h->ws<uint32_t>(h->off_wrun);
        uint32_t* ppre = wpre + (h->T + 1);
        WinPiece* pieces = h->ws<WinPiece>(h->off_wbounds);
        hipLaunchKernelGGL(window_plan_kernel, dim3(1), dim3(256), 0, st, a, wpre, ppre);
        hipLaunchKernelGGL(window_pieces_kernel, dim3(1024), dim3(256), 0, st, a, wpre, ppre, pieces);
        hipLaunchKernelGGL((window_runs_kernel<GT>), dim3(kWindowGrid), dim3(kBwdThreads), 0, st, a, pieces);
    }
    if (a.dense_thr != INT32_MAX) {
        // the runs the update kernel queued as dense: plan -> bag-slice positions -> counts x gradient block
        ScopedTimer tm(h, SLOT_DENSE_ROWS, st);
        DenseArgs d;
        d.b = a;
        d.drun = h->ws<uint32_t>(h->off_drun);
        d.dgroup = h->ws<DenseGroup>(h->off_dgroup);
        d.dbounds = h->ws<int32_t>(h->off_dbounds);
        d.nruns = &counters->dense_runs;
        d.nsub = a.dense_slices;
        d.slice_bags = kDenseSlice;
        hipLaunchKernelGGL(run_plan_kernel, dim3(1), dim3(256), 0, st, a, a.dense_cnt, a.dense_list, a.dense_thr,
                           (int)kDenseRows, h->ws<uint32_t>(h->off_drun), h->ws<DenseGroup>(h->off_dgroup),
                           &counters->dense_runs, &counters->dense_groups, a.dense_dirty);
        hipLaunchKernelGGL(run_bounds_kernel, dim3(512), dim3(256), 0, st, d);
        hipLaunchKernelGGL((dense_rows_kernel<GT>), dim3(kDenseGrid), dim3(kDenseThreads), 0, st, d);
    }
    {
        ScopedTimer tm(h, SLOT_LONG_FIXUP, st);
        hipLaunchKernelGGL((long_run_fixup_kernel<WT, GT, OPT>), grid_fix, dim3(kBwdThreads), 0, st, a);
    }
}

template <typename WT, typename GT>
static void launch_update_opt(const BwdArgs& a, dim3 grid, dim3 grid_fix, hipStream_t st, tbe_s* h)
{
    if (h->optimizer == TBE_OPT_ROWWISE_ADAGRAD)
        launch_update<WT, GT, kOptRowwiseAdagrad>(a, grid, grid_fix, st, h);
    else if (h->optimizer == TBE_OPT_ADAGRAD)
        launch_update<WT, GT, kOptAdagrad>(a, grid, grid_fix, st, h);
    else
        launch_update<WT, GT, kOptAdam>(a, grid, grid_fix, st, h);
}

template <typename WT>
static void launch_update_grad(const BwdArgs& a, dim3 grid, dim3 grid_fix, hipStream_t st, tbe_s* h)
{
    if (h->grad_dtype == TBE_DTYPE_FP32)
        launch_update_opt<WT, float>(a, grid, grid_fix, st, h);
    else if (h->grad_dtype == TBE_DTYPE_FP16)
        launch_update_opt<WT, __half>(a, grid, grid_fix, st, h);
    else
        launch_update_opt<WT, __hip_bfloat16>(a, grid, grid_fix, st, h);
}
}  // extern "C++"

struct OptCall {   // what the caller passed for this step
    int optimizer;
    float lr, eps, beta1, beta2;
    int64_t step;
};

static tbe_status_t enqueue_update(tbe_s* h, const void* d_grad_out, const OptCall& oc, hipStream_t st)
{
    const int32_t n = h->sorted_n;
    if (h->sorted_batch == 0 || n == 0)
        return TBE_OK;
    if (!d_grad_out)
        return TBE_ERR_INVALID_ARG;
    const int cur = h->final_buf;
    Counters* counters = h->ws<Counters>(h->off_counters);
    const uint32_t* row_base = h->ws<uint32_t>(h->off_rowbase);
    uint32_t* keys[2] = {h->ws<uint32_t>(h->off_keys[0]), h->ws<uint32_t>(h->off_keys[1])};
    int32_t* vals[2] = {h->ws<int32_t>(h->off_vals[0]), h->ws<int32_t>(h->off_vals[1])};
    uint32_t* unique_keys = keys[cur ^ 1];
    int32_t* seg_offsets = vals[cur ^ 1];
    int32_t* chunk_first = h->ws<int32_t>(h->off_chunk_first);
    const int num_chunks = (int)ceil_div(n, kChunk);
    // a5 + a6: on-chip aggregation per run, one AdaGrad step per touched row
    BwdArgs a;
    a.meta = h->ws<TableMeta>(h->off_meta);
    a.row_base = row_base;
    a.sorted_keys = keys[cur];
    a.sorted_vals = vals[cur];
    a.unique_keys = unique_keys;
    a.seg_offsets = seg_offsets;
    a.chunk_first_run = chunk_first;
    a.counters = counters;
    a.grad_out = d_grad_out;
    a.weights = h->d_weights;
    a.partials = h->ws<float>(h->off_partials);
    a.long_list = h->ws<uint32_t>(h->off_long_list);
    a.zero_row = h->ws<float>(h->off_zero);
    a.n = n;
    a.num_chunks = num_chunks;
    a.T = h->T;
    a.sumD = (int32_t)h->sumD;
    a.dpad = (int32_t)align_up((size_t)h->dmax, 4);
    a.batch = h->sorted_batch;
    a.table_major = h->layout;
    // dense hot rows: only when a run can exceed the threshold and the bounds table of this call fits
    const int thr = dense_threshold(h->sorted_batch);
    const bool dense_on = n > thr && dense_bounds_entries(n, h->sorted_batch, h->T) <= h->dbounds_cap &&
                          n / thr + h->T + 2 <= h->max_indices / kDenseMinRun + h->T + 2;
    a.dense_thr = dense_on ? thr : INT32_MAX;
    a.dense_slices = (int32_t)ceil_div(std::max(h->sorted_batch, 1), kDenseSlice);
    a.tstart = h->ws<int32_t>(h->off_tstart);
    a.dense_cnt = h->ws<uint32_t>(h->off_dense_cnt);
    a.dense_list = h->ws<uint32_t>(h->off_dense_list);
    a.dense_dirty = h->ws<uint32_t>(h->off_dense_dirty);
    a.win_cnt = h->ws<uint32_t>(h->off_win_cnt);
    a.win_list = h->ws<uint32_t>(h->off_win_list);
    a.grad_bytes = h->grad_dtype == TBE_DTYPE_FP32 ? 4 : 2;
    a.opt.state0 = h->d_state;
    a.opt.state1 = h->optimizer == TBE_OPT_ADAM ? h->d_state + h->weight_elems : h->d_state;
    a.opt.lr = oc.lr;
    a.opt.eps = oc.eps;
    a.opt.beta1 = oc.beta1;
    a.opt.beta2 = oc.beta2;
    a.opt.inv_bc1 = 1.0f;
    a.opt.inv_bc2 = 1.0f;
    if (h->optimizer == TBE_OPT_ADAM) {
        // bias corrections in double from the float32 betas the kernel uses
        a.opt.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)oc.beta1, (double)oc.step)));
        a.opt.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)oc.beta2, (double)oc.step)));
    }
    const int per_block = kBwdThreads / kWave;
    const dim3 grid((unsigned)ceil_div(ceil_div(num_chunks, kSpanChunks), per_block));   // a wavefront per span of chunks
    const int64_t max_long = n / kLongRun + 1;
    const dim3 grid_fix((unsigned)std::min<int64_t>(2048, ceil_div(max_long, per_block)));
    if (h->dtype == TBE_DTYPE_FP32)
        launch_update_grad<float>(a, grid, grid_fix, st, h);
    else
        launch_update_grad<__half>(a, grid, grid_fix, st, h);
    TBE_LAUNCH_CHECK(h, "reduce_update / long_run_fixup kernels");
    return TBE_OK;
}

tbe_status_t tbe_backward_sort(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                               int64_t num_indices, int32_t batch, void* stream)
{
    tbe_status_t rc = check_call(h, d_indices, d_offsets, num_indices, batch);
    if (rc != TBE_OK)
        return rc;
    return enqueue_sort(h, d_indices, d_offsets, (int32_t)num_indices, batch, static_cast<hipStream_t>(stream));
}

static tbe_status_t check_opt(tbe_s* h, const OptCall& oc)
{
    if (!h)
        return TBE_ERR_INVALID_ARG;
    if (!h->bound)
        return TBE_ERR_NOT_BOUND;
    if (h->optimizer != oc.optimizer)
        return TBE_ERR_INVALID_ARG;
    if (oc.optimizer == TBE_OPT_ADAM &&
        (oc.step < 1 || !(oc.beta1 >= 0.f && oc.beta1 < 1.f) || !(oc.beta2 >= 0.f && oc.beta2 < 1.f)))
        return TBE_ERR_INVALID_ARG;
    return TBE_OK;
}

static tbe_status_t backward_update(tbe_handle_t h, const void* d_grad_out, const OptCall& oc, void* stream)
{
    tbe_status_t rc = check_opt(h, oc);
    if (rc != TBE_OK)
        return rc;
    if (h->final_buf < 0 || h->sorted_n < 0)
        return TBE_ERR_INVALID_ARG;
    return enqueue_update(h, d_grad_out, oc, static_cast<hipStream_t>(stream));
}

static tbe_status_t backward_full(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                  int64_t num_indices, int32_t batch, const void* d_grad_out, const OptCall& oc,
                                  void* stream)
{
    tbe_status_t rc = check_call(h, d_indices, d_offsets, num_indices, batch);
    if (rc != TBE_OK)
        return rc;
    rc = check_opt(h, oc);
    if (rc != TBE_OK)
        return rc;
    if (batch > 0 && num_indices > 0 && !d_grad_out)
        return TBE_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_sort(h, d_indices, d_offsets, (int32_t)num_indices, batch, st);
    if (rc != TBE_OK)
        return rc;
    return enqueue_update(h, d_grad_out, oc, st);
}

tbe_status_t tbe_backward_update_rowwise_adagrad(tbe_handle_t h, const void* d_grad_out, float lr, float eps,
                                                 void* stream)
{
    return backward_update(h, d_grad_out, OptCall{TBE_OPT_ROWWISE_ADAGRAD, lr, eps, 0.f, 0.f, 1}, stream);
}

tbe_status_t tbe_backward_update_adagrad(tbe_handle_t h, const void* d_grad_out, float lr, float eps, void* stream)
{
    return backward_update(h, d_grad_out, OptCall{TBE_OPT_ADAGRAD, lr, eps, 0.f, 0.f, 1}, stream);
}

tbe_status_t tbe_backward_update_adam(tbe_handle_t h, const void* d_grad_out, float lr, float beta1, float beta2,
                                      float eps, int64_t step, void* stream)
{
    return backward_update(h, d_grad_out, OptCall{TBE_OPT_ADAM, lr, eps, beta1, beta2, step}, stream);
}

tbe_status_t tbe_backward_rowwise_adagrad(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                          int64_t num_indices, int32_t batch, const void* d_grad_out, float lr,
                                          float eps, void* stream)
{
    return backward_full(h, d_indices, d_offsets, num_indices, batch, d_grad_out,
                         OptCall{TBE_OPT_ROWWISE_ADAGRAD, lr, eps, 0.f, 0.f, 1}, stream);
}

tbe_status_t tbe_backward_adagrad(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                                  int64_t num_indices, int32_t batch, const void* d_grad_out, float lr, float eps,
                                  void* stream)
{
    return backward_full(h, d_indices, d_offsets, num_indices, batch, d_grad_out,
                         OptCall{TBE_OPT_ADAGRAD, lr, eps, 0.f, 0.f, 1}, stream);
}

tbe_status_t tbe_backward_adam(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                               int64_t num_indices, int32_t batch, const void* d_grad_out, float lr, float beta1,
                               float beta2, float eps, int64_t step, void* stream)
{
    return backward_full(h, d_indices, d_offsets, num_indices, batch, d_grad_out,
                         OptCall{TBE_OPT_ADAM, lr, eps, beta1, beta2, step}, stream);
}

tbe_status_t tbe_backward_artifacts(tbe_handle_t h, const uint32_t** d_sorted_keys,
                                    const int32_t** d_sorted_vals, const uint32_t** d_unique_keys,
                                    const int32_t** d_seg_offsets, const int64_t** d_num_unique)
{
    if (!h)
        return TBE_ERR_INVALID_ARG;
    if (!h->bound)
        return TBE_ERR_NOT_BOUND;
    if (h->final_buf < 0)
        return TBE_ERR_INVALID_ARG;
    const int cur = h->final_buf;
    if (d_sorted_keys)
        *d_sorted_keys = h->ws<uint32_t>(h->off_keys[cur]);
    if (d_sorted_vals)
        *d_sorted_vals = h->ws<int32_t>(h->off_vals[cur]);
    if (d_unique_keys)
        *d_unique_keys = h->ws<uint32_t>(h->off_keys[cur ^ 1]);
    if (d_seg_offsets)
        *d_seg_offsets = h->ws<int32_t>(h->off_vals[cur ^ 1]);
    if (d_num_unique)
        *d_num_unique = &h->ws<Counters>(h->off_counters)->num_unique;
    return TBE_OK;
}

tbe_status_t tbe_check_inputs(tbe_handle_t h, const int32_t* d_indices, const int64_t* d_offsets,
                              int64_t num_indices, int32_t batch, void* stream)
{
    tbe_status_t rc = check_call(h, d_indices, d_offsets, num_indices, batch);
    if (rc != TBE_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Counters* counters = h->ws<Counters>(h->off_counters);
    const int num_bags = h->T * batch;
    Counters host;
    std::memset(&host, 0, sizeof(host));
    if (num_bags == 0)
        return num_indices == 0 ? TBE_OK : TBE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(clear_check_flags_kernel, dim3(1), dim3(1), 0, st, counters);
    hipLaunchKernelGGL(check_inputs_kernel, dim3((unsigned)ceil_div(num_bags, 256)), dim3(256), 0, st,
                       h->ws<TableMeta>(h->off_meta), h->ws<uint32_t>(h->off_rowbase), d_indices, d_offsets,
                       num_indices, batch, num_bags, counters);
    TBE_LAUNCH_CHECK(h, "check_inputs_kernel");
    TBE_HIP_CHECK(h, hipMemcpyAsync(&host, counters, sizeof(host), hipMemcpyDeviceToHost, st));
    TBE_HIP_CHECK(h, hipStreamSynchronize(st));
    if (host.check_flags & 1u)
        return TBE_ERR_INVALID_ARG;
    if (host.check_flags & 2u)
        return TBE_ERR_INDEX_OUT_OF_RANGE;
    return TBE_OK;
}

tbe_status_t tbe_profile_enable(tbe_handle_t h, int32_t max_calls)
{
    if (!h || max_calls < 0)
        return TBE_ERR_INVALID_ARG;
    for (hipEvent_t e : h->ev_pool)
        (void)hipEventDestroy(e);
    h->ev_pool.clear();
    h->recs.clear();
    h->ev_used = 0;
    h->profiling = false;
    if (max_calls == 0)
        return TBE_OK;
    const size_t want = (size_t)max_calls * 2 * 24;  // <= 24 timed kernel groups per call
    h->ev_pool.reserve(want);
    for (size_t i = 0; i < want; ++i) {
        hipEvent_t e;
        TBE_HIP_CHECK(h, hipEventCreate(&e));
        h->ev_pool.push_back(e);
    }
    h->recs.reserve(want / 2);
    h->profiling = true;
    return TBE_OK;
}

tbe_status_t tbe_profile_read(tbe_handle_t h, int32_t capacity, const char** names, int64_t* launches,
                              double* total_ms, int32_t* num_slots)
{
    if (!h || capacity < SLOT_COUNT || !names || !launches || !total_ms || !num_slots)
        return TBE_ERR_INVALID_ARG;
    for (int s = 0; s < SLOT_COUNT; ++s) {
        names[s] = kSlotNames[s];
        launches[s] = 0;
        total_ms[s] = 0.0;
    }
    *num_slots = SLOT_COUNT;
    for (const ProfRec& r : h->recs) {
        TBE_HIP_CHECK(h, hipEventSynchronize(r.stop));
        float ms = 0.f;
        TBE_HIP_CHECK(h, hipEventElapsedTime(&ms, r.start, r.stop));
        launches[r.slot] += 1;
        total_ms[r.slot] += ms;
    }
    h->recs.clear();
    h->ev_used = 0;
    return TBE_OK;
}

tbe_status_t tbe_probe_read(const void* d_src, size_t bytes, int32_t passes, void* d_sink, void* stream)
{
    if (!d_src || !d_sink || bytes < 16 || passes < 1 || (reinterpret_cast<uintptr_t>(d_src) & 15u) != 0 ||
        (reinterpret_cast<uintptr_t>(d_sink) & 3u) != 0)
        return TBE_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>(8192, (n16 + 255) / 256);
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(d_src), n16, (int)passes, static_cast<uint32_t*>(d_sink));
    return hipGetLastError() == hipSuccess ? TBE_OK : TBE_ERR_HIP;
}

}  // extern "C"
