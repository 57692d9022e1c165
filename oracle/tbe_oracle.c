/*
 * CPU oracle for the table-batched embedding-bag (TBE) operator of DLRM training.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded
 * implementation of the definitions the paper gives; only tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.  It shares no code with the HIP
 * library and must never be imported by it.
 *
 * What it follows (arxiv 2104.05158):
 *   - Section 2, "Embedding operators" (Fig. 2): every index of a bag fetches a full
 *     table row and the rows of a bag are combined element-wise (sum pooling here).
 *   - Section 5.1 (Fig. 6b): all gradients that reach one embedding row, from every
 *     sample of the batch, are aggregated BEFORE the non-linear optimizer sees them;
 *     one optimizer step per touched row per call.
 *   - Section 5.2, row-wise sparse AdaGrad: one moment scalar per row (a 1-D tensor of
 *     H elements), increased by the mean over the row of the squared aggregated
 *     gradient, and used to scale the whole row's step.
 *   - Section 7.1: jagged (indices, offsets) input in the nn.EmbeddingBag sense, all
 *     tables concatenated table-major: bag id j = t*B + b.
 *
 * Readings where the paper is silent (the same list is kept in the design notes):
 *   sum pooling; a row repeated inside one bag counts once per occurrence; moments
 *   start at 0 (caller's job); the step uses the UPDATED moment; epsilon sits outside
 *   the square root: w -= lr * G / (sqrt(m_new) + eps); "average squared sum" is read
 *   as the mean of squares (1/D) * sum_d G_d^2; fp16 write-back rounds to nearest even;
 *   empty bags pool to 0; the sort of (table,row) keys is stable.
 *
 * Arithmetic: every sum is carried in double from the exactly converted stored values
 * (fp16/fp32 -> double is exact); results are rounded once to the storage type.
 *
 * Pins: all functions below are pinned by tests/test_oracle_pins.py (dense count-matrix
 * brute force, torch CPU embedding_bag + autograd, pure-gather special case, AdaGrad
 * closed forms incl. a small-gradient case that separates the epsilon placements,
 * duplicate-aggregation vs sequential steps, invariants).  Nothing here is unpinned.
 *
 * Data layout (the interface both this file and the HIP library are tested through):
 *   weights : flat array; table t occupies elements [woff_t, woff_t + H_t*D_t), row-major,
 *             woff_t = sum_{s<t} H_s*D_s.   dtype 0 = float32, 1 = IEEE binary16.
 *   moments : flat float32; table t's rows at [R_t, R_t + H_t), R_t = sum_{s<t} H_s.
 *   indices : int32[N]; offsets : int64[T*B+1], offsets[0]=0, offsets[T*B]=N.
 *   out / grad_out : float32 [B, sumD] row-major; table t owns columns [c_t, c_t + D_t).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- IEEE binary16 <-> double, written out by hand (no compiler half type) ---- */

static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24); /* subnormal or zero */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);
    return sign ? -v : v;
}

/* round-to-nearest-even, overflow to infinity */
static uint16_t double_to_half(double x)
{
    uint16_t sign = 0;
    if (isnan(x))
        return 0x7e00;
    if (signbit(x)) {
        sign = 0x8000;
        x = -x;
    }
    if (isinf(x))
        return sign | 0x7c00;
    if (x == 0.0)
        return sign;
    int ex;
    (void)frexp(x, &ex); /* x = m * 2^ex, m in [0.5,1) */
    int e = ex - 1;      /* x = (2m) * 2^e, 2m in [1,2) */
    if (e < -14)
        e = -14; /* subnormal range: fixed quantum 2^-24 */
    /* quantum of the target format at this exponent is 2^(e-10) */
    double scaled = ldexp(x, 10 - e); /* in [1024, 2048) for normals, [0,1024) for subnormals */
    double r = nearbyint(scaled);     /* default rounding mode: nearest even */
    if (r >= 2048.0) {
        r = 1024.0;
        e += 1;
    }
    if (e > 15)
        return sign | 0x7c00;
    uint32_t q = (uint32_t)r;
    if (q < 1024)
        return sign | (uint16_t)q; /* subnormal (e == -14, hidden bit absent) */
    return sign | (uint16_t)(((e + 15) << 10) | (q - 1024));
}

/* exported so that the conversion itself can be pinned against numpy's float16 */
double oracle_half_to_double(uint16_t h) { return half_to_double(h); }
uint16_t oracle_double_to_half(double x) { return double_to_half(x); }

static double load_w(const void* w, int dtype, int64_t i)
{
    if (dtype == 0)
        return (double)((const float*)w)[i];
    return half_to_double(((const uint16_t*)w)[i]);
}

static void store_w(void* w, int dtype, int64_t i, double v)
{
    if (dtype == 0)
        ((float*)w)[i] = (float)v;
    else
        ((uint16_t*)w)[i] = double_to_half(v);
}

static int check_cfg(int T, const int64_t* rows, const int32_t* dims, int dtype, int B)
{
    if (T < 1 || !rows || !dims || B < 0 || (dtype != 0 && dtype != 1))
        return -1;
    for (int t = 0; t < T; ++t)
        if (rows[t] <= 0 || dims[t] <= 0)
            return -1;
    return 0;
}

/*
 * Forward, Section 2 "Embedding operators":
 *   out[b, c_t + d] = sum_{p in bag (t,b)} W_t[indices[p], d]
 * absref (nullable, same shape as out, double) receives sum |terms|, the scale a
 * tolerance for a reordered fp32 sum must be measured against.
 * Returns 0, -1 on bad arguments, -2 on an index outside its table or bad offsets.
 */
int oracle_tbe_forward(int T, const int64_t* rows, const int32_t* dims, int dtype,
                       const void* weights, const int32_t* indices, const int64_t* offsets,
                       int B, float* out, double* absref)
{
    if (check_cfg(T, rows, dims, dtype, B) || !weights || !offsets || !out)
        return -1;
    int64_t sumD = 0;
    for (int t = 0; t < T; ++t)
        sumD += dims[t];
    int64_t woff = 0, col = 0;
    for (int t = 0; t < T; ++t) {
        int D = dims[t];
        double* acc = (double*)malloc(sizeof(double) * 2 * (size_t)D);
        double* aabs = acc + D;
        for (int b = 0; b < B; ++b) {
            int64_t j = (int64_t)t * B + b;
            int64_t lo = offsets[j], hi = offsets[j + 1];
            if (lo > hi || lo < 0) {
                free(acc);
                return -2;
            }
            for (int d = 0; d < 2 * D; ++d)
                acc[d] = 0.0;
            for (int64_t p = lo; p < hi; ++p) {
                int64_t r = indices[p];
                if (r < 0 || r >= rows[t]) {
                    free(acc);
                    return -2;
                }
                for (int d = 0; d < D; ++d) {
                    double v = load_w(weights, dtype, woff + r * D + d);
                    acc[d] += v;
                    aabs[d] += fabs(v);
                }
            }
            for (int d = 0; d < D; ++d) {
                out[(int64_t)b * sumD + col + d] = (float)acc[d];
                if (absref)
                    absref[(int64_t)b * sumD + col + d] = aabs[d];
            }
        }
        free(acc);
        woff += rows[t] * (int64_t)D;
        col += D;
    }
    return 0;
}

/* ---- (table,row) keys, their stable sort and the run-length artefacts ---- */

typedef struct {
    uint32_t key; /* R_t + row */
    int32_t val;  /* b, the bag's position inside its table's batch */
    int64_t pos;  /* original lookup position p, the stable tie-break */
} lookup_t;

static int cmp_lookup(const void* a, const void* b)
{
    const lookup_t* x = (const lookup_t*)a;
    const lookup_t* y = (const lookup_t*)b;
    if (x->key != y->key)
        return x->key < y->key ? -1 : 1;
    if (x->pos != y->pos)
        return x->pos < y->pos ? -1 : 1;
    return 0;
}

/* builds and sorts the lookup list; caller frees. NULL on error (err set). */
static lookup_t* sorted_lookups(int T, const int64_t* rows, int B, const int32_t* indices,
                                const int64_t* offsets, int64_t* n_out, int* err)
{
    int64_t total_rows = 0;
    for (int t = 0; t < T; ++t)
        total_rows += rows[t];
    *err = 0;
    if (total_rows >= ((int64_t)1 << 32)) {
        *err = -1;
        return NULL;
    }
    int64_t N = offsets[(int64_t)T * B];
    *n_out = N;
    lookup_t* v = (lookup_t*)malloc(sizeof(lookup_t) * (size_t)(N > 0 ? N : 1));
    int64_t R = 0;
    for (int t = 0; t < T; ++t) {
        for (int b = 0; b < B; ++b) {
            int64_t j = (int64_t)t * B + b;
            if (offsets[j] > offsets[j + 1] || offsets[j] < 0) {
                *err = -2;
                free(v);
                return NULL;
            }
            for (int64_t p = offsets[j]; p < offsets[j + 1]; ++p) {
                int64_t r = indices[p];
                if (r < 0 || r >= rows[t]) {
                    *err = -2;
                    free(v);
                    return NULL;
                }
                v[p].key = (uint32_t)(R + r);
                v[p].val = b;
                v[p].pos = p;
            }
        }
        R += rows[t];
    }
    qsort(v, (size_t)N, sizeof(lookup_t), cmp_lookup);
    return v;
}

/*
 * Integer artefacts of the backward pass, Section 5.1 "gradient sorting by rows":
 *   sorted_keys[N]  ascending linear row ids R_t + row
 *   sorted_vals[N]  bag position b of each sorted lookup; equal keys keep input order
 *   unique_keys[U], seg_offsets[U+1] (run u = sorted positions [seg_offsets[u], seg_offsets[u+1]))
 * Output arrays must have room for N (N+1 for seg_offsets) entries; any may be NULL.
 */
int oracle_tbe_sort_artifacts(int T, const int64_t* rows, int B, const int32_t* indices,
                              const int64_t* offsets, uint32_t* sorted_keys, int32_t* sorted_vals,
                              uint32_t* unique_keys, int64_t* seg_offsets, int64_t* num_unique)
{
    if (T < 1 || !rows || B < 0 || !offsets)
        return -1;
    int64_t N;
    int err;
    lookup_t* v = sorted_lookups(T, rows, B, indices, offsets, &N, &err);
    if (!v)
        return err;
    int64_t U = 0;
    for (int64_t q = 0; q < N; ++q) {
        if (sorted_keys)
            sorted_keys[q] = v[q].key;
        if (sorted_vals)
            sorted_vals[q] = v[q].val;
        if (q == 0 || v[q].key != v[q - 1].key) {
            if (unique_keys)
                unique_keys[U] = v[q].key;
            if (seg_offsets)
                seg_offsets[U] = q;
            ++U;
        }
    }
    if (seg_offsets)
        seg_offsets[U] = N;
    if (num_unique)
        *num_unique = U;
    free(v);
    return 0;
}

/*
 * Backward fused with row-wise AdaGrad, Sections 5.1 and 5.2.  For every touched row
 * (t,r), in ascending key order:
 *   G_d    = sum over ALL lookups p of the batch with indices[p]==r in table t of
 *            grad_out[b(p), c_t + d]                                  (aggregate first)
 *   m_new  = m_old + (1/D_t) * sum_d G_d^2                            (mean of squares)
 *   w_new  = w_old - lr * G_d / (sqrt(m_new) + eps)                   (one step per row)
 * weights and moments are updated in place; rows never looked up are not written.
 *
 * Optional outputs (NULL to skip), one block of D_t doubles per touched row, blocks in
 * ascending key order, block u starting at g_offsets[u]:
 *   G_out     aggregated gradient;  Gabs_out  sum of |terms| (tolerance scale)
 *   g_offsets int64[U+1];  m_new_out double[U] the unrounded updated moment.
 */
int oracle_tbe_backward_rowwise_adagrad(int T, const int64_t* rows, const int32_t* dims, int dtype,
                                        void* weights, float* moments, const int32_t* indices,
                                        const int64_t* offsets, int B, const float* grad_out,
                                        double lr, double eps, double* G_out, double* Gabs_out,
                                        int64_t* g_offsets, double* m_new_out)
{
    if (check_cfg(T, rows, dims, dtype, B) || !weights || !moments || !offsets || !grad_out)
        return -1;
    int64_t N;
    int err;
    lookup_t* v = sorted_lookups(T, rows, B, indices, offsets, &N, &err);
    if (!v)
        return err;

    int64_t sumD = 0;
    int maxD = 0;
    for (int t = 0; t < T; ++t) {
        sumD += dims[t];
        if (dims[t] > maxD)
            maxD = dims[t];
    }
    double* G = (double*)malloc(sizeof(double) * 2 * (size_t)maxD);
    double* Gabs = G + maxD;

    int t = 0;
    int64_t R = 0, woff = 0, col = 0; /* first row id, weight offset, output column of table t */
    int64_t U = 0, gpos = 0;
    int64_t q = 0;
    while (q < N) {
        uint32_t key = v[q].key;
        while ((int64_t)key >= R + rows[t]) { /* advance to the table that owns this key */
            R += rows[t];
            woff += rows[t] * (int64_t)dims[t];
            col += dims[t];
            ++t;
        }
        int D = dims[t];
        int64_t r = (int64_t)key - R;
        for (int d = 0; d < D; ++d)
            G[d] = Gabs[d] = 0.0;
        int64_t e = q;
        while (e < N && v[e].key == key) {
            const float* g = grad_out + (int64_t)v[e].val * sumD + col;
            for (int d = 0; d < D; ++d) {
                G[d] += (double)g[d];
                Gabs[d] += fabs((double)g[d]);
            }
            ++e;
        }
        double ss = 0.0;
        for (int d = 0; d < D; ++d)
            ss += G[d] * G[d];
        double m_new = (double)moments[key] + ss / (double)D;
        double denom = sqrt(m_new) + eps;
        for (int d = 0; d < D; ++d) {
            int64_t i = woff + r * D + d;
            double w = load_w(weights, dtype, i);
            store_w(weights, dtype, i, w - lr * G[d] / denom);
        }
        moments[key] = (float)m_new;
        if (g_offsets)
            g_offsets[U] = gpos;
        if (m_new_out)
            m_new_out[U] = m_new;
        for (int d = 0; d < D; ++d) {
            if (G_out)
                G_out[gpos + d] = G[d];
            if (Gabs_out)
                Gabs_out[gpos + d] = Gabs[d];
        }
        gpos += D;
        ++U;
        q = e;
    }
    if (g_offsets)
        g_offsets[U] = gpos;
    free(G);
    free(v);
    return 0;
}
