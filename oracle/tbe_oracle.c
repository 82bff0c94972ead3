/*
 * CPU oracle for the table-batched embedding path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded statement of what the path computes, in fp64, written from the
 * paper's definitions.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product path never does.  It shares no code with the HIP library.
 *
 * What each function follows:
 *   - lookup: an embedding table has one row per categorical id and one column per embedding
 *     dimension; the forward maps ids to rows (Section 2.1).  Pooling a bag of ids into one vector
 *     (sum or mean) is the problem statement's reading; the paper itself is silent on pooling.
 *   - only rows whose ids appear in the batch receive a gradient (Section 2.1); the row gradient is
 *     the sum over the samples that hit the row (group-gradient formula, Section 3.2); the 1/|batch|
 *     factor of that formula belongs to the loss, so grad_out arrives already scaled.
 *   - moment-scaled row-wise AdaGrad, Algorithm 1 steps 5-6:  v <- v + ||g||_2^2, then
 *     w <- w - eta / (sqrt(v / c) + eps) * g with the *updated* v.  c = 1 is the ordinary row-wise
 *     AdaGrad of Section 3.2 (eta_k = eta / (sqrt(v_k) + eps), v_k = sum_s ||g_s||^2).
 *     eps sits outside the square root (algorithm box and base definition agree; one prose sentence
 *     typesets it inside - not followed).  v is stored unscaled; c enters only the step size.
 *
 * Layout seen by this oracle: one separate array per table (row-major R_t x D_t), ids table-local,
 * table-major CSR: bag (t, b) owns positions offsets[t*B+b] .. offsets[t*B+b+1]-1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1 };
enum { ORACLE_SUM = 0, ORACLE_MEAN = 1 };

/* ---- IEEE binary16 <-> double, round-to-nearest-even, written out by hand ------------------ */
double oracle_half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double x;
    if (e == 0) {
        x = ldexp((double)m, -24);                      /* subnormal: m * 2^-24 */
    } else if (e == 31) {
        x = m ? NAN : INFINITY;
    } else {
        x = ldexp((double)(1024 + m), e - 25);          /* (1 + m/1024) * 2^(e-15) */
    }
    return sign ? -x : x;
}

uint16_t oracle_double_to_half(double x) {
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs(x);
    if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);   /* at or above the halfway point to 2^16: inf */
    if (a < ldexp(1.0, -25)) return sign;                   /* below half of the smallest subnormal -> 0 (ties to even = 0) */
    int ex;
    (void)frexp(a, &ex);                                    /* a = f * 2^ex, f in [0.5, 1)  =>  a in [2^(ex-1), 2^ex) */
    int e = ex - 1;                                         /* unbiased exponent */
    if (e < -14) e = -14;                                   /* subnormal range shares the spacing 2^-24 */
    double ulp = ldexp(1.0, e - 10);
    double q = a / ulp;                                     /* exact: power-of-two scaling */
    double r = nearbyint(q);                                /* default rounding mode = nearest even */
    double v = r * ulp;                                     /* may carry into the next binade; still representable */
    if (v >= 65536.0) return (uint16_t)(sign | 0x7C00u);
    int ex2;
    uint16_t bits;
    if (v < ldexp(1.0, -14)) {
        bits = (uint16_t)(v / ldexp(1.0, -24));             /* subnormal mantissa */
    } else {
        (void)frexp(v, &ex2);
        int e2 = ex2 - 1;
        double mant = v / ldexp(1.0, e2) - 1.0;             /* in [0,1) */
        bits = (uint16_t)(((e2 + 15) << 10) | (int)(mant * 1024.0));
    }
    return (uint16_t)(sign | bits);
}

/* ---- bfloat16 (the upper 16 bits of a binary32) <-> double, round-to-nearest-even, by hand ------------ */
double oracle_bf16_to_double(uint16_t b) {
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xFF;
    int m = b & 0x7F;
    double x;
    if (e == 0) x = ldexp((double)m, -133);                 /* subnormal: m * 2^-7 * 2^-126 */
    else if (e == 255) x = m ? NAN : INFINITY;
    else x = ldexp((double)(128 + m), e - 134);             /* (1 + m/128) * 2^(e-127) */
    return sign ? -x : x;
}

uint16_t oracle_double_to_bf16(double x) {
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs(x);
    if (isnan(x)) return (uint16_t)(sign | 0x7FC0u);
    if (isinf(x)) return (uint16_t)(sign | 0x7F80u);
    if (a < ldexp(1.0, -134)) return sign;                  /* below half of the smallest subnormal (2^-133) */
    int ex;
    (void)frexp(a, &ex);
    int e = ex - 1;
    if (e < -126) e = -126;                                 /* subnormals share the spacing 2^-133 */
    double ulp = ldexp(1.0, e - 7);
    double v = nearbyint(a / ulp) * ulp;                    /* nearest even in the default rounding mode */
    if (v >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80u);
    uint16_t bits;
    if (v < ldexp(1.0, -126)) {
        bits = (uint16_t)(v / ldexp(1.0, -133));
    } else {
        int ex2;
        (void)frexp(v, &ex2);
        int e2 = ex2 - 1;
        double mant = v / ldexp(1.0, e2) - 1.0;
        bits = (uint16_t)(((e2 + 127) << 7) | (int)(mant * 128.0));
    }
    return (uint16_t)(sign | bits);
}

/* element types of the pooled output / upstream gradient matrix */
enum { ORACLE_IO_F32 = 0, ORACLE_IO_F16 = 1, ORACLE_IO_BF16 = 2 };

static double load_io(const void* m, int io, int64_t e) {
    if (io == ORACLE_IO_F32) return (double)((const float*)m)[e];
    if (io == ORACLE_IO_F16) return oracle_half_to_double(((const uint16_t*)m)[e]);
    return oracle_bf16_to_double(((const uint16_t*)m)[e]);
}

static void store_io(void* m, int io, int64_t e, double x) {   /* one rounding, from the fp64 value */
    if (io == ORACLE_IO_F32) ((float*)m)[e] = (float)x;
    else if (io == ORACLE_IO_F16) ((uint16_t*)m)[e] = oracle_double_to_half(x);
    else ((uint16_t*)m)[e] = oracle_double_to_bf16(x);
}

static double load_w(const void* tab, int dtype, int64_t e) {
    if (dtype == ORACLE_F32) return (double)((const float*)tab)[e];
    return oracle_half_to_double(((const uint16_t*)tab)[e]);
}

static void store_w(void* tab, int dtype, int64_t e, double x) {
    if (dtype == ORACLE_F32) ((float*)tab)[e] = (float)x;
    else ((uint16_t*)tab)[e] = oracle_double_to_half(x);
}

/* pooling factor of one bag: 1 for sum; 1/L for mean (an empty bag contributes nothing) */
static double bag_scale(const int64_t* offsets, int64_t bag, int pooling) {
    int64_t L = offsets[bag + 1] - offsets[bag];
    if (pooling == ORACLE_SUM) return 1.0;
    return L > 0 ? 1.0 / (double)L : 0.0;
}

/* ---- forward -------------------------------------------------------------------------------- */
/* One bag:  out_row[j] = sum_{p in bag} W_t[indices[p], j], for mean pooling divided by the number of ids L
 * (a division, as the mean is defined: a product with the rounded reciprocal 1/L would be one more rounding, and
 * would break the tie of a 16-bit output whose exact mean lies half-way between two values by its own error).
 * Returns -1 on an id outside [0, R_t). */
int oracle_forward_bag_io(const void* table, int dtype, int64_t R, int32_t D, const int64_t* indices,
                          int64_t start, int64_t end, int pooling, void* out, int out_io, int64_t out_elem) {
    double* acc = (double*)calloc((size_t)D, sizeof(double));
    for (int64_t p = start; p < end; ++p) {
        int64_t r = indices[p];
        if (r < 0 || r >= R) { free(acc); return -1; }
        for (int32_t j = 0; j < D; ++j) acc[j] += load_w(table, dtype, r * D + j);
    }
    int64_t L = end - start;
    for (int32_t j = 0; j < D; ++j) {
        double x = acc[j];
        if (pooling != ORACLE_SUM) x = L > 0 ? x / (double)L : 0.0;
        store_io(out, out_io, out_elem + j, x);
    }
    free(acc);
    return 0;
}

int oracle_forward_bag(const void* table, int dtype, int64_t R, int32_t D, const int64_t* indices,
                       int64_t start, int64_t end, int pooling, float* out_row) {
    return oracle_forward_bag_io(table, dtype, R, D, indices, start, end, pooling, out_row, ORACLE_IO_F32, 0);
}

/* All bags: out is [B, sum(D)] row-major; bag (t,b) fills out[b, D_off[t] : D_off[t]+D_t]. */
int oracle_forward_io(int32_t T, const int64_t* rows, const int32_t* D, int dtype, const void* const* tables,
                      const int64_t* indices, const int64_t* offsets, int32_t B, int pooling, void* out, int out_io) {
    int64_t sumD = 0;
    for (int32_t t = 0; t < T; ++t) sumD += D[t];
    int64_t doff = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t b = 0; b < B; ++b) {
            int64_t bag = (int64_t)t * B + b;
            int rc = oracle_forward_bag_io(tables[t], dtype, rows[t], D[t], indices, offsets[bag], offsets[bag + 1],
                                           pooling, out, out_io, (int64_t)b * sumD + doff);
            if (rc) return rc;
        }
        doff += D[t];
    }
    return 0;
}

int oracle_forward(int32_t T, const int64_t* rows, const int32_t* D, int dtype, const void* const* tables,
                   const int64_t* indices, const int64_t* offsets, int32_t B, int pooling, float* out) {
    return oracle_forward_io(T, rows, D, dtype, tables, indices, offsets, B, pooling, out, ORACLE_IO_F32);
}

/* ---- which rows appear: linearise, stable sort, run lengths ---------------------------------- */
typedef struct { int64_t key; int64_t pos; } keypos;

/* A stable sort by key is, by definition, the sort by (key, original position). */
static int cmp_keypos(const void* a, const void* b) {
    const keypos* x = (const keypos*)a;
    const keypos* y = (const keypos*)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/* key[p] = row_base[t(p)] + indices[p] where t(p) is the table of the bag that owns position p. */
int oracle_linearize(int32_t T, const int64_t* rows, const int64_t* indices, const int64_t* offsets, int32_t B,
                     int64_t* keys /*[N]*/, int64_t* bag_of /*[N], may be NULL*/) {
    int64_t base = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t b = 0; b < B; ++b) {
            int64_t bag = (int64_t)t * B + b;
            for (int64_t p = offsets[bag]; p < offsets[bag + 1]; ++p) {
                if (indices[p] < 0 || indices[p] >= rows[t]) return -1;
                keys[p] = base + indices[p];
                if (bag_of) bag_of[p] = bag;
            }
        }
        base += rows[t];
    }
    return 0;
}

/* order = the stable ascending permutation of keys; keys_sorted[i] = keys[order[i]]. */
void oracle_stable_sort(const int64_t* keys, int64_t N, int64_t* keys_sorted, int64_t* order) {
    keypos* kp = (keypos*)malloc((size_t)(N > 0 ? N : 1) * sizeof(keypos));
    for (int64_t p = 0; p < N; ++p) { kp[p].key = keys[p]; kp[p].pos = p; }
    qsort(kp, (size_t)N, sizeof(keypos), cmp_keypos);
    for (int64_t i = 0; i < N; ++i) { keys_sorted[i] = kp[i].key; order[i] = kp[i].pos; }
    free(kp);
}

/* Run-length segmentation of a sorted key list: unique_rows[u], seg_start[u] (seg_start[U] = N). Returns U. */
int64_t oracle_run_lengths(const int64_t* keys_sorted, int64_t N, int64_t* unique_rows, int64_t* seg_start) {
    int64_t U = 0;
    for (int64_t i = 0; i < N; ++i) {
        if (i == 0 || keys_sorted[i] != keys_sorted[i - 1]) {
            unique_rows[U] = keys_sorted[i];
            seg_start[U] = i;
            ++U;
        }
    }
    seg_start[U] = N;
    return U;
}

/* ---- the optimizer step of one row (Algorithm 1, steps 5 and 6) ------------------------------ */
void oracle_adagrad_row(void* table, int dtype, int64_t r, int32_t D, float* v /* this row's moment */,
                        const double* g, double lr, double eps, double c) {
    double sq = 0.0;
    for (int32_t j = 0; j < D; ++j) sq += g[j] * g[j];
    double v_new = (double)(*v) + sq;                       /* step 5: unscaled squared L2 norm accumulates */
    /* step 6 with v_new == 0 (moments are sums of squares, so this means v == 0 and g == 0): the update term is
     * eta * 0 / (0 + eps), which is 0 for every eps > 0; its value at eps == 0 is taken to be that limit, so a row
     * whose gradient is zero keeps its bits for every eps >= 0 and no 0/0 arises */
    if (v_new == 0.0) return;
    double step = lr / (sqrt(v_new / c) + eps);             /* step 6: c divides the moment inside the root */
    for (int32_t j = 0; j < D; ++j) {
        double w = load_w(table, dtype, r * D + j);
        store_w(table, dtype, r * D + j, w - step * g[j]);
    }
    *v = (float)v_new;
}

/* Plain SGD step of one row, the conventional optimizer the paper contrasts row-wise AdaGrad with
 * (Section 3.2):  w <- w - eta * g.  No state. */
void oracle_sgd_row(void* table, int dtype, int64_t r, int32_t D, const double* g, double lr) {
    for (int32_t j = 0; j < D; ++j) {
        double w = load_w(table, dtype, r * D + j);
        store_w(table, dtype, r * D + j, w - lr * g[j]);
    }
}

/* Row gradient straight from the definition, no sorting: scan every position of table t and add the
 * bag's upstream gradient slice (times the bag's pooling factor) whenever the id equals r.
 * grad_out is [B, sumD] row-major, doff = D_off[t].  Returns the number of hits. */
int64_t oracle_row_gradient_by_scan(int32_t t, int64_t r, int32_t D, int64_t doff, int64_t sumD,
                                    const float* grad_out, const int64_t* indices, const int64_t* offsets,
                                    int32_t B, int pooling, double* g /*[D] out*/) {
    int64_t hits = 0;
    for (int32_t j = 0; j < D; ++j) g[j] = 0.0;
    for (int32_t b = 0; b < B; ++b) {
        int64_t bag = (int64_t)t * B + b;
        double s = bag_scale(offsets, bag, pooling);
        for (int64_t p = offsets[bag]; p < offsets[bag + 1]; ++p) {
            if (indices[p] != r) continue;
            ++hits;
            for (int32_t j = 0; j < D; ++j) g[j] += s * (double)grad_out[(int64_t)b * sumD + doff + j];
        }
    }
    return hits;
}

/* ---- backward + optimizer, the sorted way ----------------------------------------------------
 * linearise -> stable sort -> run lengths -> for every unique row: sum the gradient slices of its
 * segment in ascending position order (fp64), then one optimizer step.  Rows outside unique_rows are
 * never written.  Optional outputs (may be NULL): keys_sorted[N], order[N], unique_rows[N], seg_start[N+1].
 * Returns U (>= 0), or -1 on an invalid id. */
int64_t oracle_backward_rowwise_adagrad_io(int32_t T, const int64_t* rows, const int32_t* D, int dtype,
                                           void* const* tables /*in/out*/, float* state /*[sum rows] in/out*/,
                                           const void* grad_out, int grad_io, const int64_t* indices,
                                           const int64_t* offsets, int32_t B, int pooling, double lr, double eps,
                                           double c, int64_t* keys_sorted_out, int64_t* order_out,
                                           int64_t* unique_rows_out, int64_t* seg_start_out) {
    int64_t N = offsets[(int64_t)T * B];
    int64_t sumD = 0;
    int32_t maxD = 0;
    for (int32_t t = 0; t < T; ++t) { sumD += D[t]; if (D[t] > maxD) maxD = D[t]; }
    size_t n1 = (size_t)(N > 0 ? N : 1);
    int64_t* keys = (int64_t*)malloc(n1 * sizeof(int64_t));
    int64_t* bag_of = (int64_t*)malloc(n1 * sizeof(int64_t));
    int64_t* ks = (int64_t*)malloc(n1 * sizeof(int64_t));
    int64_t* order = (int64_t*)malloc(n1 * sizeof(int64_t));
    int64_t* uniq = (int64_t*)malloc(n1 * sizeof(int64_t));
    int64_t* seg = (int64_t*)malloc((n1 + 1) * sizeof(int64_t));
    double* g = (double*)malloc((size_t)(maxD > 0 ? maxD : 1) * sizeof(double));
    int64_t U = -1;
    if (oracle_linearize(T, rows, indices, offsets, B, keys, bag_of) == 0) {
        oracle_stable_sort(keys, N, ks, order);
        U = oracle_run_lengths(ks, N, uniq, seg);
        int32_t t = 0;
        int64_t base = 0, doff = 0;
        for (int64_t u = 0; u < U; ++u) {
            while (uniq[u] >= base + rows[t]) { base += rows[t]; doff += D[t]; ++t; }   /* table of this key */
            int64_t r = uniq[u] - base;
            int32_t Dt = D[t];
            for (int32_t j = 0; j < Dt; ++j) g[j] = 0.0;
            for (int64_t i = seg[u]; i < seg[u + 1]; ++i) {
                int64_t bag = bag_of[order[i]];
                int64_t b = bag - (int64_t)t * B;
                double s = bag_scale(offsets, bag, pooling);
                for (int32_t j = 0; j < Dt; ++j) g[j] += s * load_io(grad_out, grad_io, b * sumD + doff + j);
            }
            if (state) oracle_adagrad_row(tables[t], dtype, r, Dt, &state[uniq[u]], g, lr, eps, c);
            else oracle_sgd_row(tables[t], dtype, r, Dt, g, lr);      /* state == NULL: plain SGD */
        }
        if (keys_sorted_out) memcpy(keys_sorted_out, ks, (size_t)N * sizeof(int64_t));
        if (order_out) memcpy(order_out, order, (size_t)N * sizeof(int64_t));
        if (unique_rows_out) memcpy(unique_rows_out, uniq, (size_t)U * sizeof(int64_t));
        if (seg_start_out) memcpy(seg_start_out, seg, (size_t)(U + 1) * sizeof(int64_t));
    }
    free(keys); free(bag_of); free(ks); free(order); free(uniq); free(seg); free(g);
    return U;
}

int64_t oracle_backward_rowwise_adagrad(int32_t T, const int64_t* rows, const int32_t* D, int dtype,
                                        void* const* tables, float* state, const float* grad_out,
                                        const int64_t* indices, const int64_t* offsets, int32_t B, int pooling, double lr,
                                        double eps, double c, int64_t* keys_sorted_out, int64_t* order_out,
                                        int64_t* unique_rows_out, int64_t* seg_start_out) {
    return oracle_backward_rowwise_adagrad_io(T, rows, D, dtype, tables, state, grad_out, ORACLE_IO_F32, indices, offsets,
                                              B, pooling, lr, eps, c, keys_sorted_out, order_out, unique_rows_out,
                                              seg_start_out);
}

/* ---- cross-replica synchronisation (Algorithm 1, the weight-sync and moment-sync steps) -----------------
 * Every replica m = 0..M-1 holds its own copy of a buffer (weights of one table set, or the moments); after the
 * step each copy is replaced by the element-wise mean over the replicas,  x^(j) <- (1/M) sum_m x^(m)  for all j.
 * dtype: ORACLE_F32 or ORACLE_F16 (the mean is formed in fp64 and rounded once to the storage type). */
void oracle_replica_mean(void* const* replicas, int32_t M, int64_t count, int dtype) {
    for (int64_t e = 0; e < count; ++e) {
        double sum = 0.0;
        for (int32_t m = 0; m < M; ++m) sum += load_w(replicas[m], dtype, e);
        double mean = sum / (double)M;
        for (int32_t m = 0; m < M; ++m) store_w(replicas[m], dtype, e, mean);
    }
}

/* ---- non-pooled lookup (Section 2.1: the forward maps ids to embedding rows; no pooling) ------------------
 * table_offsets[T+1] ascending from 0 to nnz: table t owns positions table_offsets[t] .. table_offsets[t+1]-1.
 * out / grad_seq: one row-major [n_t, D_t] block per table, the blocks one after the other. */
int oracle_lookup_seq_io(int32_t T, const int64_t* rows, const int32_t* D, int dtype, const void* const* tables,
                         const int64_t* indices, const int64_t* table_offsets, void* out, int out_io) {
    int64_t base = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int64_t p = table_offsets[t]; p < table_offsets[t + 1]; ++p) {
            int64_t r = indices[p];
            if (r < 0 || r >= rows[t]) return -1;
            for (int32_t j = 0; j < D[t]; ++j)
                store_io(out, out_io, base + (p - table_offsets[t]) * D[t] + j, load_w(tables[t], dtype, r * D[t] + j));
        }
        base += (table_offsets[t + 1] - table_offsets[t]) * D[t];
    }
    return 0;
}

/* Backward of the non-pooled lookup with the same optimizer step: the gradient of row r of table t is the sum of
 * grad_seq rows over the positions that hold r (Section 3.2's sum over the samples that hit the row), then
 * Algorithm 1 steps 5-6 (or the SGD step when state is NULL).  Straight from the definition: the positions of each row are
 * collected by a bucket pass and their gradient rows added in ascending position order.  Returns the number of rows updated, -1 on a bad id. */
int64_t oracle_backward_seq_io(int32_t T, const int64_t* rows, const int32_t* D, int dtype, void* const* tables,
                               float* state, const void* grad_seq, int grad_io, const int64_t* indices,
                               const int64_t* table_offsets, double lr, double eps, double c) {
    int64_t updated = 0, base = 0, row_base = 0;
    for (int32_t t = 0; t < T; ++t) {
        int64_t s0 = table_offsets[t], s1 = table_offsets[t + 1];
        for (int64_t p = s0; p < s1; ++p)
            if (indices[p] < 0 || indices[p] >= rows[t]) return -1;
        /* the positions of every row, in ascending order: count, prefix sum, fill (a bucket pass, no comparison sort) */
        int64_t R = rows[t];
        int64_t* start = (int64_t*)calloc((size_t)R + 1, sizeof(int64_t));
        int64_t* fill = (int64_t*)calloc((size_t)R, sizeof(int64_t));
        int64_t* where = (int64_t*)malloc((size_t)(s1 > s0 ? s1 - s0 : 1) * sizeof(int64_t));
        double* g = (double*)malloc((size_t)D[t] * sizeof(double));
        for (int64_t p = s0; p < s1; ++p) start[indices[p] + 1] += 1;
        for (int64_t r = 0; r < R; ++r) start[r + 1] += start[r];
        for (int64_t p = s0; p < s1; ++p) { int64_t r = indices[p]; where[start[r] + fill[r]++] = p; }
        for (int64_t r = 0; r < R; ++r) {
            if (start[r + 1] == start[r]) continue;             /* the id does not appear: no gradient, no update */
            for (int32_t j = 0; j < D[t]; ++j) g[j] = 0.0;
            for (int64_t i = start[r]; i < start[r + 1]; ++i) {
                int64_t q = where[i];
                for (int32_t j = 0; j < D[t]; ++j) g[j] += load_io(grad_seq, grad_io, base + (q - s0) * D[t] + j);
            }
            if (state) oracle_adagrad_row(tables[t], dtype, r, D[t], &state[row_base + r], g, lr, eps, c);
            else oracle_sgd_row(tables[t], dtype, r, D[t], g, lr);
            ++updated;
        }
        free(start); free(fill); free(where); free(g);
        base += (s1 - s0) * D[t];
        row_base += rows[t];
    }
    return updated;
}
