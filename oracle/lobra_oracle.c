/*
 * fp64 CPU oracle for the shared-base multi-adapter LoRA linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is
 * compared against; it is never part of the product path and shares no code,
 * header, table or helper with the HIP sources.
 *
 * What it computes (paper section 2.1, "Fine-tuning based on LoRA": a frozen
 * weight W of shape in x out plus two trained low-rank factors, output
 * X W + X (down) (up); section 1 and Figure 1: tokens of several tasks are fused
 * into one batch, the base product is shared, each task applies its own
 * adapter).  The paper's letters for the two factors are the reverse of the
 * usual ones; here, as in the common convention,
 *     A_t  is the down projection, stored as r_t rows of length d_in,
 *     B_t  is the up projection,   stored as r_t rows of length d_out,
 * and a per-task scalar s_t multiplies the adapter term (the paper has s_t = 1).
 * All tasks' rows are stacked: task t owns rows rank_off[t] .. rank_off[t+1]-1
 * of A [R_tot, d_in] and B [R_tot, d_out].
 *
 * For a token i whose task is t = task_of[i] (t = -1: no adapter):
 *     h_i  = A_t x_i                       (r_t)
 *     y_i  = x_i W + s_t * (h_i B_t)       (d_out)
 *     g_i  = B_t dy_i                      (r_t)
 *     dx_i = dy_i W^T + s_t * (g_i A_t)    (d_in)
 *     dB_t = s_t * sum_{i in t} h_i^T dy_i (r_t x d_out)
 *     dA_t = s_t * sum_{i in t} g_i^T x_i  (r_t x d_in)
 * W is frozen (section 1: the base model is unaltered), so no dW exists.
 *
 * The method is exact, so the oracle is this definition written as loops:
 * every stored input value (fp32, or bf16 given as its 16 bit pattern) is
 * widened exactly to double, every sum is a plain double accumulation in index
 * order, nothing is blocked, fused or rounded in between.  OpenMP only splits
 * independent output rows across threads; it never splits a sum.
 *
 * Pins (tests/test_oracle_pins.py): base-only reduction when B = 0, merged
 * weight W + s A^T B against a library matmul, fused batch equals per-task
 * runs, adjoint identities, central finite differences, autograd of the
 * per-task formulation, structural invariances, hand-computed integer cases.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { LOBRA_ORACLE_F32 = 0, LOBRA_ORACLE_BF16 = 1 };

/* Exact widening of one stored element to double. */
static inline double load_elem(const void *p, int dtype, size_t i)
{
    if (dtype == LOBRA_ORACLE_F32)
        return (double)((const float *)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Token -> task map of a packed batch (section 1: a fused batch holds sequences
 * of several tasks, each tagged with its task).  Segment k covers tokens
 * seg_off[k] .. seg_off[k+1]-1 and carries task seg_task[k] (-1 = no adapter).
 * Returns 0, or -1 when the table is malformed.
 */
int lobra_oracle_token_task(int64_t T, int32_t S, const int32_t *seg_off,
                            const int32_t *seg_task, int32_t n_tasks,
                            int32_t *task_of)
{
    for (int64_t i = 0; i < T; ++i)
        task_of[i] = -1;
    if (S == 0)
        return T == 0 ? 0 : -1;
    if (seg_off[0] != 0 || seg_off[S] != T)
        return -1;
    for (int32_t k = 0; k < S; ++k) {
        if (seg_off[k + 1] < seg_off[k])
            return -1;
        if (seg_task[k] < -1 || seg_task[k] >= n_tasks)
            return -1;
        for (int64_t i = seg_off[k]; i < seg_off[k + 1]; ++i)
            task_of[i] = seg_task[k];
    }
    return 0;
}

/*
 * Forward rows.  rows == NULL: all T rows (nrows must equal T), else the listed
 * token indices.  y_out is [nrows, d_out]; h_out (may be NULL) is
 * [nrows, r_max] with r_max = max_t r_t and holds the unscaled h_i, zero beyond
 * r_t.
 */
int lobra_oracle_fwd(int dtype, int64_t T, int32_t d_in, int32_t d_out,
                     int32_t n_tasks, const int32_t *rank_off,
                     const int32_t *task_of, const void *x, const void *W,
                     const void *A, const void *B, const float *s,
                     int64_t nrows, const int64_t *rows, double *y_out,
                     double *h_out)
{
    int32_t r_max = 0;
    for (int32_t t = 0; t < n_tasks; ++t)
        if (rank_off[t + 1] - rank_off[t] > r_max)
            r_max = rank_off[t + 1] - rank_off[t];
    if (!rows && nrows != T)
        return -1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nrows; ++q) {
        const int64_t i = rows ? rows[q] : q;
        double *y = y_out + (size_t)q * d_out;
        for (int32_t j = 0; j < d_out; ++j)
            y[j] = 0.0;
        /* base: y = x_i W */
        for (int32_t k = 0; k < d_in; ++k) {
            const double xk = load_elem(x, dtype, (size_t)i * d_in + k);
            for (int32_t j = 0; j < d_out; ++j)
                y[j] += xk * load_elem(W, dtype, (size_t)k * d_out + j);
        }
        if (h_out)
            for (int32_t p = 0; p < r_max; ++p)
                h_out[(size_t)q * r_max + p] = 0.0;
        const int32_t t = task_of[i];
        if (t < 0)
            continue;
        const int32_t r0 = rank_off[t], r = rank_off[t + 1] - rank_off[t];
        double *h = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        /* down projection: h = A_t x_i */
        for (int32_t p = 0; p < r; ++p) {
            double acc = 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                acc += load_elem(x, dtype, (size_t)i * d_in + k) *
                       load_elem(A, dtype, (size_t)(r0 + p) * d_in + k);
            h[p] = acc;
            if (h_out)
                h_out[(size_t)q * r_max + p] = acc;
        }
        /* up projection and scale: y += s_t * (h B_t) */
        const double st = (double)s[t];
        for (int32_t j = 0; j < d_out; ++j) {
            double lo = 0.0;
            for (int32_t p = 0; p < r; ++p)
                lo += h[p] * load_elem(B, dtype, (size_t)(r0 + p) * d_out + j);
            y[j] += st * lo;
        }
        free(h);
    }
    return 0;
}

/*
 * Backward rows: dx_out is [nrows, d_in]; g_out (may be NULL) is [nrows, r_max]
 * with the unscaled g_i.
 */
int lobra_oracle_bwd_dx(int dtype, int64_t T, int32_t d_in, int32_t d_out,
                        int32_t n_tasks, const int32_t *rank_off,
                        const int32_t *task_of, const void *W, const void *A,
                        const void *B, const float *s, const void *dy,
                        int64_t nrows, const int64_t *rows, double *dx_out,
                        double *g_out)
{
    int32_t r_max = 0;
    for (int32_t t = 0; t < n_tasks; ++t)
        if (rank_off[t + 1] - rank_off[t] > r_max)
            r_max = rank_off[t + 1] - rank_off[t];
    if (!rows && nrows != T)
        return -1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nrows; ++q) {
        const int64_t i = rows ? rows[q] : q;
        double *dx = dx_out + (size_t)q * d_in;
        /* base: dx = dy_i W^T */
        for (int32_t k = 0; k < d_in; ++k) {
            double acc = 0.0;
            for (int32_t j = 0; j < d_out; ++j)
                acc += load_elem(dy, dtype, (size_t)i * d_out + j) *
                       load_elem(W, dtype, (size_t)k * d_out + j);
            dx[k] = acc;
        }
        if (g_out)
            for (int32_t p = 0; p < r_max; ++p)
                g_out[(size_t)q * r_max + p] = 0.0;
        const int32_t t = task_of[i];
        if (t < 0)
            continue;
        const int32_t r0 = rank_off[t], r = rank_off[t + 1] - rank_off[t];
        double *g = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        /* g = B_t dy_i */
        for (int32_t p = 0; p < r; ++p) {
            double acc = 0.0;
            for (int32_t j = 0; j < d_out; ++j)
                acc += load_elem(dy, dtype, (size_t)i * d_out + j) *
                       load_elem(B, dtype, (size_t)(r0 + p) * d_out + j);
            g[p] = acc;
            if (g_out)
                g_out[(size_t)q * r_max + p] = acc;
        }
        /* dx += s_t * (g A_t) */
        const double st = (double)s[t];
        for (int32_t k = 0; k < d_in; ++k) {
            double lo = 0.0;
            for (int32_t p = 0; p < r; ++p)
                lo += g[p] * load_elem(A, dtype, (size_t)(r0 + p) * d_in + k);
            dx[k] += st * lo;
        }
        free(g);
    }
    return 0;
}

/*
 * Adapter gradients over the whole batch: dA [R_tot, d_in], dB [R_tot, d_out],
 * overwritten.  Each stacked rank row is one independent sum over the tokens of
 * its task, taken in token order.
 */
int lobra_oracle_bwd_grads(int dtype, int64_t T, int32_t d_in, int32_t d_out,
                           int32_t n_tasks, const int32_t *rank_off,
                           const int32_t *task_of, const void *x,
                           const void *A, const void *B, const float *s,
                           const void *dy, double *dA, double *dB)
{
    const int32_t R_tot = n_tasks > 0 ? rank_off[n_tasks] : 0;
    if (R_tot == 0)
        return 0;
    /* per-token h_i[p] and g_i[p] for the token's own task, ragged by row */
    int32_t r_max = 0;
    for (int32_t t = 0; t < n_tasks; ++t)
        if (rank_off[t + 1] - rank_off[t] > r_max)
            r_max = rank_off[t + 1] - rank_off[t];
    double *h = (double *)calloc((size_t)(T > 0 ? T : 1) * r_max, sizeof(double));
    double *g = (double *)calloc((size_t)(T > 0 ? T : 1) * r_max, sizeof(double));
    if (!h || !g) {
        free(h);
        free(g);
        return -2;
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < T; ++i) {
        const int32_t t = task_of[i];
        if (t < 0)
            continue;
        const int32_t r0 = rank_off[t], r = rank_off[t + 1] - rank_off[t];
        for (int32_t p = 0; p < r; ++p) {
            double ah = 0.0, ag = 0.0;
            for (int32_t k = 0; k < d_in; ++k)
                ah += load_elem(x, dtype, (size_t)i * d_in + k) *
                      load_elem(A, dtype, (size_t)(r0 + p) * d_in + k);
            for (int32_t j = 0; j < d_out; ++j)
                ag += load_elem(dy, dtype, (size_t)i * d_out + j) *
                      load_elem(B, dtype, (size_t)(r0 + p) * d_out + j);
            h[(size_t)i * r_max + p] = ah;
            g[(size_t)i * r_max + p] = ag;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t R = 0; R < R_tot; ++R) {
        int32_t t = 0;
        while (rank_off[t + 1] <= R)
            ++t;
        const int32_t p = R - rank_off[t];
        double *dBrow = dB + (size_t)R * d_out;
        double *dArow = dA + (size_t)R * d_in;
        for (int32_t j = 0; j < d_out; ++j)
            dBrow[j] = 0.0;
        for (int32_t k = 0; k < d_in; ++k)
            dArow[k] = 0.0;
        for (int64_t i = 0; i < T; ++i) {
            if (task_of[i] != t)
                continue;
            const double hi = h[(size_t)i * r_max + p];
            const double gi = g[(size_t)i * r_max + p];
            for (int32_t j = 0; j < d_out; ++j)
                dBrow[j] += hi * load_elem(dy, dtype, (size_t)i * d_out + j);
            for (int32_t k = 0; k < d_in; ++k)
                dArow[k] += gi * load_elem(x, dtype, (size_t)i * d_in + k);
        }
        const double st = (double)s[t];
        for (int32_t j = 0; j < d_out; ++j)
            dBrow[j] *= st;
        for (int32_t k = 0; k < d_in; ++k)
            dArow[k] *= st;
    }
    free(h);
    free(g);
    return 0;
}
