/*
 * CPU oracle for neighbour aggregation (TEST INFRASTRUCTURE, not product code).
 *
 * Plain definition of the GCN aggregation of eq. (1)/(3) of the paper,
 *     a_v = sum over u in N_in(v) + {v} of  w(v,u) * h_u ,
 * over a matrix given in compressed sparse row form: row v lists its in-neighbours
 * u ascending with the weight w(v,u).  All arithmetic is fp64; every row is summed
 * sequentially in ascending entry order, so the result does not depend on the number
 * of threads.  No blocking, no reordering.  Shares no code with the HIP library.
 *
 * Parallelism: rows are independent (one thread sums one row), OpenMP over rows.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Y[i, 0:f] = sum_k val[k] * X[colidx[k], 0:f] for k in [rowptr[r], rowptr[r+1]),
 * r = rows[i] if rows != NULL else r = i.  Yabs (nullable) receives
 * sum_k |val[k] * X[colidx[k], j]|, the scale against which rounding error of any
 * summation order is bounded.  X is [*, ldx] doubles, Y/Yabs are [n_out, ldy]. */
void oracle_aggregate(int64_t n_out, const int64_t *rows,
                      const int64_t *rowptr, const int32_t *colidx, const float *val,
                      const double *X, int64_t ldx, int64_t f,
                      double *Y, double *Yabs, int64_t ldy)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t r = rows ? rows[i] : i;
        double *y = Y + i * ldy;
        double *ya = Yabs ? Yabs + i * ldy : NULL;
        for (int64_t j = 0; j < f; ++j) y[j] = 0.0;
        if (ya) for (int64_t j = 0; j < f; ++j) ya[j] = 0.0;
        for (int64_t k = rowptr[r]; k < rowptr[r + 1]; ++k) {
            const double w = (double)val[k];
            const double *x = X + (int64_t)colidx[k] * ldx;
            for (int64_t j = 0; j < f; ++j) {
                double t = w * x[j];
                y[j] += t;
                if (ya) ya[j] += fabs(t);
            }
        }
    }
}

/* Transposed product written as the definition of a transpose: every stored entry
 * (v, u, w) of the row-form matrix sends w * G[v, :] to row u of the output.
 * Sequential on purpose (the scatter has write conflicts); entries are visited in
 * ascending (v, k) order.  Gin must hold n_cols rows; it is overwritten. */
void oracle_aggregate_transposed_scatter(int64_t n_rows, int64_t n_cols,
                                         const int64_t *rowptr, const int32_t *colidx, const float *val,
                                         const double *G, int64_t ldg, int64_t f,
                                         double *Gin, int64_t ldo)
{
    for (int64_t u = 0; u < n_cols; ++u)
        for (int64_t j = 0; j < f; ++j) Gin[u * ldo + j] = 0.0;
    for (int64_t v = 0; v < n_rows; ++v) {
        const double *g = G + v * ldg;
        for (int64_t k = rowptr[v]; k < rowptr[v + 1]; ++k) {
            const double w = (double)val[k];
            double *o = Gin + (int64_t)colidx[k] * ldo;
            for (int64_t j = 0; j < f; ++j) o[j] += w * g[j];
        }
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the row loop uses from now on (timing on one core beside all cores; the result does not
 * depend on it: every row is summed sequentially). */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
