/*
 * CPU checker for neighbourhood aggregation -- TEST INFRASTRUCTURE, not product code.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares nothing with the HIP library.
 *
 * What it computes is the from-scratch aggregation of one snapshot (paper Section 3.2,
 * Eq. 1: Agg_t = F_t *aggr G_t), written as the plain definition:
 *
 *   deg(v)  = self_loop + number of in-edges (u -> v)
 *   Y[u]    = p(u) * X[u]
 *   S[v]    = self_loop * Y[v] + sum over in-edges (u -> v), ascending u, of Y[u]
 *   Agg[v]  = q(v) * S[v]
 *
 *   mode 0 (sum):  p = 1, q = 1
 *   mode 1 (mean): p = 1, q = 1/deg            (the paper lists mean() as built in, Section 3.2)
 *   mode 2 (sym):  p = q = deg^(-1/2)          (GCN normalisation D^-1/2 (A+I) D^-1/2 with D the
 *                                               row sums of A+I; not in the paper -- parity unpinned
 *                                               by the paper, pinned to this definition by the dense
 *                                               adjacency test)
 *   deg == 0 gives a scale of 0.
 *
 * Everything is fp64.  The graph is a CSR by destination: row v lists the sources u of (u -> v).
 * Rows are independent, so the optional OpenMP row partition does not change any result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double scale_of(int mode, int side /*0 = p (source), 1 = q (target)*/, double deg)
{
    if (mode == 0) return 1.0;
    if (mode == 1 && side == 0) return 1.0;
    if (deg <= 0.0) return 0.0;
    if (mode == 1) return 1.0 / deg;
    return 1.0 / sqrt(deg);
}

/* deg_out[N]: self_loop + in-degree */
void oracle_degrees(int64_t n, const int64_t *row_ptr, int self_loop, double *deg_out)
{
    for (int64_t v = 0; v < n; ++v) deg_out[v] = (double)(row_ptr[v + 1] - row_ptr[v]) + (self_loop ? 1.0 : 0.0);
}

/*
 * x:[n,d] row-major.  s_out (may be NULL) and agg_out: [n,d].
 * Returns 0, or -1 on a column index out of range.
 */
int oracle_aggregate(int64_t n, int32_t d, const int64_t *row_ptr, const int32_t *col, const double *x, int mode,
                     int self_loop, double *s_out, double *agg_out)
{
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        double *acc = (double *)calloc((size_t)d, sizeof(double));
        double degv = (double)(row_ptr[v + 1] - row_ptr[v]) + (self_loop ? 1.0 : 0.0);
        if (self_loop) {
            double p = scale_of(mode, 0, degv);
            for (int32_t j = 0; j < d; ++j) acc[j] += p * x[v * d + j];
        }
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            int64_t u = col[e];
            if (u < 0 || u >= n) {
                bad = 1;
                continue;
            }
            double degu = (double)(row_ptr[u + 1] - row_ptr[u]) + (self_loop ? 1.0 : 0.0);
            double p = scale_of(mode, 0, degu);
            for (int32_t j = 0; j < d; ++j) acc[j] += p * x[u * d + j];
        }
        double q = scale_of(mode, 1, degv);
        for (int32_t j = 0; j < d; ++j) {
            if (s_out) s_out[v * d + j] = acc[j];
            agg_out[v * d + j] = q * acc[j];
        }
        free(acc);
    }
    return bad ? -1 : 0;
}

/*
 * Adjoint of oracle_aggregate with respect to x: given g = dLoss/dAgg [n,d], writes
 * dx = dLoss/dX [n,d]:   dx[u] = p(u) * ( self_loop * q(u) g[u] + sum over out-edges (u -> v) of q(v) g[v] ).
 * Written as the serial scatter the definition gives (every edge pushes its target's gradient
 * back to its source); degrees are constants of the graph.
 */
int oracle_aggregate_adjoint(int64_t n, int32_t d, const int64_t *row_ptr, const int32_t *col, const double *g,
                             int mode, int self_loop, double *dx_out)
{
    memset(dx_out, 0, sizeof(double) * (size_t)n * (size_t)d);
    for (int64_t v = 0; v < n; ++v) {
        double degv = (double)(row_ptr[v + 1] - row_ptr[v]) + (self_loop ? 1.0 : 0.0);
        double q = scale_of(mode, 1, degv);
        if (self_loop) {
            double p = scale_of(mode, 0, degv);
            for (int32_t j = 0; j < d; ++j) dx_out[v * d + j] += p * q * g[v * d + j];
        }
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
            int64_t u = col[e];
            if (u < 0 || u >= n) return -1;
            double degu = (double)(row_ptr[u + 1] - row_ptr[u]) + (self_loop ? 1.0 : 0.0);
            double p = scale_of(mode, 0, degu);
            for (int32_t j = 0; j < d; ++j) dx_out[u * d + j] += p * q * g[v * d + j];
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
