/*
 * CPU oracle for the sufficient-factor (SF) hot path of Sufficient Factor
 * Broadcasting.  TEST INFRASTRUCTURE ONLY: it defines the expected results for
 * the tests, the smoke check and the bench's cpu_baseline leg.  The product
 * (the HIP library) never links, loads or calls anything in this file, and this
 * file shares no code with it.
 *
 * Everything is plain fp64, row-major, written as the defining sums with no
 * blocking, fusion or reordering; the only concession to run time is an OpenMP
 * "parallel for" over independent rows/samples.
 *
 * Notation (Section 2, problem (P)): W is J x D; a sample's update is the
 * rank-1 matrix u v^T with u = d f(Wa,b) / d(Wa), v = a (Section 2.1,
 * "Proximal SGD").  A batch of N sufficient factors is stored as U[N][J],
 * V[N][D], one SF per row (the buffer of SF pairs of Section 4.2).
 *
 * Pins: every function below is pinned by tests/test_oracle_pins.py
 * (finite differences of the stated losses, closed forms, library reductions,
 * algebraic invariants).  Values that come from the benchmark recipe and not
 * from the paper (lambda, iteration counts, margin, the 1/2 in the SC loss)
 * are pinned only through those self-consistency checks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <omp.h>

int sfbo_num_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------ */
/* Reconstruction and application of the summed rank-1 updates:        */
/*   W <- W - eta * sum_{i<N} u_i v_i^T                                 */
/* (Section 3: every worker applies the same sum over all SF pairs;     */
/*  Section 2.1: W <- W - eta * dW.)  The paper's 1/K mini-batch factor */
/* is folded into eta by the caller.                                    */
/* ------------------------------------------------------------------ */
void sfbo_apply(double* W, const double* U, const double* V,
                int64_t N, int64_t J, int64_t D, double eta)
{
    /* Row j of the sum is sum_i U[i][j] * v_i: the rank-1 terms are added one
       at a time, in index order, into a row accumulator. */
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
#pragma omp for schedule(static)
        for (int64_t j = 0; j < J; ++j) {
            for (int64_t d = 0; d < D; ++d) acc[d] = 0.0;
            for (int64_t i = 0; i < N; ++i) {
                double uij = U[i * J + j];
                for (int64_t d = 0; d < D; ++d)
                    acc[d] += uij * V[i * D + d];
            }
            for (int64_t d = 0; d < D; ++d)
                W[j * D + d] -= eta * acc[d];
        }
        free(acc);
    }
}

/* ------------------------------------------------------------------ */
/* Signed low-rank updates ("Low-rank Extensions", Section 2.1): an      */
/* update that is a short signed sum of outer products, e.g. u1 v1^T -   */
/* u2 v2^T, is applied as W <- W - eta * sum_i c_i u_i v_i^T with one    */
/* coefficient per factor pair.                                          */
/* ------------------------------------------------------------------ */
void sfbo_apply_signed(double* W, const double* U, const double* V, const double* c,
                       int64_t N, int64_t J, int64_t D, double eta)
{
    for (int64_t j = 0; j < J; ++j)
        for (int64_t d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int64_t i = 0; i < N; ++i)
                acc += c[i] * U[i * J + j] * V[i * D + d];
            W[j * D + d] -= eta * acc;
        }
}

/* ------------------------------------------------------------------ */
/* Multiclass logistic regression (Section 1; Figure 2).                */
/* f_i(z) = -log softmax(z)[y_i] with z = W x_i, so by the chain rule   */
/* u_i = softmax(z) - onehot(y_i) and v_i = x_i.  The row maximum is    */
/* subtracted before exponentiation (overflow guard, not in the paper;  */
/* it cancels exactly).                                                  */
/* loss[i] (nullable) = log sum_j exp(z_j) - z_{y_i}.                   */
/* ------------------------------------------------------------------ */
void sfbo_mlr_sf(const double* W, const double* X, const int32_t* y,
                 int64_t J, int64_t D, int64_t B, double* U, double* loss)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        double* u = U + i * J;
        for (int64_t j = 0; j < J; ++j) {
            double z = 0.0;
            for (int64_t d = 0; d < D; ++d)
                z += W[j * D + d] * X[i * D + d];
            u[j] = z;
        }
        double m = u[0];
        for (int64_t j = 1; j < J; ++j)
            if (u[j] > m) m = u[j];
        double zy = u[y[i]];
        double s = 0.0;
        for (int64_t j = 0; j < J; ++j)
            s += exp(u[j] - m);
        for (int64_t j = 0; j < J; ++j)
            u[j] = exp(u[j] - m) / s;
        u[y[i]] -= 1.0;
        if (loss) loss[i] = m + log(s) - zy;
    }
}

/* ------------------------------------------------------------------ */
/* Sparse data (Section 5, experimental setup: the data are sparse, so   */
/* the second factors v_i = x_i and the update matrices are sparse, and  */
/* work is done on the non-zeros only).  Row i of a CSR matrix holds the */
/* pairs (indices[t], values[t]), indptr[i] <= t < indptr[i+1], with     */
/* distinct column indices.                                              */
/*   z_j = sum_t W[j][indices[t]] * values[t]   (then as sfbo_mlr_sf)    */
/*   W[j][indices[t]] -= eta * sum_i U[i][j] * values[t]  (columns no    */
/*   v_i touches keep their value bit for bit)                           */
/* ------------------------------------------------------------------ */
void sfbo_mlr_sf_csr(const double* W, const int64_t* indptr, const int32_t* indices,
                     const double* values, const int32_t* y,
                     int64_t J, int64_t D, int64_t B, double* U, double* loss)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        double* u = U + i * J;
        for (int64_t j = 0; j < J; ++j) {
            double z = 0.0;
            for (int64_t t = indptr[i]; t < indptr[i + 1]; ++t)
                z += W[j * D + indices[t]] * values[t];
            u[j] = z;
        }
        double m = u[0];
        for (int64_t j = 1; j < J; ++j)
            if (u[j] > m) m = u[j];
        double zy = u[y[i]];
        double s = 0.0;
        for (int64_t j = 0; j < J; ++j)
            s += exp(u[j] - m);
        for (int64_t j = 0; j < J; ++j)
            u[j] = exp(u[j] - m) / s;
        u[y[i]] -= 1.0;
        if (loss) loss[i] = m + log(s) - zy;
    }
}

void sfbo_apply_csr(double* W, const double* U, const int64_t* indptr, const int32_t* indices,
                    const double* values, int64_t N, int64_t J, int64_t D, double eta)
{
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
        unsigned char* hit = (unsigned char*)malloc((size_t)(D > 0 ? D : 1));
#pragma omp for schedule(static)
        for (int64_t j = 0; j < J; ++j) {
            for (int64_t d = 0; d < D; ++d) { acc[d] = 0.0; hit[d] = 0; }
            for (int64_t i = 0; i < N; ++i) {
                double uij = U[i * J + j];
                for (int64_t t = indptr[i]; t < indptr[i + 1]; ++t) {
                    acc[indices[t]] += uij * values[t];
                    hit[indices[t]] = 1;
                }
            }
            for (int64_t d = 0; d < D; ++d)
                if (hit[d]) W[j * D + d] -= eta * acc[d];
        }
        free(acc);
        free(hit);
    }
}

/* ------------------------------------------------------------------ */
/* Distance metric learning (Section 2: a_i is the difference of the    */
/* pair's feature vectors; f_i is quadratic for similar pairs and a     */
/* hinge for dissimilar pairs; W is the K x D projection).              */
/*   a_i = x_i - y_i,  q_i = W a_i,  d_i = ||q_i||^2                    */
/*   similar    (sim > 0): f = d_i,                 u = 2 q_i           */
/*   dissimilar (sim < 0): f = max(0, margin - d_i), u = -2 q_i if      */
/*                         d_i < margin (strictly), else 0              */
/*   v_i = a_i.  Inactive rows of U are zero; *n_active counts rows     */
/*   with a non-zero coefficient.                                       */
/* ------------------------------------------------------------------ */
void sfbo_dml_sf(const double* W, const double* X, const double* Y,
                 const int8_t* sim, int64_t K, int64_t D, int64_t B,
                 double margin, double* U, double* V,
                 int32_t* n_active, double* loss)
{
    int32_t active = 0;
#pragma omp parallel for schedule(static) reduction(+ : active)
    for (int64_t i = 0; i < B; ++i) {
        double* v = V + i * D;
        double* u = U + i * K;
        for (int64_t d = 0; d < D; ++d)
            v[d] = X[i * D + d] - Y[i * D + d];
        double dist = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double q = 0.0;
            for (int64_t d = 0; d < D; ++d)
                q += W[k * D + d] * v[d];
            u[k] = q;
            dist += q * q;
        }
        double c, f;
        if (sim[i] > 0) {
            c = 2.0;
            f = dist;
        } else if (dist < margin) {
            c = -2.0;
            f = margin - dist;
        } else {
            c = 0.0;
            f = 0.0;
        }
        for (int64_t k = 0; k < K; ++k)
            u[k] = c * u[k];
        if (c != 0.0) active += 1;
        if (loss) loss[i] = f;
    }
    if (n_active) *n_active = active;
}

/* ------------------------------------------------------------------ */
/* Sparse coding (Section 2; Figure 3).  Rows of W are the J basis      */
/* vectors (the paper's dictionary B is W^T), a sample's code is a in   */
/* R^J, f = 1/2 ||x - W^T a||^2 + lambda ||a||_1 in a.                   */
/* Code solve (the paper leaves the solver open; the benchmark recipe   */
/* fixes it): ISTA with step 1/L, L from power iteration on W^T W.      */
/* ------------------------------------------------------------------ */

/* L estimate: b <- 1/sqrt(D) (all entries); repeat power_iters times   */
/* c = W b, g = W^T c, L = ||g||_2, b = g / L.  Returns the last L.     */
double sfbo_sc_lipschitz(const double* W, int64_t J, int64_t D, int32_t power_iters)
{
    double* b = (double*)malloc(sizeof(double) * (size_t)D);
    double* c = (double*)malloc(sizeof(double) * (size_t)J);
    double* g = (double*)malloc(sizeof(double) * (size_t)D);
    double L = 0.0;
    for (int64_t d = 0; d < D; ++d) b[d] = 1.0 / sqrt((double)D);
    for (int32_t it = 0; it < power_iters; ++it) {
        for (int64_t j = 0; j < J; ++j) {
            double s = 0.0;
            for (int64_t d = 0; d < D; ++d) s += W[j * D + d] * b[d];
            c[j] = s;
        }
        for (int64_t d = 0; d < D; ++d) {
            double s = 0.0;
            for (int64_t j = 0; j < J; ++j) s += W[j * D + d] * c[j];
            g[d] = s;
        }
        double nn = 0.0;
        for (int64_t d = 0; d < D; ++d) nn += g[d] * g[d];
        L = sqrt(nn);
        for (int64_t d = 0; d < D; ++d) b[d] = g[d] / L;
    }
    free(b); free(c); free(g);
    return L;
}

static double soft_threshold(double t, double theta)
{
    if (t > theta) return t - theta;
    if (t < -theta) return t + theta;
    return 0.0;
}

/* SFs of sparse coding: u_i = a_i (the code), v_i = x_i - W^T a_i (the  */
/* residual), so that W <- W + eta * U^T V is a descent step on f in W.  */
/*   a = 0; repeat ista_iters times:                                     */
/*      r = x - W^T a;  a <- soft(a + (W r)/L, lambda/L)                 */
/*   r = x - W^T a.                                                      */
/* L is passed in (sfbo_sc_lipschitz, or an exact eigenvalue in tests).  */
void sfbo_sc_sf(const double* W, const double* X, int64_t J, int64_t D, int64_t B,
                double lambda, int32_t ista_iters, double L,
                double* U, double* V)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        const double* x = X + i * D;
        double* a = U + i * J;
        double* r = V + i * D;
        for (int64_t j = 0; j < J; ++j) a[j] = 0.0;
        for (int32_t it = 0; it <= ista_iters; ++it) {
            for (int64_t d = 0; d < D; ++d) {
                double s = 0.0;
                for (int64_t j = 0; j < J; ++j) s += W[j * D + d] * a[j];
                r[d] = x[d] - s;
            }
            if (it == ista_iters) break;
            for (int64_t j = 0; j < J; ++j) {
                double gj = 0.0;
                for (int64_t d = 0; d < D; ++d) gj += W[j * D + d] * r[d];
                a[j] = soft_threshold(a[j] + gj / L, lambda / L);
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Proximal operator of sparse coding (Figure 3, "prox"): each basis    */
/* vector (a row of W here) is projected onto the unit l2 ball:         */
/*   mode 0 (project):   w <- w / ||w|| only if ||w|| > 1               */
/*   mode 1 (normalise): w <- w / ||w|| whenever ||w|| > 0 (benchmark    */
/*                       recipe's "row renormalisation")                */
/* ------------------------------------------------------------------ */
void sfbo_prox_rows(double* W, int64_t J, int64_t D, int32_t mode)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < J; ++j) {
        double nn = 0.0;
        for (int64_t d = 0; d < D; ++d) nn += W[j * D + d] * W[j * D + d];
        double nrm = sqrt(nn);
        int scale = (mode == 0) ? (nrm > 1.0) : (nrm > 0.0);
        if (scale)
            for (int64_t d = 0; d < D; ++d) W[j * D + d] /= nrm;
    }
}
