/*
 * CPU oracle for the factorization-machine (FM) pass of DS-FACTO.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, fp64 implementation written from
 * the paper's equations; it shares no code with the HIP library and is used
 * only by the tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * Notation (paper symbol in quotes where it differs):
 *   X  N x D sparse, CSR (rowptr,col,val) or CSC (colptr,row,cval)
 *   w0, w[D], V[D*K] row-major       model parameters (Section 3.2)
 *   a[N]   = X w                     linear aggregate (2nd term of eq. fm_model2)
 *   G[N*K] = X V                     latent aggregate, the paper's "a_ik" (eq. compute_a_jk)
 *   q[N]   = sum_j x_ij^2 |v_j|^2    the subtracted square term of eq. fm_model2
 *   r[N]                             loss multiplier, the paper's "G_i" (cases after eq. updates_v)
 *
 * Every loop follows the definition it cites; nothing is blocked, fused or
 * reordered.  OpenMP pragmas only split loops whose iterations are independent
 * (one row, or one column, per iteration), so results do not depend on the
 * thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section 3.2, eq. fm_model2 with the aggregate of eq. compute_a_jk:
 *   yhat_i = w0 + sum_j w_j x_ij + 1/2 sum_k ( G_ik^2 - sum_j v_jk^2 x_ij^2 ),
 * sums over the stored entries of row i only. */
void oracle_forward(int64_t N, int32_t K, const int64_t *rowptr, const int32_t *col,
                    const double *val, double w0, const double *w, const double *V,
                    double *a, double *G, double *q, double *yhat)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double ai = 0.0, qi = 0.0;
        double *Gi = G + i * K;
        for (int32_t k = 0; k < K; ++k) Gi[k] = 0.0;
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t j = col[e];
            const double x = val[e];
            ai += w[j] * x;
            for (int32_t k = 0; k < K; ++k) {
                const double v = V[j * K + k];
                Gi[k] += v * x;
                qi += v * v * x * x;
            }
        }
        double pair = 0.0;
        for (int32_t k = 0; k < K; ++k) pair += Gi[k] * Gi[k];
        a[i] = ai;
        q[i] = qi;
        yhat[i] = w0 + ai + 0.5 * (pair - qi);
    }
}

/* Prediction from stored aggregates (same formula, no pass over X). */
static double yhat_from_aux(double w0, double ai, const double *Gi, double qi, int32_t K)
{
    double pair = 0.0;
    for (int32_t k = 0; k < K; ++k) pair += Gi[k] * Gi[k];
    return w0 + ai + 0.5 * (pair - qi);
}

/* Loss value and multiplier r = s * dl/dyhat for one example.
 *   squared : l = 1/2 (yhat-y)^2,          dl/dyhat = yhat - y
 *   logistic: l = log(1+exp(-y yhat)),     dl/dyhat = -y / (1 + exp(y yhat)),  y in {-1,+1}
 * (the two cases printed after eq. updates_v; the loss constants are chosen so
 * that the printed multiplier is exactly the derivative).  exp() is only ever
 * taken of a non-positive argument. */
static void loss_one(int32_t loss, double s, double yh, double y, double *l, double *r)
{
    if (loss == 0) {
        const double d = yh - y;
        *l = 0.5 * d * d;
        *r = s * d;
    } else {
        const double m = y * yh;
        if (m > 0.0) {
            const double e = exp(-m);
            *l = log1p(e);
            *r = -s * y * e / (1.0 + e);
        } else {
            const double e = exp(m);
            *l = -m + log1p(e);
            *r = -s * y / (1.0 + e);
        }
    }
}

void oracle_loss_multiplier(int64_t N, int32_t loss, double s, const double *yhat,
                            const double *y, double *l, double *r)
{
    for (int64_t i = 0; i < N; ++i) loss_one(loss, s, yhat[i], y[i], &l[i], &r[i]);
}

/* CSR -> CSC by counting sort; rows come out ascending inside each column
 * because rows are visited in ascending order. */
void oracle_csr_to_csc(int64_t N, int64_t D, const int64_t *rowptr, const int32_t *col,
                       const double *val, int64_t *colptr, int32_t *row, double *cval)
{
    for (int64_t j = 0; j <= D; ++j) colptr[j] = 0;
    for (int64_t e = 0; e < rowptr[N]; ++e) colptr[col[e] + 1] += 1;
    for (int64_t j = 0; j < D; ++j) colptr[j + 1] += colptr[j];
    int64_t *next = (int64_t *)malloc((size_t)(D > 0 ? D : 1) * sizeof(int64_t));
    memcpy(next, colptr, (size_t)D * sizeof(int64_t));
    for (int64_t i = 0; i < N; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t dst = next[col[e]]++;
            row[dst] = (int32_t)i;
            cval[dst] = val[e];
        }
    free(next);
}

/* Gradient of  sum_i s*l_i + lambda_w/2 |w|^2 + lambda_v/2 |V|^2  (eq. fm_obj with
 * the data term scaled by s; r already carries s), from eqs. updates_w/updates_v
 * with the bias derivative and the regulariser signs of plain gradient descent:
 *   gw0   = sum_i r_i
 *   gw_j  = sum_i r_i x_ij + lambda_w w_j
 *   gV_jk = sum_i r_i ( x_ij G_ik - v_jk x_ij^2 ) + lambda_v v_jk */
void oracle_gradient(int64_t N, int64_t D, int32_t K, const int64_t *colptr, const int32_t *row,
                     const double *cval, const double *r, const double *G, const double *w,
                     const double *V, double lambda_w, double lambda_v,
                     double *gw0, double *gw, double *gV)
{
    double s0 = 0.0;
    for (int64_t i = 0; i < N; ++i) s0 += r[i];
    *gw0 = s0;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t j = 0; j < D; ++j) {
        double g = 0.0;
        double *gVj = gV + j * K;
        for (int32_t k = 0; k < K; ++k) gVj[k] = 0.0;
        for (int64_t e = colptr[j]; e < colptr[j + 1]; ++e) {
            const int64_t i = row[e];
            const double x = cval[e];
            g += r[i] * x;
            for (int32_t k = 0; k < K; ++k)
                gVj[k] += r[i] * (x * G[i * K + k] - V[j * K + k] * x * x);
        }
        gw[j] = g + lambda_w * w[j];
        for (int32_t k = 0; k < K; ++k) gVj[k] += lambda_v * V[j * K + k];
    }
}

/* Contiguous floor split used for both row blocks and column blocks
 * (Section 4.3: rows of X per worker, columns of {w,V} per block):
 * block b of n items in P blocks is [floor(b n / P), floor((b+1) n / P)). */
int64_t oracle_block_bound(int64_t n, int64_t P, int64_t b)
{
    return (int64_t)(((__int128)b * (__int128)n) / (__int128)P);
}

/* One cell step, phase A (Section 4.2/4.3, synchronous ring reading):
 * for the cell (rows [i_lo,i_hi), columns [j_lo,j_hi)):
 *   r_i  for the cell's rows from the aggregates as they stand,
 *   block gradient of every column of the cell over the cell's rows,
 *   gradient step on w_j, v_j with the share rho of the regulariser,
 *   record dw_j, dV_j and dn_j = |v_j new|^2 - |v_j old|^2.
 * All gradient sums use r and G as they stand when the step starts. */
void oracle_cell_update(int32_t K, int32_t loss, double s, double eta, double rho,
                        double lambda_w, double lambda_v,
                        int64_t i_lo, int64_t i_hi, int64_t j_lo, int64_t j_hi,
                        const int64_t *colptr, const int32_t *row, const double *cval,
                        const double *y, double w0, const double *a, const double *G,
                        const double *q, double *r, double *w, double *V,
                        double *dw, double *dV, double *dn)
{
    for (int64_t i = i_lo; i < i_hi; ++i) {
        double l;
        loss_one(loss, s, yhat_from_aux(w0, a[i], G + i * K, q[i], K), y[i], &l, &r[i]);
    }
    double *gV = (double *)malloc((size_t)K * sizeof(double));
    for (int64_t j = j_lo; j < j_hi; ++j) {
        double g = 0.0, s2 = 0.0;
        for (int32_t k = 0; k < K; ++k) gV[k] = 0.0;
        for (int64_t e = colptr[j]; e < colptr[j + 1]; ++e) {
            const int64_t i = row[e];
            if (i < i_lo || i >= i_hi) continue; /* entry belongs to another cell */
            const double x = cval[e];
            g += r[i] * x;
            s2 += r[i] * x * x;
            for (int32_t k = 0; k < K; ++k) gV[k] += r[i] * x * G[i * K + k];
        }
        double n_old = 0.0, n_new = 0.0;
        dw[j] = -eta * (g + rho * lambda_w * w[j]);
        w[j] += dw[j];
        for (int32_t k = 0; k < K; ++k) {
            const double v = V[j * K + k];
            const double d = -eta * (gV[k] - s2 * v + rho * lambda_v * v);
            dV[j * K + k] = d;
            V[j * K + k] = v + d;
            n_old += v * v;
            n_new += (v + d) * (v + d);
        }
        dn[j] = n_new - n_old;
    }
    free(gV);
}

/* The same cell step for a set of columns that need not be contiguous: the columns cols[0..ncols) that
 * a worker holds in one round of Algorithm 1 when every column is handed from worker to worker on its
 * own (Section 4.3: the parameter tuples circulate one by one; the initial placement is random).  The
 * step of one column is the step of oracle_cell_update restricted to that column. */
void oracle_cell_update_cols(int32_t K, int32_t loss, double s, double eta, double rho,
                             double lambda_w, double lambda_v,
                             int64_t i_lo, int64_t i_hi, int64_t ncols, const int32_t *cols,
                             const int64_t *colptr, const int32_t *row, const double *cval,
                             const double *y, double w0, const double *a, const double *G,
                             const double *q, double *r, double *w, double *V,
                             double *dw, double *dV, double *dn)
{
    for (int64_t i = i_lo; i < i_hi; ++i) {
        double l;
        loss_one(loss, s, yhat_from_aux(w0, a[i], G + i * K, q[i], K), y[i], &l, &r[i]);
    }
    double *gV = (double *)malloc((size_t)K * sizeof(double));
    for (int64_t t = 0; t < ncols; ++t) {
        const int64_t j = cols[t];
        double g = 0.0, s2 = 0.0;
        for (int32_t k = 0; k < K; ++k) gV[k] = 0.0;
        for (int64_t e = colptr[j]; e < colptr[j + 1]; ++e) {
            const int64_t i = row[e];
            if (i < i_lo || i >= i_hi) continue; /* entry belongs to another worker's rows */
            const double x = cval[e];
            g += r[i] * x;
            s2 += r[i] * x * x;
            for (int32_t k = 0; k < K; ++k) gV[k] += r[i] * x * G[i * K + k];
        }
        double n_old = 0.0, n_new = 0.0;
        dw[j] = -eta * (g + rho * lambda_w * w[j]);
        w[j] += dw[j];
        for (int32_t k = 0; k < K; ++k) {
            const double v = V[j * K + k];
            const double d = -eta * (gV[k] - s2 * v + rho * lambda_v * v);
            dV[j * K + k] = d;
            V[j * K + k] = v + d;
            n_old += v * v;
            n_new += (v + d) * (v + d);
        }
        dn[j] = n_new - n_old;
    }
    free(gV);
}

/* Phase B for such a set: the rows [i_lo,i_hi) take the changes of the columns with inset[j] != 0. */
void oracle_refresh_cols(int32_t K, int64_t i_lo, int64_t i_hi, const uint8_t *inset,
                         const int64_t *rowptr, const int32_t *col, const double *val,
                         const double *dw, const double *dV, const double *dn,
                         double *a, double *G, double *q)
{
    for (int64_t i = i_lo; i < i_hi; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t j = col[e];
            if (!inset[j]) continue;
            const double x = val[e];
            a[i] += x * dw[j];
            q[i] += x * x * dn[j];
            for (int32_t k = 0; k < K; ++k) G[i * K + k] += x * dV[j * K + k];
        }
}

/* Phase B, the incremental refresh (Section 4.2, "incremental synchronization"):
 * for rows [i_lo,i_hi) and their entries in columns [j_lo,j_hi):
 *   a_i += sum x_ij dw_j,  G_ik += sum x_ij dV_jk,  q_i += sum x_ij^2 dn_j. */
void oracle_refresh(int32_t K, int64_t i_lo, int64_t i_hi, int64_t j_lo, int64_t j_hi,
                    const int64_t *rowptr, const int32_t *col, const double *val,
                    const double *dw, const double *dV, const double *dn,
                    double *a, double *G, double *q)
{
    for (int64_t i = i_lo; i < i_hi; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t j = col[e];
            if (j < j_lo || j >= j_hi) continue;
            const double x = val[e];
            a[i] += x * dw[j];
            q[i] += x * x * dn[j];
            for (int32_t k = 0; k < K; ++k) G[i * K + k] += x * dV[j * K + k];
        }
}

/* r for every row from stored aggregates (used for the bias step that closes
 * a stratified epoch). */
void oracle_multiplier_from_aux(int64_t N, int32_t K, int32_t loss, double s, double w0,
                                const double *a, const double *G, const double *q,
                                const double *y, double *r)
{
    for (int64_t i = 0; i < N; ++i) {
        double l;
        loss_one(loss, s, yhat_from_aux(w0, a[i], G + i * K, q[i], K), y[i], &l, &r[i]);
    }
}
