/*
 * DuHL reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, sequential, double-precision CPU statement of what the DuHL hot path
 * computes: objective, per-coordinate duality gaps, top-m selection and exact
 * coordinate-descent passes for the Lasso and for the hinge-loss SVM dual.
 * It exists so that the HIP library can be checked against something that can
 * be compared with the paper by eye.  It shares no code with the HIP path, is
 * never tuned, and only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.
 *
 * Conventions (paper, Section 2, eq. (1)): A = [a_1 ... a_n] in R^{d x n};
 * coordinate i owns column a_i.  The data are given in single precision
 * (Section 5.3); every sum here is carried in double.
 *   dense : column i is the contiguous run A[i*ld .. i*ld+d)
 *   sparse: CSR of A^T, i.e. row i of the CSR arrays lists the non-zeros of a_i
 *           (for the SVM dual a column of A is one sample, Appendix D).
 * Shared vector (Appendix D): Lasso / elastic net v = A alpha - b, SVM v = A alpha.
 * Lambda := lambda * d is the product that the Lasso formulas use throughout.
 *
 * Pins: tests/test_oracle_pins.py (closed forms, brute force, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    int64_t d;             /* length of a column                       */
    int64_t n;             /* number of coordinates = columns           */
    const float *dense;    /* non-NULL: dense column-major, stride ld   */
    int64_t ld;
    const int64_t *rowptr; /* dense == NULL: CSR of A^T, n+1 entries    */
    const int32_t *colidx; /* position inside the column, in [0, d)     */
    const float *val;
} or_matrix;

/* a_j^T v */
static double col_dot(const or_matrix *M, int64_t j, const double *v)
{
    double s = 0.0;
    if (M->dense) {
        const float *a = M->dense + j * M->ld;
        for (int64_t k = 0; k < M->d; ++k) s += (double)a[k] * v[k];
    } else {
        for (int64_t p = M->rowptr[j]; p < M->rowptr[j + 1]; ++p)
            s += (double)M->val[p] * v[M->colidx[p]];
    }
    return s;
}

/* v += a_j * delta */
static void col_axpy(const or_matrix *M, int64_t j, double delta, double *v)
{
    if (M->dense) {
        const float *a = M->dense + j * M->ld;
        for (int64_t k = 0; k < M->d; ++k) v[k] += (double)a[k] * delta;
    } else {
        for (int64_t p = M->rowptr[j]; p < M->rowptr[j + 1]; ++p)
            v[M->colidx[p]] += (double)M->val[p] * delta;
    }
}

/* q_j = ||a_j||^2 for every column (Appendix D, the denominators of the updates). */
void or_col_sqnorms(const or_matrix *M, double *q)
{
    for (int64_t j = 0; j < M->n; ++j) {
        double s = 0.0;
        if (M->dense) {
            const float *a = M->dense + j * M->ld;
            for (int64_t k = 0; k < M->d; ++k) s += (double)a[k] * a[k];
        } else {
            for (int64_t p = M->rowptr[j]; p < M->rowptr[j + 1]; ++p)
                s += (double)M->val[p] * M->val[p];
        }
        q[j] = s;
    }
}

/* v := A alpha - shift (shift may be NULL).  Used for initialisation and by the
 * tests that check that the running v stays equal to its definition. */
void or_matvec(const or_matrix *M, const double *alpha, const float *shift, double *v)
{
    for (int64_t k = 0; k < M->d; ++k) v[k] = shift ? -(double)shift[k] : 0.0;
    for (int64_t j = 0; j < M->n; ++j)
        if (alpha[j] != 0.0) col_axpy(M, j, alpha[j], v);
}

/* Lasso objective, Appendix C(b): ||A alpha - b||^2 / (2d) + lambda ||alpha||_1,
 * evaluated from v = A alpha - b. */
double or_lasso_objective(const or_matrix *M, const double *v, const double *alpha,
                          double lambda)
{
    double sq = 0.0, l1 = 0.0;
    for (int64_t k = 0; k < M->d; ++k) sq += v[k] * v[k];
    for (int64_t j = 0; j < M->n; ++j) l1 += fabs(alpha[j]);
    return sq / (2.0 * (double)M->d) + lambda * l1;
}

/* SVM dual objective, Appendix C(c): -(1/n) sum y_i alpha_i + ||A alpha||^2/(2 lambda n^2),
 * evaluated from v = A alpha. */
double or_svm_objective(const or_matrix *M, const double *v, const double *alpha,
                        const float *y, double lambda)
{
    double sq = 0.0, lin = 0.0, n = (double)M->n;
    for (int64_t k = 0; k < M->d; ++k) sq += v[k] * v[k];
    for (int64_t j = 0; j < M->n; ++j) lin += (double)y[j] * alpha[j];
    return -lin / n + sq / (2.0 * lambda * n * n);
}

/* The bound of the Lipschitzing trick, Appendix E (Lasso): B = ||b||^2 / (2 lambda d). */
double or_lasso_bound(const or_matrix *M, const float *b, double lambda)
{
    double sq = 0.0;
    for (int64_t k = 0; k < M->d; ++k) sq += (double)b[k] * b[k];
    return sq / (2.0 * lambda * (double)M->d);
}

/* Lasso per-coordinate gaps, Appendix E with w := A alpha - b = v:
 *   z_i = (1/d) [ alpha_i c_i + B [|c_i| - Lambda]_+ + Lambda |alpha_i| ],  c_i = a_i^T v.
 * Evaluates coordinates idx[0..count) (idx NULL: 0..count-1), writes z[idx[k]],
 * returns the sum of what it wrote (eq. (4): the total gap when all are asked for). */
double or_lasso_gaps(const or_matrix *M, const double *v, const double *alpha,
                     double lambda, double B, const int32_t *idx, int64_t count, double *z)
{
    const double d = (double)M->d, Lam = lambda * d;
    double total = 0.0;
    for (int64_t k = 0; k < count; ++k) {
        int64_t i = idx ? idx[k] : k;
        double c = col_dot(M, i, v);
        double over = fabs(c) - Lam;
        if (over < 0.0) over = 0.0;
        z[i] = (alpha[i] * c + B * over + Lam * fabs(alpha[i])) / d;
        total += z[i];
    }
    return total;
}

/* SVM per-coordinate gaps, Appendix E with w := A alpha / (lambda n):
 *   z_i = (1/n) [ alpha_i s_i + max(0, 1 - y_i s_i) - y_i alpha_i ],  s_i = a_i^T w. */
double or_svm_gaps(const or_matrix *M, const double *v, const double *alpha, const float *y,
                   double lambda, const int32_t *idx, int64_t count, double *z)
{
    const double n = (double)M->n;
    double total = 0.0;
    for (int64_t k = 0; k < count; ++k) {
        int64_t i = idx ? idx[k] : k;
        double s = col_dot(M, i, v) / (lambda * n);
        double hinge = 1.0 - (double)y[i] * s;
        if (hinge < 0.0) hinge = 0.0;
        z[i] = (alpha[i] * s + hinge - (double)y[i] * alpha[i]) / n;
        total += z[i];
    }
    return total;
}

/* Working-set selection, eq. (11)/(13): the m coordinates with the largest z.
 * Ties go to the smaller index; the result is listed in ascending index order.
 * Implemented as the definition: sort all coordinates, keep the first m. */
typedef struct { double z; int64_t i; } or_key;
static int key_cmp(const void *pa, const void *pb)
{
    const or_key *a = (const or_key *)pa, *b = (const or_key *)pb;
    if (a->z > b->z) return -1;
    if (a->z < b->z) return 1;
    return (a->i > b->i) - (a->i < b->i);
}
static int idx_cmp(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}
int or_select_topm(int64_t n, const double *z, int64_t m, int32_t *P)
{
    if (m > n) m = n;
    or_key *keys = (or_key *)malloc((size_t)n * sizeof(or_key));
    if (!keys) return -1;
    for (int64_t i = 0; i < n; ++i) { keys[i].z = z[i]; keys[i].i = i; }
    qsort(keys, (size_t)n, sizeof(or_key), key_cmp);   /* total order: no ties left */
    for (int64_t k = 0; k < m; ++k) P[k] = (int32_t)keys[k].i;
    free(keys);
    qsort(P, (size_t)m, sizeof(int32_t), idx_cmp);
    return 0;
}

/* rho of eq. (7): mean gap over P divided by mean gap over all coordinates. */
double or_rho(int64_t n, const double *z, const int32_t *P, int64_t m)
{
    double sp = 0.0, sa = 0.0;
    for (int64_t k = 0; k < m; ++k) sp += z[P[k]];
    for (int64_t i = 0; i < n; ++i) sa += z[i];
    return (sp / (double)m) / (sa / (double)n);
}

/* One exact Lasso coordinate step (Appendix D, elastic net with eta = 0):
 *   gamma = (alpha_j q_j - a_j^T v) / q_j,  tau = Lambda / q_j,
 *   alpha_j <- sign(gamma) [|gamma| - tau]_+,  v <- v + a_j (alpha_j_new - alpha_j).
 * A zero column has its minimiser at 0. */
static void lasso_step(const or_matrix *M, int64_t j, double qj, double Lam,
                       double *alpha, double *v)
{
    double newa = 0.0;
    if (qj > 0.0) {
        double gamma = (alpha[j] * qj - col_dot(M, j, v)) / qj;
        double tau = Lam / qj;
        double mag = fabs(gamma) - tau;
        newa = mag > 0.0 ? (gamma > 0.0 ? mag : -mag) : 0.0;
    }
    double delta = newa - alpha[j];
    if (delta != 0.0) col_axpy(M, j, delta, v);
    alpha[j] = newa;
}

/* One exact SVM-dual coordinate step (Appendix D):
 *   Delta = (y_j - a_j^T v / (lambda n)) / (q_j / (lambda n)),
 *   alpha_j <- y_j max(0, min(1, y_j (alpha_j + Delta))),  v <- v + a_j (alpha_j_new - alpha_j).
 * A zero column leaves only the linear term, minimised at y_j alpha_j = 1. */
static void svm_step(const or_matrix *M, int64_t j, double qj, double lam_n, double yj,
                     double *alpha, double *v)
{
    double newa = yj;
    if (qj > 0.0) {
        double step = (yj - col_dot(M, j, v) / lam_n) / (qj / lam_n);
        double t = yj * (alpha[j] + step);
        if (t < 0.0) t = 0.0;
        if (t > 1.0) t = 1.0;
        newa = yj * t;
    }
    double delta = newa - alpha[j];
    if (delta != 0.0) col_axpy(M, j, delta, v);
    alpha[j] = newa;
}

/* One pass of coordinate descent (Algorithm 3 applied to the block, Section 3.1) over
 * order[0..count): coordinates are solved one after the other, each against the v
 * left by the previous one. */
void or_lasso_cd_pass(const or_matrix *M, const double *q, double lambda,
                      const int32_t *order, int64_t count, double *alpha, double *v)
{
    const double Lam = lambda * (double)M->d;
    for (int64_t k = 0; k < count; ++k) lasso_step(M, order[k], q[order[k]], Lam, alpha, v);
}

void or_svm_cd_pass(const or_matrix *M, const double *q, const float *y, double lambda,
                    const int32_t *order, int64_t count, double *alpha, double *v)
{
    const double lam_n = lambda * (double)M->n;
    for (int64_t k = 0; k < count; ++k)
        svm_step(M, order[k], q[order[k]], lam_n, (double)y[order[k]], alpha, v);
}

/* ---- elastic net with eta in (0,1]; eta = 1 is ridge regression (Appendix C(a), D) ---------- */

/* Objective of Appendix D: ||A alpha - b||^2/(2d) + lambda (eta/2 ||alpha||^2 + (1-eta)||alpha||_1). */
double or_enet_objective(const or_matrix *M, const double *v, const double *alpha, double lambda,
                         double eta)
{
    double sq = 0.0, l1 = 0.0, l2 = 0.0;
    for (int64_t k = 0; k < M->d; ++k) sq += v[k] * v[k];
    for (int64_t j = 0; j < M->n; ++j) { l1 += fabs(alpha[j]); l2 += alpha[j] * alpha[j]; }
    return sq / (2.0 * (double)M->d) + lambda * (0.5 * eta * l2 + (1.0 - eta) * l1);
}

/* Coordinate gaps from eq. (4) with w = A alpha - b, g_i(a) = lambda(eta/2 a^2 + (1-eta)|a|) and its
 * conjugate g_i*(u) = [|u| - lambda(1-eta)]_+^2 / (2 lambda eta):
 *   z_i = (1/d) [ alpha_i c_i + Lambda (eta/2 alpha_i^2 + (1-eta)|alpha_i|)
 *                 + [|c_i| - Lambda(1-eta)]_+^2 / (2 Lambda eta) ],   c_i = a_i^T v, Lambda = lambda d.
 * For eta = 1 this is the ridge gap printed in Appendix E. */
double or_enet_gaps(const or_matrix *M, const double *v, const double *alpha, double lambda,
                    double eta, const int32_t *idx, int64_t count, double *z)
{
    const double d = (double)M->d, Lam = lambda * d;
    double total = 0.0;
    for (int64_t k = 0; k < count; ++k) {
        int64_t i = idx ? idx[k] : k;
        double c = col_dot(M, i, v);
        double over = fabs(c) - Lam * (1.0 - eta);
        if (over < 0.0) over = 0.0;
        z[i] = (alpha[i] * c + Lam * (0.5 * eta * alpha[i] * alpha[i] + (1.0 - eta) * fabs(alpha[i]))
                + over * over / (2.0 * Lam * eta)) / d;
        total += z[i];
    }
    return total;
}

/* Exact coordinate step of Appendix D:
 *   gamma = (alpha_j q_j - a_j^T v)/(q_j + Lambda eta),  tau = Lambda(1-eta)/(q_j + Lambda eta),
 *   alpha_j <- sign(gamma)[|gamma| - tau]_+ . */
void or_enet_cd_pass(const or_matrix *M, const double *q, double lambda, double eta,
                     const int32_t *order, int64_t count, double *alpha, double *v)
{
    const double Lam = lambda * (double)M->d;
    for (int64_t k = 0; k < count; ++k) {
        const int64_t j = order[k];
        const double den = q[j] + Lam * eta;
        const double gamma = (alpha[j] * q[j] - col_dot(M, j, v)) / den;
        const double tau = Lam * (1.0 - eta) / den;
        const double mag = fabs(gamma) - tau;
        const double newa = mag > 0.0 ? (gamma > 0.0 ? mag : -mag) : 0.0;
        const double delta = newa - alpha[j];
        if (delta != 0.0) col_axpy(M, j, delta, v);
        alpha[j] = newa;
    }
}
