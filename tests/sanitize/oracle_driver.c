/* Runs every routine of the CPU oracle (oracle/duhl_oracle.c) on small instances under
 * AddressSanitizer and UndefinedBehaviorSanitizer: the three problems worked by hand from
 * App. C, D and E of the paper (tests/golden/hand_worked.json), a sparse copy of one of them, and
 * selections with ties.  Values are checked too, so that a build that "runs clean" because it does
 * nothing fails.  Exit status 0 = all checks passed and no sanitizer report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int64_t d, n;
    const float *dense;
    int64_t ld;
    const int64_t *rowptr;
    const int32_t *colidx;
    const float *val;
} or_matrix;

double or_lasso_objective(const or_matrix *, const double *, const double *, double);
double or_svm_objective(const or_matrix *, const double *, const double *, const float *, double);
double or_lasso_bound(const or_matrix *, const float *, double);
double or_lasso_gaps(const or_matrix *, const double *, const double *, double, double, const int32_t *, int64_t, double *);
double or_svm_gaps(const or_matrix *, const double *, const double *, const float *, double, const int32_t *, int64_t, double *);
int or_select_topm(int64_t, const double *, int64_t, int32_t *);
double or_rho(int64_t, const double *, const int32_t *, int64_t);
void or_col_sqnorms(const or_matrix *, double *);
void or_matvec(const or_matrix *, const double *, const float *, double *);
void or_lasso_cd_pass(const or_matrix *, const double *, double, const int32_t *, int64_t, double *, double *);
void or_svm_cd_pass(const or_matrix *, const double *, const float *, double, const int32_t *, int64_t, double *, double *);
double or_enet_objective(const or_matrix *, const double *, const double *, double, double);
double or_enet_gaps(const or_matrix *, const double *, const double *, double, double, const int32_t *, int64_t, double *);
void or_enet_cd_pass(const or_matrix *, const double *, double, double, const int32_t *, int64_t, double *, double *);

static int failures = 0;
#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)
static int near(double a, double b) { return fabs(a - b) <= 1e-12 * (1.0 + fabs(b)); }

/* every array on the heap, exactly as long as it must be: an access one past the end is caught */
static void *heap(size_t bytes, const void *init)
{
    char *p = malloc(bytes ? bytes : 1);
    for (size_t i = 0; init && i < bytes; ++i) p[i] = ((const char *)init)[i];
    return p;
}

static void lasso_identity(int sparse)
{
    /* A = I (2x2), b = (3,1), lambda = 0.5: B = 5, z(0) = (5,0), O(0) = 2.5; after steps on 0, 1:
     * alpha = (2,0), v = (-1,-1), O = 1.5, z = (0,0) */
    const float cols_[4] = {1, 0, 0, 1}, b_[2] = {3, 1}, ones_[2] = {1, 1};
    const int64_t rp_[3] = {0, 1, 2};
    const int32_t ci_[2] = {0, 1}, order_[2] = {0, 1};
    float *cols = heap(sizeof cols_, cols_), *b = heap(sizeof b_, b_), *ones = heap(sizeof ones_, ones_);
    int64_t *rp = heap(sizeof rp_, rp_);
    int32_t *ci = heap(sizeof ci_, ci_), *order = heap(sizeof order_, order_);
    or_matrix M = {2, 2, sparse ? NULL : cols, 2, sparse ? rp : NULL, sparse ? ci : NULL, sparse ? ones : NULL};
    double *q = heap(2 * sizeof(double), NULL), *alpha = heap(2 * sizeof(double), NULL);
    double *v = heap(2 * sizeof(double), NULL), *z = heap(2 * sizeof(double), NULL);
    alpha[0] = alpha[1] = 0.0;
    or_col_sqnorms(&M, q);
    CHECK(q[0] == 1.0 && q[1] == 1.0);
    or_matvec(&M, alpha, b, v);
    CHECK(v[0] == -3.0 && v[1] == -1.0);
    const double B = or_lasso_bound(&M, b, 0.5);
    CHECK(near(B, 5.0));
    CHECK(near(or_lasso_objective(&M, v, alpha, 0.5), 2.5));
    CHECK(near(or_lasso_gaps(&M, v, alpha, 0.5, B, NULL, 2, z), 5.0) && near(z[0], 5.0) && z[1] == 0.0);
    or_lasso_cd_pass(&M, q, 0.5, order, 2, alpha, v);
    CHECK(near(alpha[0], 2.0) && alpha[1] == 0.0 && near(v[0], -1.0) && near(v[1], -1.0));
    CHECK(near(or_lasso_objective(&M, v, alpha, 0.5), 1.5));
    z[0] = z[1] = -1.0;
    CHECK(near(or_lasso_gaps(&M, v, alpha, 0.5, B, order + 1, 1, z), 0.0) && z[0] == -1.0 && near(z[1], 0.0));
    free(cols); free(b); free(ones); free(rp); free(ci); free(order); free(q); free(alpha); free(v); free(z);
}

static void svm_two_points(void)
{
    /* d = 1, a_0 = (1), a_1 = (-1), y = (+1,-1), lambda = 0.5: z(0) = (1/2, 1/2), after steps
     * alpha = (1,0), v = 1, O = -0.25, z = (0,0) */
    const float cols_[2] = {1, -1}, y_[2] = {1, -1};
    const int32_t order_[2] = {0, 1};
    float *cols = heap(sizeof cols_, cols_), *y = heap(sizeof y_, y_);
    int32_t *order = heap(sizeof order_, order_);
    or_matrix M = {1, 2, cols, 1, NULL, NULL, NULL};
    double *q = heap(2 * sizeof(double), NULL), *alpha = heap(2 * sizeof(double), NULL);
    double *v = heap(1 * sizeof(double), NULL), *z = heap(2 * sizeof(double), NULL);
    alpha[0] = alpha[1] = 0.0;
    or_col_sqnorms(&M, q);
    or_matvec(&M, alpha, NULL, v);
    CHECK(v[0] == 0.0);
    CHECK(near(or_svm_gaps(&M, v, alpha, y, 0.5, NULL, 2, z), 1.0) && near(z[0], 0.5) && near(z[1], 0.5));
    CHECK(or_svm_objective(&M, v, alpha, y, 0.5) == 0.0);
    or_svm_cd_pass(&M, q, y, 0.5, order, 2, alpha, v);
    CHECK(near(alpha[0], 1.0) && alpha[1] == 0.0 && near(v[0], 1.0));
    CHECK(near(or_svm_objective(&M, v, alpha, y, 0.5), -0.25));
    CHECK(near(or_svm_gaps(&M, v, alpha, y, 0.5, NULL, 2, z), 0.0));
    free(cols); free(y); free(order); free(q); free(alpha); free(v); free(z);
}

static void ridge_one_column(void)
{
    /* d = 2, a = (1,0), b = (2,0), lambda = 0.5, eta = 1: z(0) = 1, O(0) = 1; one step: alpha = 1,
     * v = (-1,0), O = 0.5, z = 0 */
    const float cols_[2] = {1, 0}, b_[2] = {2, 0};
    const int32_t order_[1] = {0};
    float *cols = heap(sizeof cols_, cols_), *b = heap(sizeof b_, b_);
    int32_t *order = heap(sizeof order_, order_);
    or_matrix M = {2, 1, cols, 2, NULL, NULL, NULL};
    double *q = heap(sizeof(double), NULL), *alpha = heap(sizeof(double), NULL);
    double *v = heap(2 * sizeof(double), NULL), *z = heap(sizeof(double), NULL);
    alpha[0] = 0.0;
    or_col_sqnorms(&M, q);
    or_matvec(&M, alpha, b, v);
    CHECK(near(or_enet_objective(&M, v, alpha, 0.5, 1.0), 1.0));
    CHECK(near(or_enet_gaps(&M, v, alpha, 0.5, 1.0, NULL, 1, z), 1.0));
    or_enet_cd_pass(&M, q, 0.5, 1.0, order, 1, alpha, v);
    CHECK(near(alpha[0], 1.0) && near(v[0], -1.0) && v[1] == 0.0);
    CHECK(near(or_enet_objective(&M, v, alpha, 0.5, 1.0), 0.5));
    CHECK(near(or_enet_gaps(&M, v, alpha, 0.5, 1.0, NULL, 1, z), 0.0));
    free(cols); free(b); free(order); free(q); free(alpha); free(v); free(z);
}

static void selection(void)
{
    const double z_[6] = {0.5, 2.0, 0.5, 0.5, 3.0, 0.5};
    double *z = heap(sizeof z_, z_);
    int32_t *P = heap(4 * sizeof(int32_t), NULL);
    CHECK(or_select_topm(6, z, 4, P) == 0);
    CHECK(P[0] == 0 && P[1] == 1 && P[2] == 2 && P[3] == 4);          /* ties to the smaller index */
    CHECK(near(or_rho(6, z, P, 4), (6.0 / 4.0) / (7.0 / 6.0)));
    int32_t *all = heap(6 * sizeof(int32_t), NULL);
    CHECK(or_select_topm(6, z, 60, all) == 0 && all[5] == 5);          /* m > n: everything */
    free(z); free(P); free(all);
}

int main(void)
{
    lasso_identity(0);
    lasso_identity(1);
    svm_two_points();
    ridge_one_column();
    selection();
    if (failures) return 1;
    puts("oracle under sanitizers: ok");
    return 0;
}
