/* A client of libduhl written in plain C (C99, compiled with gcc): device memory from the HIP
 * runtime's C interface, the default stream, no C++ and no Python objects anywhere near the
 * library.  It shows that include/duhl.h is usable as the C ABI it claims to be, and gives the
 * tests a second, independent caller of every step of a round (Algorithm 1).
 *
 * duhl_c_client_rounds: dense Lasso with the matrix in device memory; `rounds` rounds of
 *     gap (eq. (4)) -> select m (eq. (11)) -> commit -> one sequential pass in ascending order
 * and the state after them copied back.  Returns 0, or the negative duhl_status / 100 + the
 * positive HIP error of the call that failed. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdlib.h>

#include "duhl.h"

#define HIP_TRY(expr)                          \
    do {                                       \
        hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) {                \
            rc = 100 + (int)e_;                \
            goto done;                         \
        }                                      \
    } while (0)

#define DUHL_TRY(expr)                         \
    do {                                       \
        duhl_status s_ = (expr);               \
        if (s_ != DUHL_OK) {                   \
            rc = (int)s_;                      \
            goto done;                         \
        }                                      \
    } while (0)

int duhl_c_client_rounds(const float *A_host, const float *b_host, int64_t d, int64_t n, int64_t ld,
                         double lambda, int64_t m, int rounds, float *alpha_out, float *v_out,
                         float *z_out, int32_t *P_out, double *objective_out, double *gap_out)
{
    int rc = 0;
    float *A = NULL, *b = NULL;
    duhl_ctx *ctx = NULL;
    HIP_TRY(hipSetDevice(0));
    HIP_TRY(hipMalloc((void **)&A, sizeof(float) * (size_t)(ld * n)));
    HIP_TRY(hipMalloc((void **)&b, sizeof(float) * (size_t)d));
    HIP_TRY(hipMemcpy(A, A_host, sizeof(float) * (size_t)(ld * n), hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(b, b_host, sizeof(float) * (size_t)d, hipMemcpyHostToDevice));
    DUHL_TRY(duhl_create(&ctx, DUHL_LASSO, d, n, m, 0, NULL, NULL));
    DUHL_TRY(duhl_set_data_dense(ctx, A, ld, DUHL_RESIDENT_DEVICE, b, lambda));
    for (int r = 0; r < rounds; ++r) {
        double rho = 0.0;
        int64_t swapped = 0;
        DUHL_TRY(duhl_gap(ctx, NULL, 0, NULL));
        DUHL_TRY(duhl_select(ctx, m, NULL, &swapped, &rho));
        if (!(rho >= 1.0 - 1e-9) || swapped < 0 || swapped > m) {
            rc = -50;                                       /* eq. (7): rho >= 1 for the top m */
            goto done;
        }
        DUHL_TRY(duhl_commit_swap(ctx));
        if (duhl_working_set_size(ctx) != m) {
            rc = -51;
            goto done;
        }
        DUHL_TRY(duhl_cd_epoch(ctx, DUHL_CD_SEQUENTIAL, NULL, 0, 0, 0));
    }
    DUHL_TRY(duhl_gap(ctx, NULL, 0, gap_out));
    DUHL_TRY(duhl_objective(ctx, objective_out));
    DUHL_TRY(duhl_get(ctx, DUHL_ALPHA, alpha_out, n));
    DUHL_TRY(duhl_get(ctx, DUHL_V, v_out, d));
    DUHL_TRY(duhl_get(ctx, DUHL_Z, z_out, n));
    DUHL_TRY(duhl_get(ctx, DUHL_P, P_out, m));
done:
    duhl_destroy(ctx);
    if (A) (void)hipFree(A);
    if (b) (void)hipFree(b);
    return rc;
}

/* Calls whose arguments are rejected before any device work: each must return the documented
 * status and touch nothing.  Needs no GPU; the tests run it under AddressSanitizer.  Returns 0, or
 * the number of the first check that failed. */
int duhl_c_client_argument_checks(void)
{
    duhl_ctx *ctx = NULL;
    float buf[8] = {0};
    double sum = 0.0;
    int64_t n_out = 0;
    char err[64];
    int k = 0;
#define EXPECT(call, want) do { ++k; if ((call) != (want)) return k; } while (0)
    EXPECT(duhl_create(NULL, DUHL_LASSO, 4, 4, 2, 0, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_create(&ctx, (duhl_model)9, 4, 4, 2, 0, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_create(&ctx, DUHL_LASSO, 0, 4, 2, 0, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_create(&ctx, DUHL_LASSO, 4, -1, 2, 0, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_create(&ctx, DUHL_LASSO, 4, 4, 0, 0, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_create(&ctx, DUHL_LASSO, (int64_t)1 << 29, 4, 2, 0, NULL, NULL), DUHL_EINVAL);
    if (ctx != NULL) return 100;
    EXPECT(duhl_set_eta(NULL, 0.5), DUHL_EINVAL);
    EXPECT(duhl_set_wait_limit(NULL, 1), DUHL_EINVAL);
    EXPECT(duhl_set_data_dense(NULL, buf, 4, DUHL_RESIDENT_DEVICE, buf, 0.1), DUHL_EINVAL);
    EXPECT(duhl_set_data_dense_chunks(NULL, NULL, 1, 1, 4, buf, 0.1), DUHL_EINVAL);
    EXPECT(duhl_set_data_csr(NULL, NULL, NULL, NULL, DUHL_RESIDENT_DEVICE, buf, 0.1), DUHL_EINVAL);
    EXPECT(duhl_gap(NULL, NULL, 0, &sum), DUHL_EINVAL);
    EXPECT(duhl_select(NULL, 1, NULL, &n_out, &sum), DUHL_EINVAL);
    EXPECT(duhl_select_rule_apply(NULL, DUHL_SELECT_RANDOM, 0, 1, NULL, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_host_sample_begin(NULL, NULL, 0, 1), DUHL_EINVAL);
    EXPECT(duhl_host_sample_end(NULL, 1, &n_out), DUHL_EINVAL);
    EXPECT(duhl_commit_swap(NULL), DUHL_EINVAL);
    EXPECT(duhl_cd_epoch(NULL, DUHL_CD_ASYNC, NULL, 0, 0, 0), DUHL_EINVAL);
    EXPECT(duhl_run(NULL, NULL, NULL), DUHL_EINVAL);
    EXPECT(duhl_objective(NULL, &sum), DUHL_EINVAL);
    EXPECT(duhl_recompute_v(NULL), DUHL_EINVAL);
    EXPECT(duhl_get(NULL, DUHL_ALPHA, buf, 4), DUHL_EINVAL);
    EXPECT(duhl_set(NULL, DUHL_ALPHA, buf, 4), DUHL_EINVAL);
    EXPECT(duhl_device_ptr(NULL, DUHL_ALPHA, NULL), DUHL_EINVAL);
    EXPECT(duhl_probe_stream_read(NULL, buf, 16, 1, &sum), DUHL_EINVAL);
    EXPECT(duhl_selection_threshold(NULL, buf), DUHL_EINVAL);
    EXPECT(duhl_resident_columns(NULL, &n_out), DUHL_EINVAL);
    EXPECT(duhl_swap_stats(NULL, &n_out, &sum), DUHL_EINVAL);
    EXPECT(duhl_cd_stats(NULL, &n_out, &n_out, &n_out, &sum), DUHL_EINVAL);
    EXPECT(duhl_probe_scatter_add(NULL, 1000, 1, &sum), DUHL_EINVAL);
    if (duhl_working_set_size(NULL) != 0) return 101;
    if (duhl_last_error(NULL) == NULL) return 102;
    duhl_destroy(NULL);
    /* the entry point without a context checks everything it can on the host */
    EXPECT(duhl_gap_dense_static((duhl_model)7, 4, 2, buf, 4, buf, buf, NULL, 0.1, 1.0, 1.0, NULL, 0, buf, NULL, 0,
                                 NULL, err, (int64_t)sizeof err), DUHL_EINVAL);
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 0, 2, buf, 4, buf, buf, NULL, 0.1, 1.0, 1.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, (int64_t)sizeof err), DUHL_EINVAL);
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 4, 2, NULL, 4, buf, buf, NULL, 0.1, 1.0, 1.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, (int64_t)sizeof err), DUHL_EINVAL);
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 4, 2, buf, 3, buf, buf, NULL, 0.1, 1.0, 1.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, (int64_t)sizeof err), DUHL_EINVAL);
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 4, 2, buf, 4, buf, buf, NULL, -0.1, 1.0, 1.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, 1), DUHL_EINVAL);                     /* a one-byte error buffer */
    EXPECT(duhl_gap_dense_static(DUHL_ELASTIC_NET, 4, 2, buf, 4, buf, buf, NULL, 0.1, 0.0, 0.0, NULL, 0, buf, NULL, 0,
                                 NULL, NULL, 0), DUHL_EINVAL);
    EXPECT(duhl_gap_dense_static(DUHL_SVM, 4, 2, buf, 4, buf, buf, NULL, 0.1, 1.0, 0.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, (int64_t)sizeof err), DUHL_EINVAL);   /* no labels */
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 4, 2, buf, 4, buf, buf, NULL, 0.1, 1.0, -1.0, NULL, 0, buf, NULL, 0, NULL,
                                 err, (int64_t)sizeof err), DUHL_EINVAL);   /* negative bound */
    EXPECT(duhl_gap_dense_static(DUHL_LASSO, 4, 2, buf, 4, buf, buf, NULL, 0.1, 1.0, 1.0, (const int32_t *)buf, 3, buf,
                                 NULL, 0, NULL, err, (int64_t)sizeof err), DUHL_EINVAL);   /* count > n */
#undef EXPECT
    return 0;
}

