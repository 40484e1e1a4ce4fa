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
