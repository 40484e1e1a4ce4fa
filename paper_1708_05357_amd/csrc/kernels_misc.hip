// Small kernels around the hot path: objective, (re)building the shared vector, input checks.
#include "duhl_internal.h"

namespace duhl {

namespace {

// Sum of squares of v (all models) and, over the coordinates, sum |alpha_i| (Lasso),
// sum y_i alpha_i (SVM) or eta/2 sum alpha_i^2 + (1-eta) sum |alpha_i| (elastic net): the two
// reductions of the objectives in Appendix C / D.
template <int MODEL>
__global__ __launch_bounds__(256) void objective_kernel(const float *v, int64_t d, const float *alpha,
                                                        const float *y, int64_t n, double *partials,
                                                        double eta)
{
    __shared__ double sh[2][4];
    double sq = 0.0, lin = 0.0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < d; i += stride) {
        const double x = (double)v[i];
        sq += x * x;
    }
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const double ai = (double)alpha[i];
        if (MODEL == DUHL_LASSO) lin += fabs(ai);
        else if (MODEL == DUHL_ELASTIC_NET) lin += 0.5 * eta * ai * ai + (1.0 - eta) * fabs(ai);
        else lin += (double)y[i] * ai;
    }
    sq = wave_sum(sq);
    lin = wave_sum(lin);
    if ((threadIdx.x & 63) == 0) { sh[0][threadIdx.x >> 6] = sq; sh[1][threadIdx.x >> 6] = lin; }
    __syncthreads();
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = (sh[0][0] + sh[0][1]) + (sh[0][2] + sh[0][3]);
        partials[2 * blockIdx.x + 1] = (sh[1][0] + sh[1][1]) + (sh[1][2] + sh[1][3]);
    }
}

__global__ __launch_bounds__(1024) void objective_finish_kernel(const double *partials, int64_t blocks,
                                                                double *scalars)
{
    __shared__ double sh[2][16];
    double sq = 0.0, lin = 0.0;
    for (int64_t i = threadIdx.x; i < blocks; i += 1024) { sq += partials[2 * i]; lin += partials[2 * i + 1]; }
    sq = wave_sum(sq);
    lin = wave_sum(lin);
    if ((threadIdx.x & 63) == 0) { sh[0][threadIdx.x >> 6] = sq; sh[1][threadIdx.x >> 6] = lin; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < 16; ++w) { a += sh[0][w]; b += sh[1][w]; }
        scalars[S_OBJ_SQ] = a;
        scalars[S_OBJ_LIN] = b;
    }
}

// v := -b (Lasso, Appendix D: v = A alpha - b) or 0 (SVM: v = A alpha).
__global__ void init_v_kernel(float *v, const float *b, int64_t d)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < d) v[i] = b ? -b[i] : 0.0f;
}

// v += sum_j a_j alpha_j, one wavefront per column with alpha_j != 0.
__global__ __launch_bounds__(256) void accumulate_v_kernel(const ColView cv, int64_t d, int64_t n,
                                                           const float *alpha, float *v)
{
    const int lane = threadIdx.x & 63;
    const int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n) return;
    const float aj = alpha[j];
    if (aj == 0.0f) return;
    if (cv.base) {
        const float *col = cv.col(j);
        for (int64_t r = lane; r < d; r += 64)
            (void)__hip_atomic_fetch_add(v + r, col[r] * aj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        for (int64_t e = cv.rowptr[j] + lane; e < cv.rowptr[j + 1]; e += 64)
            (void)__hip_atomic_fetch_add(v + cv.colidx[e], cv.val[e] * aj, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    }
}

// u += a_j / ||a_j|| for `samples` evenly spaced columns j: ||u||^2 then tells how strongly the
// columns share a direction (samples + samples*(samples-1)*mean cosine).
__global__ __launch_bounds__(256) void corr_sample_kernel(const ColView cv, int64_t d, int64_t n,
                                                          const float *q, int samples, float *u)
{
    const int lane = threadIdx.x & 63;
    const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= samples) return;
    const int64_t j = s * (n / samples);
    const float qj = q[j];
    if (!(qj > 0.0f)) return;
    const float w = rsqrtf(qj);
    if (cv.base) {
        const float *col = cv.col(j);
        for (int64_t r = lane; r < d; r += 64)
            (void)__hip_atomic_fetch_add(u + r, col[r] * w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        for (int64_t e = cv.rowptr[j] + lane; e < cv.rowptr[j + 1]; e += 64)
            (void)__hip_atomic_fetch_add(u + cv.colidx[e], cv.val[e] * w, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The same two passes over a batch of columns staged from host memory: column s of the batch holds
// coordinate idx[s].
__global__ __launch_bounds__(256) void accumulate_v_staged_kernel(const float *stage, int64_t lds, int64_t d,
                                                                  const int32_t *idx, int64_t count,
                                                                  const float *alpha, float *v)
{
    const int lane = threadIdx.x & 63;
    const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= count) return;
    const float aj = alpha[idx[s]];
    if (aj == 0.0f) return;
    const float *col = stage + s * lds;
    for (int64_t r = lane; r < d; r += 64)
        (void)__hip_atomic_fetch_add(v + r, col[r] * aj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__global__ __launch_bounds__(256) void corr_sample_staged_kernel(const float *stage, int64_t lds, int64_t d,
                                                                 const int32_t *idx, int64_t count,
                                                                 const float *q, float *u)
{
    const int lane = threadIdx.x & 63;
    const int64_t s = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= count) return;
    const float qj = q[idx[s]];
    if (!(qj > 0.0f)) return;
    const float w = rsqrtf(qj);
    const float *col = stage + s * lds;
    for (int64_t r = lane; r < d; r += 64)
        (void)__hip_atomic_fetch_add(u + r, col[r] * w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ||b||^2 in double (for the Lipschitzing bound of Appendix E).
__global__ __launch_bounds__(1024) void sumsq_kernel(const float *b, int64_t d, double *out)
{
    __shared__ double sh[16];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < d; i += 1024) s += (double)b[i] * (double)b[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += sh[w];
        *out = t;
    }
}

// Input checks; bits of *flags: 1 = label not +-1, 2 = rowptr[0] != 0, decreasing, negative or beyond nnz,
// 4 = column index out of range or not strictly increasing inside a row, 8 = non-finite target.
__global__ void validate_kernel(int model, int64_t d, int64_t n, const float *target,
                                const int64_t *rowptr, const int32_t *colidx, int64_t nnz, uint32_t *flags)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t f = 0;
    if (model == DUHL_SVM) {
        if (i < n && !(target[i] == 1.0f || target[i] == -1.0f)) f |= 1u;
    } else {
        if (i < d && !isfinite(target[i])) f |= 8u;
    }
    if (rowptr && i < n) {
        const int64_t beg = rowptr[i], end = rowptr[i + 1];
        if (i == 0 && beg != 0) f |= 2u;
        // a row is only walked if it lies inside the arrays: a rowptr that is locally increasing
        // but points past the nnz = rowptr[n] entries the caller allocated must not be followed
        if (beg < 0 || end < beg || end > nnz) f |= 2u;
        else {
            int32_t prev = -1;
            for (int64_t e = beg; e < end; ++e) {
                const int32_t k = colidx[e];
                if (k <= prev || k >= d) { f |= 4u; break; }
                prev = k;
            }
        }
    }
    if (f) atomicOr(flags, f);
}

// Bit 16 of *flags: a column norm that is not finite, i.e. a NaN or an infinity (or an overflow of
// the sum of squares) somewhere in that column of the matrix.
__global__ void check_norms_kernel(const float *q, int64_t n, uint32_t *flags)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && !isfinite(q[i])) atomicOr(flags, 16u);
}

__global__ void fill_i32_kernel(int32_t *p, int64_t n, int32_t value)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}
__global__ void fill_f32_kernel(float *p, int64_t n, float value)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

}  // namespace

hipError_t launch_objective(duhl_ctx *c)
{
    const int64_t len = c->d > c->n ? c->d : c->n;
    int64_t grid = (len + 255) / 256;
    if (grid > 1024) grid = 1024;
    if (c->model == DUHL_LASSO)
        hipLaunchKernelGGL(objective_kernel<DUHL_LASSO>, dim3(grid), dim3(256), 0, c->compute, c->v,
                           c->d, c->alpha, c->target, c->n, c->partials, 0.0);
    else if (c->model == DUHL_ELASTIC_NET)
        hipLaunchKernelGGL(objective_kernel<DUHL_ELASTIC_NET>, dim3(grid), dim3(256), 0, c->compute, c->v,
                           c->d, c->alpha, c->target, c->n, c->partials, c->eta_active);
    else
        hipLaunchKernelGGL(objective_kernel<DUHL_SVM>, dim3(grid), dim3(256), 0, c->compute, c->v,
                           c->d, c->alpha, c->target, c->n, c->partials, 0.0);
    hipLaunchKernelGGL(objective_finish_kernel, dim3(1), dim3(1024), 0, c->compute, c->partials, grid,
                       c->scalars);
    return hipGetLastError();
}

hipError_t launch_init_v(duhl_ctx *c)
{
    hipLaunchKernelGGL(init_v_kernel, dim3((c->d + 255) / 256), dim3(256), 0, c->compute, c->v,
                       c->model != DUHL_SVM ? c->target : nullptr, c->d);
    if (c->model == DUHL_LASSO)
        hipLaunchKernelGGL(sumsq_kernel, dim3(1), dim3(1024), 0, c->compute, c->target, c->d,
                           c->scalars + S_BSQ);
    return hipGetLastError();
}

hipError_t launch_accumulate_v(duhl_ctx *c)
{
    if (c->pageable) return staged_accumulate_v(c);
    hipLaunchKernelGGL(accumulate_v_kernel, dim3((c->n + 3) / 4), dim3(256), 0, c->compute, c->cv, c->d,
                       c->n, c->alpha, c->v);
    return hipGetLastError();
}

hipError_t launch_corr_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx, float *u)
{
    hipLaunchKernelGGL(corr_sample_staged_kernel, dim3((b.count + 3) / 4), dim3(256), 0, c->compute, b.stage,
                       b.lds, c->d, idx + b.k0, b.count, c->q, u);
    return hipGetLastError();
}

hipError_t launch_accumulate_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx)
{
    hipLaunchKernelGGL(accumulate_v_staged_kernel, dim3((b.count + 3) / 4), dim3(256), 0, c->compute, b.stage,
                       b.lds, c->d, idx + b.k0, b.count, c->alpha, c->v);
    return hipGetLastError();
}

hipError_t launch_corr_sample(duhl_ctx *c, float *u, int samples)
{
    hipLaunchKernelGGL(fill_f32_kernel, dim3((c->d + 255) / 256), dim3(256), 0, c->compute, u, c->d, 0.0f);
    if (c->pageable) {
        const hipError_t e = staged_corr_sample(c, u, samples);
        if (e != hipSuccess) return e;
    } else {
        hipLaunchKernelGGL(corr_sample_kernel, dim3((samples + 3) / 4), dim3(256), 0, c->compute, c->cv, c->d,
                           c->n, c->q, samples, u);
    }
    hipLaunchKernelGGL(sumsq_kernel, dim3(1), dim3(1024), 0, c->compute, u, c->d, c->scalars + S_CORR);
    return hipGetLastError();
}

// Read-only streaming yardstick: grid-stride 16-byte non-temporal loads, 8 in flight per lane.
// The sum is compared with a value it cannot take so that the loads stay.
__global__ __launch_bounds__(256) void stream_read_kernel(const float4 *p, int64_t n4, float *sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float acc = 0.0f;
    for (; i + stride * 7 < n4; i += stride * 8) {
        float4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = stream_load4(p + i + stride * u);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (x[u].x + x[u].y) + (x[u].z + x[u].w);
    }
    for (; i < n4; i += stride) {
        const float4 x = stream_load4(p + i);
        acc += (x.x + x.y) + (x.z + x.w);
    }
    if (acc == -1.2345678e38f) *sink = acc;
}

hipError_t launch_stream_read(duhl_ctx *c, const void *dev, int64_t bytes, float *sink)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(c->num_cu * 32), dim3(256), 0, c->compute,
                       static_cast<const float4 *>(dev), bytes / 16, sink);
    return hipGetLastError();
}

// Scatter yardstick: fp32 atomic adds of +0 to pseudo-random elements of x (which they leave as it
// is), `per` from each of the grid's threads -- the memory operation behind the concurrent steps on
// CSR data, with nothing else around it.
__global__ __launch_bounds__(256) void scatter_add_kernel(float *x, uint32_t n, int per)
{
    const uint32_t tid = blockIdx.x * 256u + threadIdx.x;
    for (int k = 0; k < per; ++k) {
        uint32_t h = tid * 0x9e3779b9u + (uint32_t)k * 0x85ebca6bu;
        h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
        (void)__hip_atomic_fetch_add(x + h % n, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

hipError_t launch_scatter_add(duhl_ctx *c, int64_t ops, int64_t *done)
{
    const int64_t threads = (int64_t)c->num_cu * 8 * 256;
    int64_t per = (ops + threads - 1) / threads;
    if (per < 1) per = 1;
    if (per > (1 << 20)) per = 1 << 20;
    *done = per * threads;
    hipLaunchKernelGGL(scatter_add_kernel, dim3(c->num_cu * 8), dim3(256), 0, c->compute, c->v, (uint32_t)c->d, (int)per);
    return hipGetLastError();
}

hipError_t launch_validate(duhl_ctx *c)
{
    const int64_t len = c->d > c->n ? c->d : c->n;
    hipLaunchKernelGGL(validate_kernel, dim3((len + 255) / 256), dim3(256), 0, c->compute, (int)c->model,
                       c->d, c->n, c->target, c->cv.rowptr, c->cv.colidx, c->nnz, &c->sel->error);
    return hipGetLastError();
}

hipError_t launch_check_norms(duhl_ctx *c)
{
    hipLaunchKernelGGL(check_norms_kernel, dim3((c->n + 255) / 256), dim3(256), 0, c->compute, c->q, c->n,
                       &c->sel->error);
    return hipGetLastError();
}

hipError_t launch_fill_i32(hipStream_t s, int32_t *p, int64_t n, int32_t value)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n, value);
    return hipGetLastError();
}
hipError_t launch_fill_f32(hipStream_t s, float *p, int64_t n, float value)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n, value);
    return hipGetLastError();
}

}  // namespace duhl
