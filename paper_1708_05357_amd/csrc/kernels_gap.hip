// Per-coordinate duality gaps (eq. (4) of the paper, model formulas of Appendix E).
//
// Dense: the pass is a transposed matrix-vector product c = A^T v followed by a scalar formula
// per column -- 2 flops per 4 bytes of A, so it is bound by HBM bandwidth.  One wavefront owns
// COLS columns at a time and streams them with 16-byte loads; the chunk of v it multiplies with
// is loaded once and reused for the COLS columns, so v costs 1/COLS of the traffic of A and is
// served by the cache hierarchy.  One group of columns per wavefront, one launch covers all
// groups: the hardware dispatcher balances the tail.
// Sparse: one group of G lanes per CSR row (rows of the paper's workloads have ~100 non-zeros,
// far fewer than a wavefront would need), gathers of v served by L2.
#include "duhl_internal.h"

namespace duhl {

struct GapArgs {
    ColView cv;
    ModelConst mc;
    int64_t d, n, count;
    const int32_t *idx;       // coordinates to refresh, or nullptr for 0..count-1
    const int32_t *slot_col;  // non-null: entry k is device slot k, refresh the column it holds
    const float *v, *alpha, *target;
    float *z, *q;
    double *partials;
};

// Which coordinate does list entry k stand for (-1: nothing to do).
__device__ __forceinline__ int64_t list_entry(const GapArgs &a, int64_t k)
{
    if (k >= a.count) return -1;
    if (a.slot_col) {
        const int32_t j = a.slot_col[k];
        return (j >= 0 && a.cv.col_slot[j] == (int32_t)k) ? j : -1;   // skip empty / unpublished
    }
    if (!a.idx) return k;
    const int64_t j = a.idx[k];
    return (uint64_t)j < (uint64_t)a.n ? j : -1;        // entries that name no coordinate are skipped
}

__device__ __forceinline__ float dot4(const float4 x, const float4 y, float acc)
{
    acc = fmaf(x.x, y.x, acc);
    acc = fmaf(x.y, y.y, acc);
    acc = fmaf(x.z, y.z, acc);
    acc = fmaf(x.w, y.w, acc);
    return acc;
}

__device__ __forceinline__ void block_partial(double wsum, double *partials)
{
    __shared__ double sh[4];
    wsum = wave_sum(wsum);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sh[w] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

template <int MODEL, int COLS, bool VEC4, bool NORMS>
__global__ __launch_bounds__(256) void gap_dense_kernel(const GapArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t group = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    int64_t j[COLS];
    const float *p[COLS];
    bool any = false;
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        j[c] = list_entry(a, group * COLS + c);
        any |= j[c] >= 0;
    }
    double wsum = 0.0;
    if (any) {
        int64_t jany = 0;
#pragma unroll
        for (int c = 0; c < COLS; ++c)
            if (j[c] >= 0) jany = j[c];
#pragma unroll
        for (int c = 0; c < COLS; ++c) p[c] = a.cv.col(j[c] >= 0 ? j[c] : jany);

        float acc0[COLS], acc1[COLS], nq[COLS];
#pragma unroll
        for (int c = 0; c < COLS; ++c) acc0[c] = acc1[c] = nq[c] = 0.0f;

        int64_t done = 0;   // rows handled by the vector part
        if (VEC4) {
            const int64_t d4 = a.d >> 2;
            const float4 *vp = reinterpret_cast<const float4 *>(a.v);
            int64_t r = lane;
            for (; r + 64 < d4; r += 128) {
                const float4 v0 = vp[r], v1 = vp[r + 64];
                float4 x0[COLS], x1[COLS];
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    x0[c] = stream_load4(reinterpret_cast<const float4 *>(p[c]) + r);
                    x1[c] = stream_load4(reinterpret_cast<const float4 *>(p[c]) + r + 64);
                }
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    acc0[c] = dot4(x0[c], v0, acc0[c]);
                    acc1[c] = dot4(x1[c], v1, acc1[c]);
                    if (NORMS) nq[c] = dot4(x0[c], x0[c], dot4(x1[c], x1[c], nq[c]));
                }
            }
            if (r < d4) {
                const float4 v0 = vp[r];
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    const float4 x0 = stream_load4(reinterpret_cast<const float4 *>(p[c]) + r);
                    acc0[c] = dot4(x0, v0, acc0[c]);
                    if (NORMS) nq[c] = dot4(x0, x0, nq[c]);
                }
            }
            done = d4 << 2;
        }
        for (int64_t r = done + lane; r < a.d; r += 64) {
            const float vv = a.v[r];
#pragma unroll
            for (int c = 0; c < COLS; ++c) {
                const float x = p[c][r];
                acc0[c] = fmaf(x, vv, acc0[c]);
                if (NORMS) nq[c] = fmaf(x, x, nq[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            const float dotc = wave_sum(acc0[c] + acc1[c]);
            float qc = 0.0f;
            if (NORMS) qc = wave_sum(nq[c]);
            if (lane == c && j[c] >= 0) {
                const float y = (MODEL == DUHL_SVM) ? a.target[j[c]] : 0.0f;
                const float zz = gap_value<MODEL>(a.mc, dotc, a.alpha[j[c]], y);
                a.z[j[c]] = zz;
                if (NORMS) a.q[j[c]] = qc;
                wsum += (double)zz;
            }
        }
    }
    block_partial(wsum, a.partials);
}

template <int MODEL, int G, bool NORMS>
__global__ __launch_bounds__(256) void gap_csr_kernel(const GapArgs a)
{
    constexpr int ROWS = 256 / G;
    constexpr int K = 8;                      // non-zeros per lane fetched at once
    const int sub = threadIdx.x % G;
    const int64_t k = (int64_t)blockIdx.x * ROWS + threadIdx.x / G;
    const int64_t j = list_entry(a, k);
    double wsum = 0.0;
    float acc = 0.0f, nq = 0.0f;
    if (j >= 0) {
        const int64_t beg = a.cv.rowptr[j], end = a.cv.rowptr[j + 1];
        // all index/value loads of a batch are issued before the gathers that depend on them, so
        // a lane has K gathers of v in flight instead of one
        for (int64_t e0 = beg + sub; e0 < end; e0 += (int64_t)G * K) {
            int32_t ci[K];
            float xv[K];
#pragma unroll
            for (int u = 0; u < K; ++u) {
                const int64_t e = e0 + (int64_t)u * G;
                const bool in = e < end;
                ci[u] = in ? a.cv.colidx[e] : 0;
                xv[u] = in ? a.cv.val[e] : 0.0f;
            }
            float vv[K];
#pragma unroll
            for (int u = 0; u < K; ++u) vv[u] = a.v[ci[u]];
#pragma unroll
            for (int u = 0; u < K; ++u) {
                acc = fmaf(xv[u], vv[u], acc);
                if (NORMS) nq = fmaf(xv[u], xv[u], nq);
            }
        }
    }
    acc = group_sum<G>(acc);
    if (NORMS) nq = group_sum<G>(nq);
    if (j >= 0 && sub == 0) {
        const float y = (MODEL == DUHL_SVM) ? a.target[j] : 0.0f;
        const float zz = gap_value<MODEL>(a.mc, acc, a.alpha[j], y);
        a.z[j] = zz;
        if (NORMS) a.q[j] = nq;
        wsum = (double)zz;
    }
    block_partial(wsum, a.partials);
}

// Sum of `count` per-block partials in a fixed order -> scalars[slot].
__global__ __launch_bounds__(1024) void sum_partials_kernel(const double *partials, int64_t count,
                                                            double *out)
{
    __shared__ double sh[16];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 1024) s += partials[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += sh[w];
        *out = t;
    }
}

hipError_t launch_sum_partials(duhl_ctx *c, int64_t count, int scalar_slot)
{
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(1024), 0, c->compute, c->partials, count,
                       c->scalars + scalar_slot);
    return hipGetLastError();
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <int MODEL, bool NORMS>
static hipError_t launch_gap_model(duhl_ctx *c, const GapArgs &a, int64_t *grid_out)
{
    int64_t grid;
    if (c->sparse) {
        const int64_t avg = c->n > 0 ? c->nnz / c->n : 0;
        if (avg > 256) {
            grid = (a.count + 3) / 4;
            hipLaunchKernelGGL((gap_csr_kernel<MODEL, 64, NORMS>), dim3(grid), dim3(256), 0,
                               c->compute, a);
        } else {
            grid = (a.count + 15) / 16;
            hipLaunchKernelGGL((gap_csr_kernel<MODEL, 16, NORMS>), dim3(grid), dim3(256), 0,
                               c->compute, a);
        }
    } else {
        const bool vec = c->a_aligned16 && (a.cv.ld % 4 == 0) && aligned16(a.v) &&
                         (!a.cv.col_slot || (aligned16(a.cv.slots) && a.cv.ld_s % 4 == 0));
        // Short columns: more columns per wavefront to keep enough bytes in flight.
        const int cols = c->gap_cols;
        const int64_t groups = (a.count + cols - 1) / cols;
        grid = (groups + 3) / 4;
#define DUHL_GAP_LAUNCH(COLS, VEC)                                                              \
    hipLaunchKernelGGL((gap_dense_kernel<MODEL, COLS, VEC, NORMS>), dim3(grid), dim3(256), 0, \
                       c->compute, a)
        if (vec) {
            if (cols == 8) DUHL_GAP_LAUNCH(8, true);
            else if (cols == 4) DUHL_GAP_LAUNCH(4, true);
            else if (cols == 2) DUHL_GAP_LAUNCH(2, true);
            else DUHL_GAP_LAUNCH(1, true);
        } else {
            if (cols == 8) DUHL_GAP_LAUNCH(8, false);
            else if (cols == 4) DUHL_GAP_LAUNCH(4, false);
            else if (cols == 2) DUHL_GAP_LAUNCH(2, false);
            else DUHL_GAP_LAUNCH(1, false);
        }
#undef DUHL_GAP_LAUNCH
    }
    *grid_out = grid;
    return hipGetLastError();
}

hipError_t launch_gap(duhl_ctx *c, const int32_t *idx, int64_t count, bool slot_list,
                      bool with_norms)
{
    GapArgs a;
    a.cv = c->cv;
    a.mc = c->mc;
    a.d = c->d;
    a.n = c->n;
    a.count = count;
    a.idx = idx;
    a.slot_col = slot_list ? c->slot_col : nullptr;
    a.v = c->v;
    a.alpha = c->alpha;
    a.target = c->target;
    a.z = c->z;
    a.q = c->q;
    a.partials = c->partials;
    if (count <= 0) {
        return launch_sum_partials(c, 0, S_GAP_SUM);
    }
    int64_t grid = 0;
    hipError_t e;
    // sparse data: from the blocked copy -- the full pass, and lists so long that the dot
    // products of all rows from that copy cost less than those of the listed rows from the CSR
    // arrays (the plain kernel moves about four times the bytes per row)
    int64_t list_min = c->csr_blocked_list_min;
    if (list_min < 0) list_min = c->n / 4 + 1;
    if (c->sparse && c->cb_R > 0 && !slot_list && !with_norms &&
        (idx ? count >= list_min : count == c->n)) {
        e = launch_gap_csr_blocked(c, idx, count, &grid);
        if (e != hipSuccess) return e;
        return launch_sum_partials(c, grid, S_GAP_SUM);
    }
    if (c->model == DUHL_LASSO)
        e = with_norms ? launch_gap_model<DUHL_LASSO, true>(c, a, &grid)
                       : launch_gap_model<DUHL_LASSO, false>(c, a, &grid);
    else if (c->model == DUHL_ELASTIC_NET)
        e = with_norms ? launch_gap_model<DUHL_ELASTIC_NET, true>(c, a, &grid)
                       : launch_gap_model<DUHL_ELASTIC_NET, false>(c, a, &grid);
    else
        e = with_norms ? launch_gap_model<DUHL_SVM, true>(c, a, &grid)
                       : launch_gap_model<DUHL_SVM, false>(c, a, &grid);
    if (e != hipSuccess) return e;
    return launch_sum_partials(c, grid, S_GAP_SUM);
}

}  // namespace duhl
