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
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>

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
    int64_t first;            // idx == nullptr: list entry k stands for coordinate first + k
    const float *stage;       // non-null: the column of list entry k is at stage + k*stage_ld (a batch of
    int64_t stage_ld;         // columns staged from host memory) instead of where cv finds coordinate j
    float *pdot;              // gap_dense_lds_kernel with parts > 1: partial dot products, [part][list entry]
    int parts, cpb;           // the same kernel: parts v is cut into, list entries per workgroup
};

// Which coordinate does list entry k stand for (-1: nothing to do).
__device__ __forceinline__ int64_t list_entry(const GapArgs &a, int64_t k)
{
    if (k >= a.count) return -1;
    if (a.slot_col) {
        const int32_t j = a.slot_col[k];
        return (j >= 0 && a.cv.col_slot[j] == (int32_t)k) ? j : -1;   // skip empty / unpublished
    }
    if (!a.idx) return k + a.first;
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
        int cany = 0;
#pragma unroll
        for (int c = 0; c < COLS; ++c)
            if (j[c] >= 0) { jany = j[c]; cany = c; }
#pragma unroll
        for (int c = 0; c < COLS; ++c)
            p[c] = a.stage ? a.stage + (group * COLS + (j[c] >= 0 ? c : cany)) * a.stage_ld
                           : a.cv.col(j[c] >= 0 ? j[c] : jany);

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

// The same pass for long lists of long, 16-byte aligned columns, with v on chip.  v is cut into
// `parts` ranges of at most 100 KB; a workgroup of 16 wavefronts copies one range into LDS once and
// then streams that range of `cpb` columns, one column per wavefront at a time with eight 16-byte
// loads in flight per lane -- one stream per wavefront instead of COLS interleaved ones, and no
// traffic for v beyond the workgroup's one copy (a plain read-only kernel reaches 7.0 TB/s with
// this access pattern, 6.6 with the pattern above, on the same device).  The wavefront leaves the
// partial dot product in pdot[part][entry]; gap_lds_finish_kernel adds the parts up in a fixed order
// and applies the model's formula.
__global__ __launch_bounds__(1024) void gap_dense_lds_kernel(const GapArgs a)
{
    extern __shared__ float4 vs[];
    constexpr int U = 8;
    const int parts = a.parts;
    const int part = (int)(blockIdx.x % parts);
    const int64_t blk = blockIdx.x / parts;
    const int64_t d4 = a.d >> 2;
    const int64_t p4 = (d4 + parts - 1) / parts;                 // 16-byte chunks per part
    const int64_t r0 = part * p4;
    const int64_t len = r0 + p4 < d4 ? p4 : (d4 > r0 ? d4 - r0 : 0);
    const float4 *vp = reinterpret_cast<const float4 *>(a.v);
    for (int64_t r = threadIdx.x; r < len; r += 1024) vs[r] = vp[r0 + r];
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const bool ragged = part == parts - 1 && (d4 << 2) < a.d;    // d % 4 last rows: the last part's
    for (int c = w; c < a.cpb; c += 16) {
        const int64_t k = blk * a.cpb + c;
        if (k >= a.count) break;
        const int64_t j = list_entry(a, k);                      // (the same in all lanes)
        float dotc = 0.0f;
        if (j >= 0) {
            const float *col = a.cv.col(j);
            const float4 *p = reinterpret_cast<const float4 *>(col) + r0;
            float acc0 = 0.0f, acc1 = 0.0f;
            int64_t r = lane;
            for (; r + 64 * (U - 1) < len; r += 64 * U) {
                float4 x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) x[u] = stream_load4(p + r + 64 * u);
#pragma unroll
                for (int u = 0; u < U; u += 2) {
                    acc0 = dot4(x[u], vs[r + 64 * u], acc0);
                    acc1 = dot4(x[u + 1], vs[r + 64 * (u + 1)], acc1);
                }
            }
            for (; r < len; r += 64) acc0 = dot4(stream_load4(p + r), vs[r], acc0);
            if (ragged)
                for (int64_t e = (d4 << 2) + lane; e < a.d; e += 64) acc1 = fmaf(col[e], a.v[e], acc1);
            dotc = wave_sum(acc0 + acc1);
        }
        if (lane == 0) a.pdot[(int64_t)part * a.count + k] = dotc;
    }
}

template <int MODEL>
__global__ __launch_bounds__(256) void gap_lds_finish_kernel(const GapArgs a)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double zsum = 0.0;
    const int64_t j = list_entry(a, k);
    if (j >= 0) {
        float c = 0.0f;
        for (int p = 0; p < a.parts; ++p) c += a.pdot[(int64_t)p * a.count + k];
        const float y = (MODEL == DUHL_SVM) ? a.target[j] : 0.0f;
        const float zz = gap_value<MODEL>(a.mc, c, a.alpha[j], y);
        a.z[j] = zz;
        zsum = (double)zz;
    }
    block_partial(zsum, a.partials);
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
                                                            double *out, bool accumulate = false)
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
        *out = accumulate ? *out + t : t;
    }
}

hipError_t launch_sum_partials(duhl_ctx *c, int64_t count, int scalar_slot)
{
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(1024), 0, c->compute, c->partials, count,
                       c->scalars + scalar_slot, false);
    return hipGetLastError();
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// What a launch of the gap kernels needs to know beyond GapArgs.
struct GapLaunch {
    bool sparse;
    int64_t avg_nnz;      // sparse: mean non-zeros per row
    bool a_aligned16;     // dense: the matrix (every piece of it) starts on a 16-byte boundary
    int cols;             // dense: columns per wavefront (1, 2, 4 or 8)
    hipStream_t stream;
    float *pdot = nullptr;    // dense: room for parts * count partial dot products (nullptr: the kernel
    int64_t pdot_cap = 0;     // with v on chip is only used where one part holds all of v)
    int num_cu = 256;
    bool lds = false;         // dense: the kernel with v on chip may be used ...
    int64_t lds_min_parts = 2, lds_max_count = 49152;   // ... for columns this long and lists this short
};

constexpr int64_t kLdsPartBytes = 102400;     // most of v that a workgroup of gap_dense_lds_kernel keeps on chip
// Where it pays (defaults of DUHL_GAP_LDS_MIN_PARTS / DUHL_GAP_LDS_MAX_COUNT): columns of at least two parts
// and lists of at most 49,152 entries.  The pass with COLS columns per wavefront has COLS whole columns as
// its unit of work and is at its best on long lists; measured on lists of 5,000 / 10,000 / 20,000 / 40,000
// entries, time with v on chip over time with COLS columns per wavefront: 0.85 / 0.91 / 0.99 / 0.96 for
// columns of 50,000 entries, 0.82 / 0.91 / 1.01 / 0.97 for 100,000, 0.79 / 0.90 / 1.00 / 0.96 for 200,704;
// 60,000 columns of 100,000 entries 1.04, the 500,000 columns of 50,000 entries of the largest workload 1.01.

// Workgroups the launch of the gap kernels has for `count` list entries (= partial sums written).
static int64_t gap_grid(const GapLaunch &L, int64_t count)
{
    if (L.sparse) return L.avg_nnz > 256 ? (count + 3) / 4 : (count + 15) / 16;
    const int64_t groups = (count + L.cols - 1) / L.cols;
    return (groups + 3) / 4;
}

template <int MODEL, bool NORMS>
static hipError_t launch_gap_model(const GapLaunch &L, const GapArgs &a, int64_t *grid_out)
{
    const int64_t grid = gap_grid(L, a.count);
    if (L.sparse) {
        if (L.avg_nnz > 256)
            hipLaunchKernelGGL((gap_csr_kernel<MODEL, 64, NORMS>), dim3(grid), dim3(256), 0, L.stream, a);
        else
            hipLaunchKernelGGL((gap_csr_kernel<MODEL, 16, NORMS>), dim3(grid), dim3(256), 0, L.stream, a);
    } else {
        const bool vec = a.stage ? (aligned16(a.stage) && a.stage_ld % 4 == 0 && aligned16(a.v))
                                 : L.a_aligned16 && (a.cv.ld % 4 == 0) && aligned16(a.v) &&
                                       (!a.cv.col_slot || (aligned16(a.cv.slots) && a.cv.ld_s % 4 == 0));
        // Long lists of long columns: v on chip, one column per wavefront (gap_dense_lds_kernel).
        const int64_t parts = (a.d * 4 + kLdsPartBytes - 1) / kLdsPartBytes;
        if (L.lds && vec && !NORMS && !a.stage && parts >= L.lds_min_parts && a.count <= L.lds_max_count &&
            a.count * parts >= (int64_t)L.num_cu * 16) {
            GapArgs b = a;
            b.parts = (int)parts;
            if (L.pdot && parts * a.count <= L.pdot_cap) {
                // enough workgroups for eight rounds of the device, at most 128 columns each
                int64_t cpb = a.count * b.parts / ((int64_t)L.num_cu * 8);
                cpb = cpb > 128 ? 128 : (cpb < 16 ? 16 : cpb / 16 * 16);
                b.cpb = (int)cpb;
                b.pdot = L.pdot;
                const int64_t blocks = (a.count + cpb - 1) / cpb * b.parts;
                const int64_t p4 = ((a.d >> 2) + b.parts - 1) / b.parts;
                const size_t lds = (size_t)p4 * 16;
                // (more dynamic LDS than the default limit: asked for once per device)
                static bool asked[64] = {};
                int dev = 0;
                hipError_t e = hipGetDevice(&dev);
                if (e == hipSuccess && dev >= 0 && dev < 64 && !asked[dev]) {
                    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gap_dense_lds_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPartBytes);
                    asked[dev] = e == hipSuccess;
                }
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(gap_dense_lds_kernel, dim3(blocks), dim3(1024), lds, L.stream, b);
                const int64_t fgrid = (a.count + 255) / 256;
                hipLaunchKernelGGL((gap_lds_finish_kernel<MODEL>), dim3(fgrid), dim3(256), 0, L.stream, b);
                *grid_out = fgrid;
                return hipGetLastError();
            }
        }
        // Short columns: more columns per wavefront to keep enough bytes in flight.
        const int cols = L.cols;
#define DUHL_GAP_LAUNCH(COLS, VEC)                                                              \
    hipLaunchKernelGGL((gap_dense_kernel<MODEL, COLS, VEC, NORMS>), dim3(grid), dim3(256), 0, \
                       L.stream, a)
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

static hipError_t launch_gap_any(const GapLaunch &L, const GapArgs &a, bool with_norms, int64_t *grid)
{
    if (a.mc.model == DUHL_LASSO)
        return with_norms ? launch_gap_model<DUHL_LASSO, true>(L, a, grid)
                          : launch_gap_model<DUHL_LASSO, false>(L, a, grid);
    if (a.mc.model == DUHL_ELASTIC_NET)
        return with_norms ? launch_gap_model<DUHL_ELASTIC_NET, true>(L, a, grid)
                          : launch_gap_model<DUHL_ELASTIC_NET, false>(L, a, grid);
    return with_norms ? launch_gap_model<DUHL_SVM, true>(L, a, grid)
                      : launch_gap_model<DUHL_SVM, false>(L, a, grid);
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
    a.first = 0;
    a.stage = nullptr;
    a.stage_ld = 0;
    if (count <= 0) {
        return launch_sum_partials(c, 0, S_GAP_SUM);
    }
    // a matrix in pageable host memory: whatever is not asked for by slot crosses the link in batches
    if (c->pageable && !slot_list) return staged_gap(c, idx, 0, count, with_norms);
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
    GapLaunch L;
    L.sparse = c->sparse;
    L.avg_nnz = c->n > 0 ? c->nnz / c->n : 0;
    L.a_aligned16 = c->a_aligned16;
    L.cols = c->gap_cols;
    L.stream = c->compute;
    L.num_cu = c->num_cu;
    L.lds = c->gap_lds != 0 && !c->sparse && !with_norms;
    L.lds_min_parts = c->gap_lds_min_parts;
    L.lds_max_count = c->gap_lds_max_count;
    if (L.lds && c->d * 4 > (L.lds_min_parts - 1) * kLdsPartBytes) {
        // room for the partial dot products of a pass whose v does not fit one workgroup's LDS
        const int64_t parts = (c->d * 4 + kLdsPartBytes - 1) / kLdsPartBytes;
        const int64_t most = c->res == DUHL_RESIDENT_HOST && c->budget > c->n ? c->budget : c->n;
        if (!c->gap_pdot) {
            e = hipMalloc(reinterpret_cast<void **>(&c->gap_pdot), sizeof(float) * (size_t)(parts * most));
            if (e != hipSuccess) return e;
            c->gap_pdot_cap = parts * most;
        }
        L.pdot = c->gap_pdot;
        L.pdot_cap = c->gap_pdot_cap;
    }
    e = launch_gap_any(L, a, with_norms, &grid);
    if (e != hipSuccess) return e;
    return launch_sum_partials(c, grid, S_GAP_SUM);
}

// One batch of a gap pass over columns staged from host memory.
hipError_t launch_gap_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx, int64_t first, bool with_norms,
                            bool first_batch)
{
    GapArgs a{};
    a.cv = c->cv;
    a.mc = c->mc;
    a.d = c->d;
    a.n = c->n;
    a.count = b.count;
    a.idx = idx ? idx + b.k0 : nullptr;
    a.slot_col = nullptr;
    a.v = c->v;
    a.alpha = c->alpha;
    a.target = c->target;
    a.z = c->z;
    a.q = c->q;
    a.partials = c->partials;
    a.first = first + b.k0;
    a.stage = b.stage;
    a.stage_ld = b.lds;
    GapLaunch L;
    L.sparse = false;
    L.avg_nnz = 0;
    L.a_aligned16 = true;
    L.cols = c->gap_cols;
    L.stream = c->compute;
    int64_t grid = 0;
    hipError_t e = launch_gap_any(L, a, with_norms, &grid);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(1024), 0, c->compute, c->partials, grid,
                       c->scalars + S_GAP_SUM, !first_batch);
    return hipGetLastError();
}

// ---- the gap pass for callers that cannot allocate ------------------------------------------------
// The per-workgroup partial sums of duhl_gap_dense_static live in this array instead of a buffer
// from hipMalloc.  Every device the library runs on holds its own copy until the process ends.  The
// name below is only a host-side handle: the device address is asked for once per device
// (static_partials) and that pointer is what the kernels receive.
constexpr int64_t kStaticGroups = DUHL_GAP_STATIC_MAX_GROUPS;
static __device__ __align__(256) double scratch[kStaticGroups];

constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static double *g_static_ptr[kMaxDevices];

// Device address of `scratch` on `device` (which must be current); nullptr and *e set on failure.
static double *static_partials(int device, hipError_t *e)
{
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (!g_static_ptr[device]) {
        double *ptr = nullptr;
        *e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (*e != hipSuccess) return nullptr;
        g_static_ptr[device] = ptr;
    }
    return g_static_ptr[device];
}

}  // namespace duhl

using namespace duhl;

static duhl_status static_fail(char *err, int64_t err_len, duhl_status st, const char *fmt, long long a = 0,
                               long long b = 0)
{
    if (err && err_len > 0) snprintf(err, (size_t)err_len, fmt, a, b);
    return st;
}

extern "C" duhl_status duhl_gap_dense_static(duhl_model model, int64_t d, int64_t n, const float *A,
                                             int64_t ld, const float *v, const float *alpha,
                                             const float *target, double lambda, double eta, double bound,
                                             const int32_t *idx, int64_t count, float *z, double *gap_sum,
                                             int device, void *stream, char *err, int64_t err_len)
{
    if (model != DUHL_LASSO && model != DUHL_SVM && model != DUHL_ELASTIC_NET)
        return static_fail(err, err_len, DUHL_EINVAL, "unknown model");
    if (d <= 0 || n <= 0 || n > 0x7fffffffll || d >= (1ll << 29))
        return static_fail(err, err_len, DUHL_EINVAL, "need 1 <= d < 2^29 and 1 <= n < 2^31");
    if (!A || !v || !alpha || !z) return static_fail(err, err_len, DUHL_EINVAL, "A, v, alpha or z is NULL");
    if (model == DUHL_SVM && !target) return static_fail(err, err_len, DUHL_EINVAL, "the SVM needs its labels");
    if (ld < d) return static_fail(err, err_len, DUHL_EINVAL, "ld (%lld) < d (%lld)", ld, d);
    if (!(lambda > 0.0) || !std::isfinite(lambda))
        return static_fail(err, err_len, DUHL_EINVAL, "lambda must be finite and > 0");
    if (model == DUHL_ELASTIC_NET && (!(eta > 0.0) || !(eta <= 1.0)))
        return static_fail(err, err_len, DUHL_EINVAL, "eta must be in (0, 1]");
    if (model == DUHL_LASSO && (!(bound >= 0.0) || !std::isfinite(bound)))
        return static_fail(err, err_len, DUHL_EINVAL, "the Lasso needs its bound B = ||b||^2/(2 lambda d) >= 0");
    if (idx ? (count < 0 || count > n) : false)
        return static_fail(err, err_len, DUHL_EINVAL, "count (%lld) must be in [0, n = %lld]", count, n);
    if (device < 0 || device >= kMaxDevices) return static_fail(err, err_len, DUHL_EINVAL, "bad device ordinal");
    if (hipSetDevice(device) != hipSuccess) return static_fail(err, err_len, DUHL_EHIP, "hipSetDevice failed");

    const int64_t entries = idx ? count : n;
    int num_cu = 256;
    (void)hipDeviceGetAttribute(&num_cu, hipDeviceAttributeMultiprocessorCount, device);
    GapLaunch L;
    L.sparse = false;
    L.avg_nnz = 0;
    L.a_aligned16 = (reinterpret_cast<uintptr_t>(A) & 15) == 0;
    L.cols = default_gap_cols(d, n, num_cu);
    L.stream = reinterpret_cast<hipStream_t>(stream);
    const int64_t grid = gap_grid(L, entries);
    if (grid > kStaticGroups)
        return static_fail(err, err_len, DUHL_EINVAL,
                           "%lld coordinates need %lld workgroups, more than the static scratch array holds; "
                           "use duhl_gap, or split the list",
                           entries, grid);
    hipError_t e = hipSuccess;
    double *partials = static_partials(device, &e);
    if (!partials) return static_fail(err, err_len, DUHL_EHIP, "hipGetSymbolAddress failed for the scratch array");

    GapArgs a{};
    a.cv.base = A;
    a.cv.ld = ld;
    a.mc = model_constants(model, d, n, lambda, eta, bound);
    a.d = d;
    a.n = n;
    a.count = entries;
    a.idx = idx;
    a.slot_col = nullptr;
    a.v = v;
    a.alpha = alpha;
    a.target = target;
    a.z = z;
    a.q = nullptr;
    a.partials = partials;
    int64_t launched = 0;
    if (entries > 0) {
        e = launch_gap_any(L, a, false, &launched);
        if (e != hipSuccess) return static_fail(err, err_len, DUHL_EHIP, "a kernel launch failed (HIP error %lld)", (long long)e);
    }
    if (gap_sum) {
        hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(1024), 0, L.stream, partials, launched, gap_sum, false);
        e = hipGetLastError();
        if (e != hipSuccess) return static_fail(err, err_len, DUHL_EHIP, "a kernel launch failed (HIP error %lld)", (long long)e);
    }
    return DUHL_OK;
}
