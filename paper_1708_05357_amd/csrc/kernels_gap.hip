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
};

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
