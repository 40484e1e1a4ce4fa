// Gap pass over sparse data (eq. (4), Appendix E) from a copy of the matrix that is blocked by
// ranges of the shared vector and stored in slices of 64 rows.
//
// The plain CSR pass gathers v from the cache hierarchy, four bytes out of every 128-byte line it
// moves; on the paper-shaped sparse workload that, not HBM, sets its speed.  Here the rows of v
// are cut into R ranges of W <= 34,560 entries, each small enough for the LDS of one compute
// unit, and the non-zeros are stored once more, range after range, with 16-bit indices relative
// to the range (6 bytes per non-zero instead of 8).  Inside a range the rows are taken in windows
// of 1,024, sorted by their length in the range, and cut into slices of 64 rows: one row per lane
// of a wavefront.  A slice is stored quad-row after quad-row -- the k-th four entries ("quad") of
// each of its 64 rows side by side -- and is as long as its longest row (the others end in
// zeros; sorting keeps that padding to a few per cent).  A wavefront thus reads a contiguous
// stream with one 8-byte and one 16-byte load per lane and quad-row, every lane adds up its own
// row, and no lane ever talks to another: about twenty instructions per quad, which lets the pass
// run at the speed of the stream (a layout with rows laid end to end needs cross-lane sums and
// per-row bookkeeping, some 85 instructions per quad, and was bound by instruction issue).
// A workgroup loads its range of v into LDS once and then streams its share of the range's
// slices; gathers hit LDS.  Each (range, row) pair yields a partial dot product; a second kernel
// adds the R partials of a row in a fixed order and applies the gap formula.
// The copy is built once per duhl_set_data_csr call; the coordinate-descent kernels keep using
// the caller's CSR arrays (a step needs the whole row at once).
#include "duhl_internal.h"

namespace duhl {

namespace {

constexpr int kRangeMax = 34560;    // floats of v per range: 135 KB of the 160 KB LDS
constexpr int kMaxRanges = 8;
constexpr int kSlice = 64;          // rows per slice: one per lane
constexpr int kWindow = 1024;       // rows that are sorted by length together: 16 slices
constexpr int kSlicesWg = 96;       // most slices per workgroup: 6,144 row sums (24 KB) wait in LDS
constexpr int kDepth = 8;           // quad-rows a wavefront keeps in flight
constexpr int kScanChunk = 2048;
static_assert((int64_t)kSlicesWg * (kRangeMax / 4 + kDepth) * (kSlice * 16) < ((int64_t)1 << 31),
              "32-bit byte offsets into a workgroup's stream");

// ---- building the copy ---------------------------------------------------------------------------

// len[r*n + i] = number of non-zeros of row i whose column lies in range r (rows are sorted).
__global__ void seg_len_kernel(const int64_t *rowptr, const int32_t *colidx, int64_t n, int R, int W,
                               int32_t *len)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t beg = rowptr[i], end = rowptr[i + 1];
    int64_t prev = beg;
    for (int r = 1; r <= R; ++r) {
        int64_t lo = prev, hi = end;                    // first entry with column >= r*W
        if (r < R) {
            const int32_t bound = r * W;
            while (lo < hi) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (colidx[mid] < bound) lo = mid + 1; else hi = mid;
            }
        } else {
            lo = end;
        }
        len[(int64_t)(r - 1) * n + i] = (int32_t)(lo - prev);
        prev = lo;
    }
}

// One workgroup per (range, window): the window's rows in ascending order of their length in
// quads (ties by row number, so the layout is reproducible).  perm[...] = row at each position
// (-1 past the last row), slen[...] = quads of the longest row of each slice.  Rows hold each
// column at most once (checked when the data are set), so a length is at most W / 4 quads.
__global__ __launch_bounds__(kWindow) void sort_window_kernel(const int32_t *len, int64_t n, int64_t nwin,
                                                              int32_t *perm, int32_t *slen)
{
    __shared__ uint32_t key[kWindow];
    const int t = threadIdx.x;
    const int64_t r = blockIdx.x / nwin, w = blockIdx.x % nwin;
    const int32_t *lr = len + r * n;
    const int64_t row = w * kWindow + t;
    const uint32_t quads = row < n ? ((uint32_t)lr[row] + 3u) >> 2 : 0u;
    key[t] = (quads << 10) | (uint32_t)t;
    __syncthreads();
    for (int k = 2; k <= kWindow; k <<= 1) {             // bitonic sort, ascending
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int other = t ^ j;
            if (other > t) {
                const uint32_t x = key[t], y = key[other];
                const bool up = (t & k) == 0;
                if ((x > y) == up) {
                    key[t] = y;
                    key[other] = x;
                }
            }
            __syncthreads();
        }
    }
    const uint32_t mine = key[t];
    const int64_t srow = w * kWindow + (int64_t)(mine & 1023u);
    perm[(r * nwin + w) * kWindow + t] = srow < n ? (int32_t)srow : -1;
    if ((t & (kSlice - 1)) == kSlice - 1)                // ascending: the slice's last row is its longest
        slen[(r * nwin + w) * (kWindow / kSlice) + (t >> 6)] = (int32_t)(mine >> 10);
}

// Exclusive prefix sum of N lengths into N+1 int64 offsets, three launches.
__global__ __launch_bounds__(256) void scan_local_kernel(const int32_t *len, int64_t N, int64_t *out,
                                                         int64_t *csum)
{
    __shared__ int64_t wsum[4];
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * 8;
    int64_t x[8], run = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t t = base + u;
        run += t < N ? (int64_t)len[t] : 0;
        x[u] = run;                                      // inclusive within the thread
    }
    int64_t incl = run;                                  // inclusive scan of thread totals in the wave
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t y = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int64_t before = incl - run;
    for (int u = 0; u < w; ++u) before += wsum[u];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t t = base + u;
        if (t < N) out[t + 1] = before + x[u];           // still without the chunks before this one
    }
    if (threadIdx.x == 255) csum[blockIdx.x] = before + run;
}

__global__ __launch_bounds__(1024) void scan_chunks_kernel(int64_t *csum, int64_t nchunks)
{
    __shared__ int64_t tot[1024];
    const int64_t per = (nchunks + 1023) / 1024;
    const int64_t lo = threadIdx.x * per, hi = lo + per < nchunks ? lo + per : nchunks;
    int64_t s = 0;
    for (int64_t k = lo; k < hi; ++k) s += csum[k];
    tot[threadIdx.x] = s;
    __syncthreads();
    int64_t off = 0;
    for (int t = 0; t < (int)threadIdx.x; ++t) off += tot[t];
    for (int64_t k = lo; k < hi; ++k) {
        const int64_t v = csum[k];
        csum[k] = off;
        off += v;
    }
}

__global__ __launch_bounds__(256) void scan_add_kernel(int64_t *out, int64_t N, const int64_t *csum)
{
    const int64_t off = csum[blockIdx.x];
    const int64_t base = (int64_t)blockIdx.x * kScanChunk;
    for (int u = 0; u < kScanChunk / 256; ++u) {
        const int64_t t = base + u * 256 + threadIdx.x;
        if (t < N) out[t + 1] += off;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[0] = 0;
}

typedef unsigned int duhl_u2 __attribute__((ext_vector_type(2)));
typedef int duhl_i2 __attribute__((ext_vector_type(2)));
typedef int duhl_i4 __attribute__((ext_vector_type(4)));

// One thread per (range, position): the non-zeros of that row in that range, quad by quad, to
// lane (position % 64) of the slice's quad-rows.  The arrays were cleared, which is the padding.
__global__ __launch_bounds__(256) void scatter_sliced_kernel(const int64_t *rowptr, const int32_t *colidx,
                                                             const float *val, int64_t n, int64_t npad, int R,
                                                             int W, const int32_t *len, const int32_t *perm,
                                                             const int64_t *soff, uint16_t *idx16, float *valb)
{
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= (int64_t)R * npad) return;
    const int32_t row = perm[p];
    if (row < 0) return;
    const int r = (int)(p / npad);
    int64_t src = rowptr[row];
    for (int q = 0; q < r; ++q) src += len[(int64_t)q * n + row];
    const int count = len[(int64_t)r * n + row];
    const int64_t at = soff[p >> 6] * kSlice + (p & (kSlice - 1));   // number of the row's first quad
    const int32_t first = r * W;
    for (int k = 0; k < count; k += 4) {
        uint32_t ci[4] = {0u, 0u, 0u, 0u};
        float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int e = 0; e < 4 && k + e < count; ++e) {
            ci[e] = (uint32_t)(colidx[src + k + e] - first);
            x[e] = val[src + k + e];
        }
        const int64_t quad = at + (int64_t)(k >> 2) * kSlice;
        duhl_u2 packed;
        packed.x = ci[0] | (ci[1] << 16);
        packed.y = ci[2] | (ci[3] << 16);
        reinterpret_cast<duhl_u2 *>(idx16)[quad] = packed;
        reinterpret_cast<float4 *>(valb)[quad] = make_float4(x[0], x[1], x[2], x[3]);
    }
}

// ---- the pass -----------------------------------------------------------------------------------

struct SlicedArgs {
    const int64_t *soff;     // R*nslices + 1 slice starts, in quad-rows, ordered (range, slice)
    const int32_t *perm;     // R*npad rows by position, -1: none
    const uint16_t *idx16;
    const float *valb;
    const float *v;
    float *partial;          // R*n partial dot products, ordered (range, row)
    int64_t n, d, npad, nslices;
    int R, W;
    int per_wg;              // slices per workgroup, <= kSlicesWg
};

// The workgroup (r, b) takes slices [b*per_wg, (b+1)*per_wg) of range r.  Their quad-rows are one
// contiguous stream, which its 16 wavefronts share evenly -- cutting slices where the shares end,
// so a row's sum may come from two wavefronts (more, if a slice is longer than a share) and is
// put together in LDS.  Nothing is stored to device memory before the stream is through: a store
// between the loads would make every wait for one load a wait for all (loads and stores retire
// through one counter, in order only among their own kind).
__global__ __launch_bounds__(1024) void csr_sliced_dot_kernel(const SlicedArgs a)
{
    __shared__ float vs[kRangeMax];
    __shared__ float res[kSlicesWg * kSlice];
    __shared__ int32_t qoff[kSlicesWg + 1];              // slice starts, relative to the workgroup's first
    const int R = a.R;
    const int r = blockIdx.x % R;
    const int64_t b = blockIdx.x / R;
    const int64_t s0 = b * a.per_wg;
    const int ns = (int)(s0 + a.per_wg <= a.nslices ? a.per_wg : a.nslices - s0);
    const int64_t *so = a.soff + (int64_t)r * a.nslices + s0;
    const int64_t Q0 = so[0];
    // The wavefront's share of the stream, and its first quad-rows requested before anything
    // else: they are on their way while v is loaded.  Loads past the share return zeros (the
    // descriptors end there), so the loop below can run in whole rounds of kDepth; a workgroup's
    // stream is at most kSlicesWg slices of kRangeMax / 4 quad-rows, so byte offsets fit 32 bits.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int total = (int)(so[ns] - Q0);
    const int share = (total + 15) / 16;
    const int qb = wave * share < total ? wave * share : total;
    const int qe = qb + share < total ? qb + share : total;
    const __amdgpu_buffer_rsrc_t rs_i = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.idx16) + Q0 * (kSlice * 4), 0, qe * (kSlice * 8), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.valb) + Q0 * (kSlice * 4), 0, qe * (kSlice * 16), 0x00020000);
    const int off_i = lane * 8, off_x = lane * 16;
    duhl_i2 ci[kDepth];
    duhl_i4 xv[kDepth];
#pragma unroll
    for (int i = 0; i < kDepth; ++i) {
        ci[i] = __builtin_amdgcn_raw_buffer_load_b64(rs_i, off_i, (qb + i) * (kSlice * 8), 2);
        xv[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, off_x, (qb + i) * (kSlice * 16), 2);
        // issued in the order the loop uses and re-issues them: the wait for a quad-row then
        // leaves the younger ones in flight on the first round as on all later ones
        __builtin_amdgcn_sched_barrier(0);
    }
    // this range of v into LDS: all of a thread's 16-byte loads are issued before the first
    // store (W is a multiple of 4 and v is allocated with four spare entries, so whole float4s
    // can be read at the end of the vector)
    {
        const int64_t v0 = (int64_t)r * a.W;
        const int vlen = (int)(a.d - v0 < a.W ? a.d - v0 : a.W);
        const int n4 = (vlen + 3) >> 2;
        const float4 *src = reinterpret_cast<const float4 *>(a.v + v0);
        constexpr int kFill = (kRangeMax / 4 + 1023) / 1024;
        float4 tmp[kFill];
#pragma unroll
        for (int i = 0; i < kFill; ++i) {
            const int t = threadIdx.x + i * 1024;
            tmp[i] = src[t < n4 ? t : 0];
        }
#pragma unroll
        for (int i = 0; i < kFill; ++i) {
            const int t = threadIdx.x + i * 1024;
            if (t < n4) reinterpret_cast<float4 *>(vs)[t] = tmp[i];
        }
    }
    for (int t = threadIdx.x; t <= ns; t += 1024) qoff[t] = (int32_t)(so[t] - Q0);
    for (int t = threadIdx.x; t < ns * kSlice; t += 1024) res[t] = 0.0f;
    __syncthreads();

    if (qb < qe) {
        // the slice that holds quad-row qb: the last one that starts at or before it
        int lo = 0, hi = ns - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (__builtin_amdgcn_readfirstlane(qoff[mid]) <= qb) lo = mid; else hi = mid - 1;
        }
        int s = lo;
        int send = __builtin_amdgcn_readfirstlane(qoff[s + 1]);
        float acc = 0.0f;
        int q = qb;
        while (q < qe) {
#pragma unroll
            for (int i = 0; i < kDepth; ++i) {
                const uint32_t c0 = (uint32_t)ci[i].x, c1 = (uint32_t)ci[i].y;
                acc = fmaf(__int_as_float(xv[i].x), vs[c0 & 0xffffu], acc);
                acc = fmaf(__int_as_float(xv[i].y), vs[c0 >> 16], acc);
                acc = fmaf(__int_as_float(xv[i].z), vs[c1 & 0xffffu], acc);
                acc = fmaf(__int_as_float(xv[i].w), vs[c1 >> 16], acc);
                ci[i] = __builtin_amdgcn_raw_buffer_load_b64(rs_i, off_i, (q + kDepth) * (kSlice * 8), 2);
                xv[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, off_x, (q + kDepth) * (kSlice * 16), 2);
                ++q;
                if (q == send) {                         // the slice is through (same in all lanes)
                    if (s < ns) atomicAdd(&res[s * kSlice + lane], acc);
                    acc = 0.0f;
                    do {                                 // on to the next slice that is not empty
                        ++s;
                        send = s < ns ? __builtin_amdgcn_readfirstlane(qoff[s + 1]) : 0x7fffffff;
                    } while (send == q);
                }
            }
        }
        if (s < ns) atomicAdd(&res[s * kSlice + lane], acc);   // what the share held of its last slice
    }
    __syncthreads();
    const int32_t *pm = a.perm + (int64_t)r * a.npad + s0 * kSlice;
    float *out = a.partial + (int64_t)r * a.n;
    for (int t = threadIdx.x; t < ns * kSlice; t += 1024) {
        const int32_t row = pm[t];
        if (row >= 0) out[row] = res[t];
    }
}

struct FinishArgs {
    ModelConst mc;
    const float *partial, *alpha, *target;
    const int32_t *idx;      // the coordinates whose gaps are wanted, or nullptr for all n
    float *z;
    double *partials;
    int64_t n, count;
    int R;
};

template <int MODEL>
__global__ __launch_bounds__(256) void csr_blocked_finish_kernel(const FinishArgs a)
{
    __shared__ double sh[4];
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double wsum = 0.0;
    const int64_t i = k < a.count ? (a.idx ? (int64_t)a.idx[k] : k) : -1;
    if ((uint64_t)i < (uint64_t)a.n) {
        float c = 0.0f;
        for (int r = 0; r < a.R; ++r) c += a.partial[(int64_t)r * a.n + i];
        const float y = (MODEL == DUHL_SVM) ? a.target[i] : 0.0f;
        const float zz = gap_value<MODEL>(a.mc, c, a.alpha[i], y);
        a.z[i] = zz;
        wsum = (double)zz;
    }
    wsum = wave_sum(wsum);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) a.partials[blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

}  // namespace

void csr_blocked_free(duhl_ctx *c)
{
    (void)hipFree(c->cb_soff); c->cb_soff = nullptr;
    (void)hipFree(c->cb_perm); c->cb_perm = nullptr;
    (void)hipFree(c->cb_idx); c->cb_idx = nullptr;
    (void)hipFree(c->cb_val); c->cb_val = nullptr;
    (void)hipFree(c->cb_partial); c->cb_partial = nullptr;
    c->cb_R = 0;
}

// Build the blocked copy of the current CSR data.  Leaves c->cb_R == 0 (and the plain pass in
// charge) when the copy does not apply: too many ranges, rows of such uneven length that the
// slices would be mostly padding, no memory for it, or switched off.
hipError_t csr_blocked_build(duhl_ctx *c)
{
    csr_blocked_free(c);
    if (!c->sparse || !c->csr_blocked || c->nnz <= 0) return hipSuccess;
    const int64_t d = c->d, n = c->n;
    const int R = (int)((d + kRangeMax - 1) / kRangeMax);
    if (R > kMaxRanges) return hipSuccess;
    const int W = (int)(((d + R - 1) / R + 3) / 4 * 4);     // multiple of 4: ranges start 16-byte aligned
    const int64_t nwin = (n + kWindow - 1) / kWindow;
    const int64_t npad = nwin * kWindow, nslices = npad / kSlice;
    const int64_t N = (int64_t)R * nslices;              // slices in all
    int32_t *len = nullptr, *slen = nullptr;
    int64_t *csum = nullptr;
    const int64_t nchunks = (N + kScanChunk - 1) / kScanChunk;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&len), (size_t)R * n * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&slen), (size_t)N * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&csum), (size_t)nchunks * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_soff), (size_t)(N + 1) * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_perm), (size_t)R * npad * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_partial), (size_t)R * n * sizeof(float));
    int64_t quadrows = 0;                                // length of the copy, padding included
    if (e == hipSuccess) {
        hipLaunchKernelGGL(seg_len_kernel, dim3((n + 255) / 256), dim3(256), 0, c->compute, c->cv.rowptr,
                           c->cv.colidx, n, R, W, len);
        hipLaunchKernelGGL(sort_window_kernel, dim3((unsigned)(R * nwin)), dim3(kWindow), 0, c->compute, len, n,
                           nwin, c->cb_perm, slen);
        hipLaunchKernelGGL(scan_local_kernel, dim3(nchunks), dim3(256), 0, c->compute, slen, N, c->cb_soff, csum);
        hipLaunchKernelGGL(scan_chunks_kernel, dim3(1), dim3(1024), 0, c->compute, csum, nchunks);
        hipLaunchKernelGGL(scan_add_kernel, dim3(nchunks), dim3(256), 0, c->compute, c->cb_soff, N, csum);
        e = hipGetLastError();
        if (e == hipSuccess)
            e = hipMemcpyAsync(&quadrows, c->cb_soff + N, sizeof(int64_t), hipMemcpyDeviceToHost, c->compute);
        if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    }
    // Rows of very uneven length: a slice is as long as its longest row, and when that leaves the
    // copy more than half padding the plain pass reads less.
    const int64_t entries = quadrows * (kSlice * 4);
    const bool fits = e == hipSuccess && entries <= 2 * c->nnz + 8 * (int64_t)kSlice * N;
    if (fits) {
        const size_t alloc = (size_t)entries + 4;
        e = hipMalloc(reinterpret_cast<void **>(&c->cb_idx), alloc * sizeof(uint16_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_val), alloc * sizeof(float));
        if (e == hipSuccess) e = hipMemsetAsync(c->cb_idx, 0, alloc * sizeof(uint16_t), c->compute);
        if (e == hipSuccess) e = hipMemsetAsync(c->cb_val, 0, alloc * sizeof(float), c->compute);   // padding = 0
        if (e == hipSuccess) {
            const int64_t threads = (int64_t)R * npad;
            hipLaunchKernelGGL(scatter_sliced_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                               c->compute, c->cv.rowptr, c->cv.colidx, c->cv.val, n, npad, R, W, len,
                               c->cb_perm, c->cb_soff, c->cb_idx, c->cb_val);
            e = hipGetLastError();
            if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
        }
    }
    (void)hipFree(len);
    (void)hipFree(slen);
    (void)hipFree(csum);
    if (e != hipSuccess || !fits) {
        csr_blocked_free(c);
        if (e == hipErrorOutOfMemory) {                  // no room for the copy: the plain pass stays
            (void)hipGetLastError();
            return hipSuccess;
        }
        return e;
    }
    c->cb_R = R;
    c->cb_W = W;
    c->cb_slices = nslices;
    return hipSuccess;
}

// Gaps of all n coordinates (idx == nullptr) or of the listed ones from the blocked copy: the
// dot products of all rows, then the gap formula for those that were asked for.
// *grid_out = number of per-block partial sums.
hipError_t launch_gap_csr_blocked(duhl_ctx *c, const int32_t *idx, int64_t count, int64_t *grid_out)
{
    SlicedArgs a;
    a.soff = c->cb_soff;
    a.perm = c->cb_perm;
    a.idx16 = c->cb_idx;
    a.valb = c->cb_val;
    a.v = c->v;
    a.partial = c->cb_partial;
    a.n = c->n;
    a.d = c->d;
    a.nslices = c->cb_slices;
    a.npad = c->cb_slices * kSlice;
    a.R = c->cb_R;
    a.W = c->cb_W;
    // one workgroup per compute unit at a time (its LDS holds a range of v); a few rounds of them
    // so that the tail is short, and more when a workgroup could not hold its rows' sums
    int64_t groups = (int64_t)c->num_cu * c->csr_blocked_waves / a.R;
    if (groups < 1) groups = 1;
    int64_t per_wg = (a.nslices + groups - 1) / groups;
    if (per_wg > kSlicesWg) per_wg = kSlicesWg;
    if (per_wg < 1) per_wg = 1;
    groups = (a.nslices + per_wg - 1) / per_wg;
    a.per_wg = (int)per_wg;
    hipLaunchKernelGGL(csr_sliced_dot_kernel, dim3((unsigned)(groups * a.R)), dim3(1024), 0, c->compute, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    FinishArgs f;
    f.mc = c->mc;
    f.partial = c->cb_partial;
    f.alpha = c->alpha;
    f.target = c->target;
    f.idx = idx;
    f.z = c->z;
    f.partials = c->partials;
    f.n = c->n;
    f.count = idx ? count : c->n;
    f.R = c->cb_R;
    const int64_t fgrid = (f.count + 255) / 256;
    if (c->model == DUHL_LASSO)
        hipLaunchKernelGGL(csr_blocked_finish_kernel<DUHL_LASSO>, dim3(fgrid), dim3(256), 0, c->compute, f);
    else if (c->model == DUHL_ELASTIC_NET)
        hipLaunchKernelGGL(csr_blocked_finish_kernel<DUHL_ELASTIC_NET>, dim3(fgrid), dim3(256), 0, c->compute, f);
    else
        hipLaunchKernelGGL(csr_blocked_finish_kernel<DUHL_SVM>, dim3(fgrid), dim3(256), 0, c->compute, f);
    *grid_out = fgrid;
    return hipGetLastError();
}

}  // namespace duhl
