// Full gap pass over sparse data (eq. (4), Appendix E) from a copy of the matrix that is blocked
// by ranges of the shared vector.
//
// The plain CSR pass gathers v from the cache hierarchy, four bytes out of every 128-byte line it
// moves; on the paper-shaped sparse workload that, not HBM, sets its speed.  Here the rows of v
// are cut into R ranges of W <= 36,864 entries, each small enough for the LDS of one compute
// unit, and the non-zeros are stored once more, range after range and row after row inside a
// range, with 16-bit indices relative to the range (6 bytes per non-zero instead of 8) and each
// (range, row) segment padded with zeros to a multiple of four entries, so that a lane fetches
// four entries with one 8-byte and one 16-byte load and all four belong to the same row.  A
// workgroup loads its range of v into LDS once and then streams the non-zeros of that range with
// fully coalesced loads; gathers hit LDS.  Each (range, row) pair yields a partial dot product; a
// second kernel adds the R partials of a row in a fixed order and applies the gap formula.
// The copy is built once per duhl_set_data_csr call; the coordinate-descent kernels keep using
// the caller's CSR arrays (a step needs the whole row at once).
#include "duhl_internal.h"

namespace duhl {

namespace {

constexpr int kRangeMax = 36864;   // floats of v per range: 144 KB of the 160 KB LDS
constexpr int kMaxRanges = 8;
constexpr int kScanChunk = 2048;

// ---- building the blocked copy ---------------------------------------------------------------

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

// Exclusive prefix sum of the N padded segment lengths into N+1 int64 offsets, three launches.
__global__ __launch_bounds__(256) void scan_local_kernel(const int32_t *len, int64_t N, int64_t *out,
                                                         int64_t *csum)
{
    __shared__ int64_t wsum[4];
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * 8;
    int64_t x[8], run = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t t = base + u;
        run += t < N ? (int64_t)((len[t] + 3) & ~3) : 0;   // segments are padded to whole quads
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

// Copy row i's non-zeros to their places: 16 lanes per row.
__global__ __launch_bounds__(256) void scatter_blocked_kernel(const int64_t *rowptr, const int32_t *colidx,
                                                              const float *val, int64_t n, int R, int W,
                                                              const int32_t *len, const int64_t *bptr,
                                                              uint16_t *idx16, float *valb)
{
    const int sub = threadIdx.x & 15;
    const int64_t i = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    if (i >= n) return;
    const int64_t beg = rowptr[i], end = rowptr[i + 1];
    int64_t src[kMaxRanges + 1], dst[kMaxRanges];        // where range r of this row starts
    src[0] = beg;
    for (int r = 0; r < R; ++r) {
        dst[r] = bptr[(int64_t)r * n + i];
        src[r + 1] = src[r] + len[(int64_t)r * n + i];
    }
    for (int64_t e = beg + sub; e < end; e += 16) {
        const int32_t c = colidx[e];
        int r = 0;
        for (int q = 1; q < R; ++q) r += e >= src[q];
        const int64_t to = dst[r] + (e - src[r]);
        idx16[to] = (uint16_t)(c - r * W);
        valb[to] = val[e];
    }
}

// ---- the pass -----------------------------------------------------------------------------------

struct BlockedArgs {
    const int64_t *bptr;     // R*n + 1 offsets into idx16 / valb, ordered (range, row)
    const uint16_t *idx16;
    const float *valb;
    const float *v;
    float *partial;          // R*count partial dot products, ordered (range, list position)
    const int32_t *idx;      // the rows to evaluate (then one row per span), or nullptr for all n
    int64_t n, d, count;     // count = n without a list
    int R, W;
};

typedef unsigned int duhl_u2 __attribute__((ext_vector_type(2)));

// What a group holds of one span: where it starts, the row starts inside it (in quads, rb[U] = its
// length) and the first batch of its entries.
template <int U, int K>
struct SpanBuf {
    const uint16_t *pi;
    const float *px;
    int rb[U + 1];
    duhl_u2 ci[K];
    float4 xv[K];
};

// One batch of a span: K quads per lane at quad positions q0 + k*G, clamped into the span so that
// the loads need no predicate (quads read twice are masked out when they are added).  last >= 0.
template <int G, int K>
__device__ __forceinline__ void load_batch(const uint16_t *pi, const float *px, int q0, int last,
                                           duhl_u2 (&ci)[K], float4 (&xv)[K])
{
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int q = q0 + k * G;
        const int qc = q < last ? q : last;
        ci[k] = __builtin_nontemporal_load(reinterpret_cast<const duhl_u2 *>(pi) + qc);
        xv[k] = stream_load4(reinterpret_cast<const float4 *>(px) + qc);
    }
}

// acc[u] += the products of the batch's quads that belong to row u of the span.  A quad never
// straddles two rows (segments are padded), and padding entries are zeros.
template <int G, int U, int K>
__device__ __forceinline__ void add_batch(const float *vs, int q0, const int (&rb)[U + 1],
                                          const duhl_u2 (&ci)[K], const float4 (&xv)[K], float (&acc)[U])
{
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int q = q0 + k * G;
        float p = xv[k].x * vs[ci[k].x & 0xffffu];
        p = fmaf(xv[k].y, vs[ci[k].x >> 16], p);
        p = fmaf(xv[k].z, vs[ci[k].y & 0xffffu], p);
        p = fmaf(xv[k].w, vs[ci[k].y >> 16], p);
        if (U == 1) {
            acc[0] += q < rb[1] ? p : 0.0f;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] += (q >= rb[u] && q < rb[u + 1]) ? p : 0.0f;
        }
    }
}

// Sum over the G lanes of a group; every lane gets it.
template <int G>
__device__ __forceinline__ float span_group_sum(float x)
{
    if (G == 2 || G == 4 || G == 8) {
        x = dpp_add<0xB1>(x);                   // quad_perm [1,0,3,2]: lane ^ 1
        if (G >= 4) x = dpp_add<0x4E>(x);       // quad_perm [2,3,0,1]: lane ^ 2
        if (G == 8) x = dpp_add<0x141>(x);      // row_half_mirror: the other quad of the 8
        return x;
    }
    if (G == 16) {
        x = dpp_add<0x128>(x);                  // row_ror:8, 4, 2, 1
        x = dpp_add<0x124>(x);
        x = dpp_add<0x122>(x);
        x = dpp_add<0x121>(x);
        return x;
    }
    return group_sum<G>(x);
}

// The values that lanes 0 and 1 of the group hold, in every lane of the group.
template <int G>
__device__ __forceinline__ void group_first_two(int64_t x, int sub, int64_t &x0, int64_t &x1)
{
    if (G == 2) {
        x0 = dpp_mov64<0xA0>(x);                // quad_perm [0,0,2,2]
        x1 = dpp_mov64<0xF5>(x);                // quad_perm [1,1,3,3]
    } else if (G == 4 || G == 8) {
        x0 = dpp_mov64<0x00>(x);                // quad_perm [0,0,0,0]
        x1 = dpp_mov64<0x55>(x);                // quad_perm [1,1,1,1]
        if (G == 8) {                           // second quad: from the first, mirrored
            const int64_t m0 = dpp_mov64<0x141>(x0), m1 = dpp_mov64<0x141>(x1);
            if (sub >= 4) { x0 = m0; x1 = m1; }
        }
    } else {
        x0 = __shfl(x, 0, G);
        x1 = __shfl(x, 1, G);
    }
}

// A group of G lanes takes U consecutive rows of one range at a time: their entries are one
// contiguous span, streamed K quads per lane at a time (4*G*K is chosen to hold a typical span;
// longer ones take further batches); which of the U rows a quad belongs to is decided by
// comparing its position with the rows' boundaries.  The loop is software-pipelined by hand over a
// ring of NB buffers that change roles: while a span is being multiplied, the entries of the
// group's next NB-1 spans and the boundaries of the one after those are in flight.
template <int G, int U, int K, int NB>
__global__ __launch_bounds__(1024) void csr_blocked_dot_kernel(const BlockedArgs a)
{
    static_assert(U + 1 <= G, "a group loads its U+1 row boundaries with one lane each");
    __shared__ float vs[kRangeMax];
    const int R = a.R;
    const int r = blockIdx.x % R;
    const int64_t b = blockIdx.x / R, nb = gridDim.x / R;
    // this range of v into LDS: all of a thread's 16-byte loads are issued before the first
    // store (W is a multiple of 4 and v is allocated with four spare entries, so whole float4s
    // can be read at the end of the vector)
    {
        const int64_t v0 = (int64_t)r * a.W;
        const int vlen = (int)(a.d - v0 < a.W ? a.d - v0 : a.W);
        const int n4 = (vlen + 3) >> 2;
        const float4 *src = reinterpret_cast<const float4 *>(a.v + v0);
        constexpr int kFill = kRangeMax / 4 / 1024;
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
    __syncthreads();

    const int sub = threadIdx.x % G;
    const int64_t group = threadIdx.x / G;
    constexpr int64_t kGroups = 1024 / G;
    const int64_t *rp = a.bptr + (int64_t)r * a.n;       // boundaries of this range's rows
    float *out = a.partial + (int64_t)r * a.count;
    // a workgroup streams its own contiguous share of the range's spans
    const int64_t all_spans = (a.count + U - 1) / U;
    const int64_t share = ((all_spans + nb - 1) / nb + kGroups - 1) / kGroups * kGroups;
    const int64_t first = b * share;
    const int64_t nspans = first + share < all_spans ? first + share : all_spans;
    constexpr int64_t stride = kGroups;
    // lane `sub` (<= U) fetches the boundary of row s*U + sub; rows past n are empty, and so are
    // the spans past the last one (all boundaries 0: an empty span at the start of the arrays)
    auto boundary = [&](int64_t s) -> int64_t {
        if (sub > U || s >= nspans) return 0;
        if (U == 1 && a.idx) {                           // a listed row; entries that name none: empty
            const int64_t j = a.idx[s];
            return (uint64_t)j < (uint64_t)a.n ? rp[j + sub] : 0;
        }
        const int64_t row = s * U + sub;
        return rp[row < a.n ? row : a.n];
    };
    // start a span: descriptor from its boundaries, first batch of entries on its way
    auto begin = [&](int64_t bnd, SpanBuf<U, K> &sb) {
        int64_t base;
        if (U == 1) {
            int64_t end;
            group_first_two<G>(bnd, sub, base, end);
            sb.rb[0] = 0;
            sb.rb[U] = (int)((end - base) >> 2);
        } else {
            base = __shfl(bnd, 0, G);
#pragma unroll
            for (int u = 0; u <= U; ++u) sb.rb[u] = (int)((__shfl(bnd, u, G) - base) >> 2);
        }
        sb.pi = a.idx16 + base;
        sb.px = a.valb + base;
        load_batch<G, K>(sb.pi, sb.px, sub, sb.rb[U] > 0 ? sb.rb[U] - 1 : 0, sb.ci, sb.xv);
    };
    // finish a span whose first batch has been requested by begin()
    auto finish = [&](int64_t span, const SpanBuf<U, K> &sb) {
        float acc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = 0.0f;
        add_batch<G, U, K>(vs, sub, sb.rb, sb.ci, sb.xv, acc);
        for (int q0 = sub + G * K; q0 < sb.rb[U]; q0 += G * K) {   // a span longer than 4*G*K entries
            duhl_u2 cj[K];
            float4 xj[K];
            load_batch<G, K>(sb.pi, sb.px, q0, sb.rb[U] - 1, cj, xj);
            add_batch<G, U, K>(vs, q0, sb.rb, cj, xj, acc);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float s = span_group_sum<G>(acc[u]);
            const int64_t row = span * U + u;
            if (sub == u && row < a.count) out[row] = s;
        }
    };

    int64_t span = first + group;
    SpanBuf<U, K> buf[NB];
#pragma unroll
    for (int i = 0; i < NB - 1; ++i) begin(boundary(span + i * stride), buf[i]);
    int64_t bnd = boundary(span + (NB - 1) * stride);    // boundaries of the next span to begin
    while (span < nspans) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (span < nspans) {
                const int64_t bnd_new = boundary(span + NB * stride);
                begin(bnd, buf[(i + NB - 1) % NB]);
                finish(span, buf[i]);
                bnd = bnd_new;
                span += stride;
            }
        }
    }
}

struct FinishArgs {
    ModelConst mc;
    const float *partial, *alpha, *target;
    const int32_t *idx;
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
        for (int r = 0; r < a.R; ++r) c += a.partial[(int64_t)r * a.count + k];
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
    (void)hipFree(c->cb_ptr); c->cb_ptr = nullptr;
    (void)hipFree(c->cb_idx); c->cb_idx = nullptr;
    (void)hipFree(c->cb_val); c->cb_val = nullptr;
    (void)hipFree(c->cb_partial); c->cb_partial = nullptr;
    c->cb_R = 0;
}

// Build the blocked copy of the current CSR data.  Leaves c->cb_R == 0 (and the plain pass in
// charge) when the copy does not apply: too many ranges, or switched off.
hipError_t csr_blocked_build(duhl_ctx *c)
{
    csr_blocked_free(c);
    if (!c->sparse || !c->csr_blocked || c->nnz <= 0) return hipSuccess;
    const int64_t d = c->d, n = c->n;
    const int R = (int)((d + kRangeMax - 1) / kRangeMax);
    if (R > kMaxRanges) return hipSuccess;
    const int W = (int)(((d + R - 1) / R + 3) / 4 * 4);     // multiple of 4: ranges start 16-byte aligned
    const int64_t N = (int64_t)R * n;
    int32_t *len = nullptr;
    int64_t *csum = nullptr;
    const int64_t nchunks = (N + kScanChunk - 1) / kScanChunk;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&len), (size_t)N * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&csum), (size_t)nchunks * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_ptr), (size_t)(N + 1) * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_partial), (size_t)N * sizeof(float));
    int64_t padded = 0;                                  // entries of the copy, padding included
    if (e == hipSuccess) {
        hipLaunchKernelGGL(seg_len_kernel, dim3((n + 255) / 256), dim3(256), 0, c->compute, c->cv.rowptr,
                           c->cv.colidx, n, R, W, len);
        hipLaunchKernelGGL(scan_local_kernel, dim3(nchunks), dim3(256), 0, c->compute, len, N, c->cb_ptr, csum);
        hipLaunchKernelGGL(scan_chunks_kernel, dim3(1), dim3(1024), 0, c->compute, csum, nchunks);
        hipLaunchKernelGGL(scan_add_kernel, dim3(nchunks), dim3(256), 0, c->compute, c->cb_ptr, N, csum);
        e = hipGetLastError();
        if (e == hipSuccess)
            e = hipMemcpyAsync(&padded, c->cb_ptr + N, sizeof(int64_t), hipMemcpyDeviceToHost, c->compute);
        if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    }
    // + 4: the kernel may read one quad at the position where an empty last span begins
    const size_t entries = (size_t)padded + 4;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_idx), entries * sizeof(uint16_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->cb_val), entries * sizeof(float));
    if (e == hipSuccess) e = hipMemsetAsync(c->cb_idx, 0, entries * sizeof(uint16_t), c->compute);
    if (e == hipSuccess) e = hipMemsetAsync(c->cb_val, 0, entries * sizeof(float), c->compute);   // padding = 0
    if (e == hipSuccess) {
        hipLaunchKernelGGL(scatter_blocked_kernel, dim3((n + 15) / 16), dim3(256), 0, c->compute, c->cv.rowptr,
                           c->cv.colidx, c->cv.val, n, R, W, len, c->cb_ptr, c->cb_idx, c->cb_val);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    }
    (void)hipFree(len);
    (void)hipFree(csum);
    if (e != hipSuccess) {
        csr_blocked_free(c);
        if (e == hipErrorOutOfMemory) {                  // no room for the copy: the plain pass stays
            (void)hipGetLastError();
            return hipSuccess;
        }
        return e;
    }
    c->cb_R = R;
    c->cb_W = W;
    return hipSuccess;
}

// Gaps of all n coordinates (idx == nullptr) or of the listed ones from the blocked copy;
// *grid_out = number of per-block partial sums.
hipError_t launch_gap_csr_blocked(duhl_ctx *c, const int32_t *idx, int64_t count, int64_t *grid_out)
{
    BlockedArgs a;
    a.bptr = c->cb_ptr;
    a.idx16 = c->cb_idx;
    a.valb = c->cb_val;
    a.v = c->v;
    a.partial = c->cb_partial;
    a.n = c->n;
    a.d = c->d;
    a.idx = idx;
    a.count = idx ? count : c->n;
    a.R = c->cb_R;
    a.W = c->cb_W;
    // one workgroup per compute unit at a time (its LDS holds a range of v); a few rounds of
    // them so that the tail is short
    int64_t per_range = (int64_t)c->num_cu * c->csr_blocked_waves / a.R;   // no partly filled last round
    // Shape of a group's work by the mean length of a (range, row) segment in quads: groups of 16
    // lanes (64 for long rows) with 2 or 4 quads per lane, and enough rows per span to fill them.
    const double quads = ((double)c->nnz / ((double)a.R * (double)c->n) + 1.5) / 4.0 + 0.5;
    const int shape = c->csr_blocked_shape;              // 100000*G + 1000*U + 10*K + NB, 0 = choose
    int G = 16, U = 1, K = 2, NB = 3;
    if (shape > 0) {
        G = shape / 100000;
        U = (shape / 1000) % 100;
        K = (shape / 10) % 100;
        NB = shape % 10;
    } else if (idx && quads <= 12.0) {                   // a list: one row per span, so fewer lanes
        G = 4; U = 1; K = 3;
    } else if (!idx && quads <= 4.5) {
        U = 6; NB = 2;
    } else if (!idx && quads <= 9.5) {
        U = 3;
    } else if (quads <= 28.0) {
        U = 1;
    } else if (quads <= 56.0) {
        U = 1; K = 4;
    } else if (quads <= 112.0) {
        G = 64; U = 1; K = 2;
    } else {
        G = 64; U = 1; K = 4; NB = 2;
    }
    if (idx && U != 1) { G = 16; U = 1; K = 2; NB = 3; }   // (a forced shape that does not fit a list)
    const int64_t spans = (a.count + U - 1) / U;
    const int64_t max_useful = (spans + (1024 / G) - 1) / (1024 / G);
    if (per_range > max_useful) per_range = max_useful;
    if (per_range < 1) per_range = 1;
    const dim3 grid((unsigned)(per_range * a.R));
#define DUHL_CB(GG, UU, KK, NN)                                                                  \
    if (G == GG && U == UU && K == KK && NB == NN) {                                             \
        hipLaunchKernelGGL((csr_blocked_dot_kernel<GG, UU, KK, NN>), grid, dim3(1024), 0, c->compute, a); \
        launched = true;                                                                         \
    }
    bool launched = false;
    DUHL_CB(4, 1, 3, 3)
    DUHL_CB(8, 1, 2, 3)
    DUHL_CB(16, 1, 2, 3)
    DUHL_CB(16, 1, 4, 3)
    DUHL_CB(16, 3, 2, 2)
    DUHL_CB(16, 3, 2, 3)
    DUHL_CB(16, 6, 2, 2)
    DUHL_CB(64, 1, 2, 3)
    DUHL_CB(64, 1, 4, 2)
    if (!launched) hipLaunchKernelGGL((csr_blocked_dot_kernel<16, 3, 2, 3>), grid, dim3(1024), 0, c->compute, a);
#undef DUHL_CB
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
    f.count = a.count;
    f.R = c->cb_R;
    const int64_t fgrid = (a.count + 255) / 256;
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
