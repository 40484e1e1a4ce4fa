// One pass of exact coordinate steps over the working set (Algorithm 3 / Appendix D).
//
// Sequential scheme: a single workgroup (dense) or wavefront (sparse) visits the coordinates in
// the given order; reductions run in a fixed order, so the pass is reproducible.
//
// Asynchronous scheme (the TPA-SCD idea of Appendix D re-designed for wave64 hardware): a group
// of T threads owns one coordinate at a time.  It streams the column once from HBM with 16-byte
// loads and KEEPS IT IN REGISTERS, forms a_j^T v against the live shared vector (loads at agent
// scope, so updates made on other XCDs are seen), solves the coordinate exactly and, only if
// alpha_j moved, adds a_j * delta to v with hardware fp32 atomics straight from those registers
// -- the column is read from memory exactly once per update.  T is 64 (one wavefront, short
// columns), 256 or 1024 so that a column fits the group's registers.  Groups take coordinates
// with a fixed stride; the number of groups is the number of coordinates in flight.
#include "duhl_internal.h"

namespace duhl {

namespace {

struct CdArgs {
    ColView cv;
    ModelConst mc;
    int64_t d, count;
    const int32_t *order;   // explicit visiting order, or nullptr
    const int32_t *P;       // working set (used when order == nullptr)
    int permute;            // visit P through a pseudo-random bijection
    uint32_t pbits, pmul[3], padd[3];
    float *alpha, *v;
    const float *q, *target;
};

// Bijection on [0, count): multiply-add and xor-shift steps are each invertible on pbits bits;
// values that fall outside [0, count) are walked on until they land inside (cycle walking).
__device__ __forceinline__ int64_t permuted(const CdArgs &a, int64_t t)
{
    const uint32_t mask = (1u << a.pbits) - 1u, sh = (a.pbits >> 1) ? (a.pbits >> 1) : 1u;
    uint32_t x = (uint32_t)t;
    do {
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            x = (x * a.pmul[r] + a.padd[r]) & mask;
            x ^= x >> sh;
        }
    } while ((int64_t)x >= a.count);
    return (int64_t)x;
}

__device__ __forceinline__ int64_t coord_at(const CdArgs &a, int64_t t)
{
    if (a.order) return a.order[t];
    return a.P[a.permute ? permuted(a, t) : t];
}

// Loads of the shared vector that must observe other workgroups' atomic adds.
__device__ __forceinline__ float live_load(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 live_load4(const float *p)
{
    float4 r;
    r.x = live_load(p);
    r.y = live_load(p + 1);
    r.z = live_load(p + 2);
    r.w = live_load(p + 3);
    return r;
}
__device__ __forceinline__ void live_add(float *p, float x)
{
    (void)__hip_atomic_fetch_add(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float dot4(const float4 x, const float4 y, float acc)
{
    acc = fmaf(x.x, y.x, acc);
    acc = fmaf(x.y, y.y, acc);
    acc = fmaf(x.z, y.z, acc);
    acc = fmaf(x.w, y.w, acc);
    return acc;
}

// Sum over the T threads that share a coordinate; every thread gets the result.
template <int T>
__device__ __forceinline__ float group_reduce(float x, float (*red)[16], int parity)
{
    x = wave_sum(x);
    if (T == 64) return x;
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[parity][w] = x;
    __syncthreads();
    float s = 0.0f;
#pragma unroll
    for (int u = 0; u < T / 64; ++u) s += red[parity][u];
    return s;
}

// ---- asynchronous, dense ------------------------------------------------------------------------
template <int MODEL, int T, int NREG, bool VEC4>
__global__ __launch_bounds__(T == 64 ? 256 : T) void cd_dense_async_kernel(const CdArgs a)
{
    constexpr int BLOCK = T == 64 ? 256 : T;
    __shared__ float red[2][16];
    const int tid = threadIdx.x % T;
    const int64_t ngroups = (int64_t)gridDim.x * (BLOCK / T);
    const int64_t d4 = VEC4 ? (a.d >> 2) : 0;
    int parity = 0;
    for (int64_t t = (int64_t)blockIdx.x * (BLOCK / T) + threadIdx.x / T; t < a.count;
         t += ngroups) {
        const int64_t j = coord_at(a, t);
        const float *col = a.cv.col(j);
        const float4 *c4 = reinterpret_cast<const float4 *>(col);
        float4 x[NREG];
        float acc = 0.0f;
        if (VEC4) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int64_t r = tid + (int64_t)i * T;
                x[i] = r < d4 ? c4[r] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            // v is consumed four chunks at a time so that its values never crowd out the column
#pragma unroll
            for (int i0 = 0; i0 < NREG; i0 += 4) {
#pragma unroll
                for (int i = i0; i < (i0 + 4 < NREG ? i0 + 4 : NREG); ++i) {
                    const int64_t r = tid + (int64_t)i * T;
                    if (r < d4) acc = dot4(x[i], live_load4(a.v + 4 * r), acc);
                }
                if (i0 + 4 < NREG) __builtin_amdgcn_sched_barrier(0);
            }
            for (int64_t r = tid + (int64_t)NREG * T; r < d4; r += T)     // beyond the registers
                acc = dot4(c4[r], live_load4(a.v + 4 * r), acc);
        }
        for (int64_t r = (d4 << 2) + tid; r < a.d; r += T) acc = fmaf(col[r], live_load(a.v + r), acc);
        const float c = group_reduce<T>(acc, red, parity);
        parity ^= 1;

        const float old = a.alpha[j];
        const float y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
        const float now = cd_new_alpha<MODEL>(a.mc, c, old, a.q[j], y);
        const float delta = now - old;
        if (delta != 0.0f) {
            if (VEC4) {
#pragma unroll
                for (int i = 0; i < NREG; ++i) {
                    const int64_t r = tid + (int64_t)i * T;
                    if (r < d4) {
                        float *p = a.v + 4 * r;
                        live_add(p, x[i].x * delta);
                        live_add(p + 1, x[i].y * delta);
                        live_add(p + 2, x[i].z * delta);
                        live_add(p + 3, x[i].w * delta);
                    }
                }
                for (int64_t r = tid + (int64_t)NREG * T; r < d4; r += T) {
                    const float4 xx = c4[r];
                    float *p = a.v + 4 * r;
                    live_add(p, xx.x * delta);
                    live_add(p + 1, xx.y * delta);
                    live_add(p + 2, xx.z * delta);
                    live_add(p + 3, xx.w * delta);
                }
            }
            for (int64_t r = (d4 << 2) + tid; r < a.d; r += T) live_add(a.v + r, col[r] * delta);
            if (tid == 0) a.alpha[j] = now;
        }
    }
}

// ---- asynchronous, sparse: G lanes per coordinate -------------------------------------------------
template <int MODEL, int G>
__global__ __launch_bounds__(256) void cd_csr_async_kernel(const CdArgs a)
{
    const int sub = threadIdx.x % G;
    const int64_t ngroups = (int64_t)gridDim.x * (256 / G);
    for (int64_t t = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G; t < a.count; t += ngroups) {
        const int64_t j = coord_at(a, t);
        const int64_t beg = a.cv.rowptr[j], end = a.cv.rowptr[j + 1];
        float acc = 0.0f;
        for (int64_t e = beg + sub; e < end; e += G)
            acc = fmaf(a.cv.val[e], live_load(a.v + a.cv.colidx[e]), acc);
        const float c = group_sum<G>(acc);
        const float old = a.alpha[j];
        const float y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
        const float now = cd_new_alpha<MODEL>(a.mc, c, old, a.q[j], y);
        const float delta = now - old;
        if (delta != 0.0f) {
            for (int64_t e = beg + sub; e < end; e += G)
                live_add(a.v + a.cv.colidx[e], a.cv.val[e] * delta);
            if (sub == 0) a.alpha[j] = now;
        }
    }
}

// ---- sequential ----------------------------------------------------------------------------------
// One workgroup of 1024 threads.  Thread k always owns the same elements of v, so the vector
// needs no synchronisation between coordinates; only the dot product is reduced across threads.
template <int MODEL, bool VEC4>
__global__ __launch_bounds__(1024) void cd_dense_seq_kernel(const CdArgs a)
{
    constexpr int T = 1024;
    __shared__ float red[2][16];
    const int tid = threadIdx.x;
    const int64_t d4 = VEC4 ? (a.d >> 2) : 0;
    float4 *v4 = reinterpret_cast<float4 *>(a.v);
    int parity = 0;
    for (int64_t t = 0; t < a.count; ++t) {
        const int64_t j = coord_at(a, t);
        const float *col = a.cv.col(j);
        const float4 *c4 = reinterpret_cast<const float4 *>(col);
        float acc = 0.0f;
        for (int64_t r = tid; r < d4; r += T) acc = dot4(c4[r], v4[r], acc);
        for (int64_t r = (d4 << 2) + tid; r < a.d; r += T) acc = fmaf(col[r], a.v[r], acc);
        const float c = group_reduce<T>(acc, red, parity);
        parity ^= 1;
        const float old = a.alpha[j];
        const float y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
        const float now = cd_new_alpha<MODEL>(a.mc, c, old, a.q[j], y);
        const float delta = now - old;
        if (delta != 0.0f) {
            for (int64_t r = tid; r < d4; r += T) {
                const float4 xx = c4[r];
                float4 vv = v4[r];
                vv.x = fmaf(xx.x, delta, vv.x);
                vv.y = fmaf(xx.y, delta, vv.y);
                vv.z = fmaf(xx.z, delta, vv.z);
                vv.w = fmaf(xx.w, delta, vv.w);
                v4[r] = vv;
            }
            for (int64_t r = (d4 << 2) + tid; r < a.d; r += T) a.v[r] = fmaf(col[r], delta, a.v[r]);
        }
        __syncthreads();                       // alpha[j] may be read again by a later visit
        if (tid == 0 && delta != 0.0f) a.alpha[j] = now;
    }
}

// One wavefront; the barrier orders the scattered updates of v before the next gathers.
template <int MODEL>
__global__ __launch_bounds__(64) void cd_csr_seq_kernel(const CdArgs a)
{
    const int lane = threadIdx.x;
    for (int64_t t = 0; t < a.count; ++t) {
        const int64_t j = coord_at(a, t);
        const int64_t beg = a.cv.rowptr[j], end = a.cv.rowptr[j + 1];
        float acc = 0.0f;
        for (int64_t e = beg + lane; e < end; e += 64) acc = fmaf(a.cv.val[e], a.v[a.cv.colidx[e]], acc);
        const float c = wave_sum(acc);
        const float old = a.alpha[j];
        const float y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
        const float now = cd_new_alpha<MODEL>(a.mc, c, old, a.q[j], y);
        const float delta = now - old;
        if (delta != 0.0f) {
            for (int64_t e = beg + lane; e < end; e += 64) {
                const int32_t k = a.cv.colidx[e];
                a.v[k] = fmaf(a.cv.val[e], delta, a.v[k]);
            }
        }
        __syncthreads();
        if (lane == 0 && delta != 0.0f) a.alpha[j] = now;
        __syncthreads();
    }
}

uint64_t splitmix64(uint64_t &s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <int MODEL, int T, int NREG>
hipError_t launch_async_dense_t(duhl_ctx *c, const CdArgs &a, int inflight, bool vec)
{
    constexpr int BLOCK = T == 64 ? 256 : T;
    constexpr int PER = BLOCK / T;
    int64_t grid = (inflight + PER - 1) / PER;
    if (grid < 1) grid = 1;
    if (vec)
        hipLaunchKernelGGL((cd_dense_async_kernel<MODEL, T, NREG, true>), dim3(grid), dim3(BLOCK), 0,
                           c->compute, a);
    else
        hipLaunchKernelGGL((cd_dense_async_kernel<MODEL, T, 1, false>), dim3(grid), dim3(BLOCK), 0,
                           c->compute, a);
    return hipGetLastError();
}

template <int MODEL, int T>
hipError_t launch_async_dense_n(duhl_ctx *c, const CdArgs &a, int inflight, bool vec)
{
    const int64_t chunks = ((c->d >> 2) + T - 1) / T;   // float4 per thread to hold a column
    if (chunks <= 1) return launch_async_dense_t<MODEL, T, 1>(c, a, inflight, vec);
    if (chunks <= 2) return launch_async_dense_t<MODEL, T, 2>(c, a, inflight, vec);
    if (chunks <= 4) return launch_async_dense_t<MODEL, T, 4>(c, a, inflight, vec);
    if (chunks <= 8) return launch_async_dense_t<MODEL, T, 8>(c, a, inflight, vec);
    if (chunks <= 13) return launch_async_dense_t<MODEL, T, 13>(c, a, inflight, vec);
    if (chunks <= 16) return launch_async_dense_t<MODEL, T, 16>(c, a, inflight, vec);
    return launch_async_dense_t<MODEL, T, 20>(c, a, inflight, vec);
}

int threads_per_coordinate(const duhl_ctx *c)
{
    if (c->cd_threads == 64 || c->cd_threads == 256 || c->cd_threads == 1024) return c->cd_threads;
    if (c->d <= 2048) return 64;
    if (c->d <= 16384) return 256;
    return 1024;
}

template <int MODEL>
hipError_t launch_cd_model(duhl_ctx *c, duhl_cd_mode mode, const CdArgs &a, int max_inflight)
{
    const bool vec = !c->sparse && aligned16(a.cv.base) && (a.cv.ld % 4 == 0) && aligned16(a.v) &&
                     (!a.cv.col_slot || (aligned16(a.cv.slots) && a.cv.ld_s % 4 == 0));
    if (mode == DUHL_CD_SEQUENTIAL) {
        if (c->sparse)
            hipLaunchKernelGGL(cd_csr_seq_kernel<MODEL>, dim3(1), dim3(64), 0, c->compute, a);
        else if (vec)
            hipLaunchKernelGGL((cd_dense_seq_kernel<MODEL, true>), dim3(1), dim3(1024), 0, c->compute, a);
        else
            hipLaunchKernelGGL((cd_dense_seq_kernel<MODEL, false>), dim3(1), dim3(1024), 0, c->compute, a);
        return hipGetLastError();
    }
    // Coordinates in flight: a hardware ceiling, and by default at most count/8 so that
    // concurrent steps stay a small fraction of the block (each step sees a slightly stale v).
    if (c->sparse) {
        const int64_t avg = c->n > 0 ? c->nnz / c->n : 0;
        const int G = avg > 256 ? 64 : 16;
        int64_t cap = (int64_t)c->num_cu * 8 * (256 / G);
        int64_t inflight = max_inflight > 0 ? max_inflight : (a.count / 8 > 0 ? a.count / 8 : 1);
        if (inflight > cap) inflight = cap;
        if (inflight > a.count) inflight = a.count;
        const int64_t grid = (inflight + 256 / G - 1) / (256 / G);
        if (G == 64)
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 64>), dim3(grid), dim3(256), 0, c->compute, a);
        else
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 16>), dim3(grid), dim3(256), 0, c->compute, a);
        return hipGetLastError();
    }
    const int T = threads_per_coordinate(c);
    int64_t cap = (int64_t)c->num_cu * (2048 / T);
    int64_t inflight = max_inflight > 0 ? max_inflight : (a.count / 8 > 0 ? a.count / 8 : 1);
    if (inflight > cap) inflight = cap;
    if (inflight > a.count) inflight = a.count;
    if (T == 64) return launch_async_dense_n<MODEL, 64>(c, a, (int)inflight, vec);
    if (T == 256) return launch_async_dense_n<MODEL, 256>(c, a, (int)inflight, vec);
    return launch_async_dense_n<MODEL, 1024>(c, a, (int)inflight, vec);
}

}  // namespace

hipError_t launch_cd(duhl_ctx *c, duhl_cd_mode mode, const int32_t *order, int64_t count,
                     uint64_t seed, int max_inflight)
{
    CdArgs a;
    a.cv = c->cv;
    a.mc = c->mc;
    a.d = c->d;
    a.order = order;
    a.P = c->P_cur;
    a.count = order ? count : c->m_cur;
    a.permute = (!order && mode == DUHL_CD_ASYNC) ? 1 : 0;
    a.alpha = c->alpha;
    a.v = c->v;
    a.q = c->q;
    a.target = c->target;
    a.pbits = 1;
    while ((1ll << a.pbits) < a.count) ++a.pbits;
    uint64_t s = seed ^ (0xD1B54A32D192ED03ull * (c->pass_counter + 1));
    for (int r = 0; r < 3; ++r) {
        a.pmul[r] = (uint32_t)splitmix64(s) | 1u;     // odd: invertible modulo a power of two
        a.padd[r] = (uint32_t)splitmix64(s);
    }
    if (a.count <= 0) return hipSuccess;
    return c->model == DUHL_LASSO ? launch_cd_model<DUHL_LASSO>(c, mode, a, max_inflight)
                                  : launch_cd_model<DUHL_SVM>(c, mode, a, max_inflight);
}

}  // namespace duhl
