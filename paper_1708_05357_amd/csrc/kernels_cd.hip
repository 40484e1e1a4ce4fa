// One pass of exact coordinate steps over the working set (Algorithm 3 / Appendix D).
//
// Sequential scheme: a single workgroup (dense) or wavefront (sparse) visits the coordinates in
// the given order; reductions run in a fixed order, so the pass is reproducible.
//
// Atomic scheme (the TPA-SCD idea of Appendix D on wave64 hardware): a group of T threads owns
// one coordinate at a time.  It streams the column once from HBM with 16-byte loads and keeps it
// in registers, forms a_j^T v against the live shared vector (16-byte buffer loads at agent scope,
// so updates made on other XCDs are seen), solves the coordinate exactly and, only if alpha_j
// moved, adds a_j * delta to v with hardware fp32 atomics straight from those registers.
//
// Asynchronous scheme for dense data, built around what the atomic units of this chip can
// sustain (about 0.3 T fp32 atomic adds/s device-wide, far below the 2 T floats/s that HBM
// streams): a pass is cut into sub-passes of at most `inflight` coordinates.  Inside a sub-pass
// every worker (a group of T threads) keeps its OWN copy of v in registers, visits its share of
// the coordinates one after the other -- each step exact against that copy, so a worker is a
// sequential solver -- and finally stores its accumulated change of v to a private buffer; a
// merge kernel adds the buffers to v in a fixed order.  Per update the only memory traffic is
// the column itself, read once; there are no atomics and the result is reproducible.  Workers do
// not see each other inside a sub-pass, exactly like concurrently running thread blocks that
// read a stale v; `inflight` bounds that staleness.  A worker is a wavefront, a quarter of a
// workgroup or a whole 1024-thread workgroup by column length; for columns beyond what one
// compute unit can hold on chip (a copy of v plus the column), two or four workgroups on
// different compute units form one worker and exchange their partial dot products per
// coordinate.  Sparse data keeps the atomic scheme: its scattered updates are few and spread
// over all of v.
#include <cmath>

#include "duhl_internal.h"

namespace duhl {

namespace {

// What a sparse step needs to know before it can fetch its row, gathered once per pass for every
// position of the visiting order (32 bytes, read with two 16-byte loads).
struct CdPlan {
    int64_t beg;            // first entry of the row
    int32_t j, len;         // coordinate (-1: skip) and its number of entries
    float alpha, q, y, pad;
};
static_assert(sizeof(CdPlan) == 32, "two 16-byte loads");

struct CdArgs {
    ColView cv;
    ModelConst mc;
    int64_t d, n, count;
    int64_t groups;         // concurrent schemes: groups of threads that take coordinates
    const int32_t *order;   // explicit visiting order, or nullptr
    const int32_t *P;       // working set (used when order == nullptr)
    int permute;            // visit P through a pseudo-random bijection
    uint32_t pbits, pmul[3], padd[3];
    float *alpha, *v;
    const float *q, *target;
    CdPlan *plan;           // sparse sub-passes only
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

// Coordinate visited at position t; -1 for an entry of a caller's list that names no coordinate
// (such entries are skipped: the value is the same in all threads that share the coordinate).
__device__ __forceinline__ int64_t coord_at(const CdArgs &a, int64_t t)
{
    if (a.order) {
        const int64_t j = a.order[t];
        return (uint64_t)j < (uint64_t)a.n ? j : -1;
    }
    const int64_t j = a.P[a.permute ? permuted(a, t) : t];
    return (uint64_t)j < (uint64_t)a.n ? j : -1;
}

// Loads of the shared vector that must observe other workgroups' atomic adds.
__device__ __forceinline__ float live_load(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same for 16 bytes in one instruction: a raw buffer load whose cache-policy operand carries
// the agent-scope bit (sc1); rs describes v, byte_off is bounds-checked by the hardware.
typedef int v4i_t __attribute__((ext_vector_type(4)));
// Plain 16-byte buffer load / store: address = base + voff (per lane) + soff (uniform); accesses
// past the size recorded in rs return 0 / are dropped, so ragged ends need no branch.
__device__ __forceinline__ float4 buffer_load4(__amdgpu_buffer_rsrc_t rs, int voff, int soff)
{
    const v4i_t raw = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
    return make_float4(__int_as_float(raw.x), __int_as_float(raw.y), __int_as_float(raw.z),
                       __int_as_float(raw.w));
}
// Column data whose start is only 4-byte aligned (leading dimension not a multiple of four floats):
// the same 16 bytes as four dword loads.  STREAM selects the non-temporal hint.
template <bool XVEC, bool STREAM>
__device__ __forceinline__ float4 column_load4(__amdgpu_buffer_rsrc_t rs, int voff, int soff)
{
    constexpr int kAux = STREAM ? 2 : 0;
    if (XVEC) {
        const v4i_t raw = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, kAux);
        return make_float4(__int_as_float(raw.x), __int_as_float(raw.y), __int_as_float(raw.z),
                           __int_as_float(raw.w));
    }
    return make_float4(__int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, kAux)),
                       __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff + 4, kAux)),
                       __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff + 8, kAux)),
                       __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff + 12, kAux)));
}
__device__ __forceinline__ void buffer_store4(__amdgpu_buffer_rsrc_t rs, int voff, int soff, float4 x)
{
    v4i_t raw;
    raw.x = __float_as_int(x.x);
    raw.y = __float_as_int(x.y);
    raw.z = __float_as_int(x.z);
    raw.w = __float_as_int(x.w);
    __builtin_amdgcn_raw_buffer_store_b128(raw, rs, voff, soff, 0);
}
// 16 bytes written through to device-coherent memory (the store's cache-policy operand carries the
// agent-scope bit), for data that another workgroup of the same launch reads or overwrites.
__device__ __forceinline__ void coherent_store4(__amdgpu_buffer_rsrc_t rs, int byte_off, float4 x)
{
    v4i_t raw;
    raw.x = __float_as_int(x.x);
    raw.y = __float_as_int(x.y);
    raw.z = __float_as_int(x.z);
    raw.w = __float_as_int(x.w);
    __builtin_amdgcn_raw_buffer_store_b128(raw, rs, byte_off, 0, 16);
}
__device__ __forceinline__ float4 live_load4(__amdgpu_buffer_rsrc_t rs, int byte_off)
{
    const v4i_t raw = __builtin_amdgcn_raw_buffer_load_b128(rs, byte_off, 0, 16);
    return make_float4(__int_as_float(raw.x), __int_as_float(raw.y), __int_as_float(raw.z),
                       __int_as_float(raw.w));
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
__global__ __launch_bounds__(T == 64 ? 256 : T) void cd_dense_atomic_kernel(const CdArgs a)
{
    constexpr int BLOCK = T == 64 ? 256 : T;
    __shared__ float red[2][16];
    const int tid = threadIdx.x % T;
    // a.groups of the launched groups work (the last workgroup may hold idle ones, which only
    // happens for T = 64, where a group is a wavefront and shares no barrier with its neighbours)
    const int64_t ngroups = a.groups;
    const int64_t d4 = VEC4 ? (a.d >> 2) : 0;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(a.v, 0, (int)(a.d * 4), 0x00020000);
    int parity = 0;
    const int64_t first = (int64_t)blockIdx.x * (BLOCK / T) + threadIdx.x / T;
    if (first >= ngroups) return;
    for (int64_t t = first; t < a.count; t += ngroups) {
        const int64_t j = coord_at(a, t);
        if (j < 0) continue;
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
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int64_t r = tid + (int64_t)i * T;
                if (r < d4) acc = dot4(x[i], live_load4(rs, (int)(r * 16)), acc);
            }
            for (int64_t r = tid + (int64_t)NREG * T; r < d4; r += T)     // beyond the registers
                acc = dot4(c4[r], live_load4(rs, (int)(r * 16)), acc);
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


// A worker (or a group of lanes of the sparse kernel) sits a sub-pass out when the guard asks for
// fewer concurrent steps than the host knew of when it cut the pass into sub-passes: the host reads
// the guard's books without waiting and may be many passes ahead of the device.  With e halvings
// outstanding only every 2^e-th worker takes its share, so a sub-pass solves 1/2^e of its
// coordinates -- the pass still descends, on a random part of the working set -- until the host
// catches up and cuts its passes finer.
__device__ __forceinline__ bool guard_sits_out(const GuardState *st, int host_shift, int64_t worker)
{
    if (!st) return false;
    // (a plain, cached load: the word only changes at the end of a pass, i.e. between kernels)
    const int dev_shift = (int)st->shift;
    const int e = dev_shift - host_shift;
    return e > 0 && (worker & ((1ll << e) - 1)) != 0;
}

// ---- workers that span several compute units -----------------------------------------------------
// The CUS workgroups of one worker each hold a slice of the private v and of every column; per
// coordinate they exchange their partial dot products through a pair of 8-byte slots per
// workgroup in device memory: (sequence number, value) written and read as one word at agent
// scope.  Slot (seq & 1) is written for sequence number seq; a workgroup writes seq + 2 only
// after it has read every partner's seq + 1, which a partner writes only after it has read this
// workgroup's seq -- so two slots are enough.  The sum runs over the partners in a fixed order,
// hence every workgroup gets the same bits.  Waiting is bounded: after spin_limit polls (seconds
// with the default of 2^22) the workgroup raises the abort flag, which makes all of them leave
// their loops.
template <int CUS>
__device__ __forceinline__ float partner_sum(float mine, uint64_t *slots, int part, uint32_t seq,
                                             uint32_t *abort_flag, int spin_limit, float (*bcast)[2],
                                             int parity, bool &failed)
{
    if (threadIdx.x == 0) {
        uint64_t *mine_slot = slots + (seq & 1u) * CUS;
        __hip_atomic_store(mine_slot + part, ((uint64_t)seq << 32) | __float_as_uint(mine),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float total = 0.0f;
        bool ok = true;
        for (int q = 0; q < CUS; ++q) {
            float val = mine;
            if (q != part && ok) {
                uint64_t got = 0;
                int spins = 0;
                for (;;) {
                    got = __hip_atomic_load(mine_slot + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((uint32_t)(got >> 32) == seq) break;
                    ++spins;
                    if (spins > spin_limit ||
                        ((spins & 1023) == 0 &&
                         __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                        ok = false;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                val = __uint_as_float((uint32_t)got);
            }
            total += val;
        }
        if (!ok) __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bcast[parity][0] = total;
        bcast[parity][1] = ok ? 0.0f : 1.0f;
    }
    __syncthreads();
    failed = bcast[parity][1] != 0.0f;
    return bcast[parity][0];
}

// ---- asynchronous, dense: workers with a private copy of v --------------------------------------
// One sub-pass over positions [t_begin, t_end) of the visiting order.  The worker's copy of v is
// NR 16-byte chunks per thread in registers plus NL chunks per thread in LDS (each thread only ever
// touches its own LDS entries, so no barrier is needed for them).  CACHE_X keeps the column in
// registers between the dot product and the update (one read per update); without it (very long
// columns: the registers are needed for v) the column is read again, only when alpha_j moved.
// EXT: columns longer than registers and LDS can hold a copy of v for (T*(NR+NL) float4).  The rest
// of the worker's copy lives in its private buffer in device memory -- 400 KB or more per worker
// that it re-reads for every coordinate, so it is served by L2 / the memory-side cache while the
// column streams from HBM.  Each thread only touches its own rows there as well.
// CUS > 1: a worker is CUS workgroups, each with rows [part*S, (part+1)*S) of v and of the columns,
// S = T*(NR+NL)*4, all of it on chip and the column cached; they meet once per coordinate in
// partner_sum.  Workgroups 8 apart belong together: consecutive workgroups are dealt to the eight
// dies in turn, so partners share a die and its L2 (a matter of speed only).
template <int MODEL, int T, int NR, int NL, bool CACHE_X, bool EXT = false, bool XVEC = true, int CUS = 1>
__global__ __launch_bounds__(T == 64 ? 256 : T) void cd_dense_worker_kernel(
    const CdArgs a, const int64_t t_begin, const int64_t t_end, float *dv, const int64_t dv_stride,
    int32_t *dirty, uint64_t *xch, const uint32_t seq_base, uint32_t *abort_flag, const int spin_limit,
    uint64_t *alpha_old, const uint32_t stamp, const GuardState *guard, const int host_shift, double2 *wbook)
{
    static_assert(CUS == 1 || (T == 1024 && !EXT && CACHE_X), "multi-unit workers: cached, on chip");
    constexpr int BLOCK = T == 64 ? 256 : T;
    constexpr int NC = NR + NL;                        // chunks per thread that cover a column
    constexpr int kStep = T * 16;                      // bytes between a thread's chunks
    constexpr int KB = NR >= 14 ? 4 : 8;               // column chunks in flight when not cached
    __shared__ float red[2][16];
    __shared__ float xsum[2][2];
    __shared__ float4 vs[NL > 0 ? NL * BLOCK : 1];
    const int tid = threadIdx.x % T;
    // the worker index is the same in all lanes of a wavefront: say so to the compiler
    int w = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (BLOCK / T) + threadIdx.x / T));
    int64_t nworkers = (int64_t)gridDim.x * (BLOCK / T);
    int part = 0;                                      // which slice of the rows this workgroup holds
    if (CUS > 1) {
        const int local = blockIdx.x % (8 * CUS);
        part = local / 8;
        w = (int)(blockIdx.x / (8 * CUS)) * 8 + local % 8;
        nworkers = gridDim.x / CUS;
    }
    const int64_t d4 = a.d >> 2;
    const int tail = part == CUS - 1 ? (int)(a.d - (d4 << 2)) : 0;   // ragged rows: last slice
    const int64_t slice = (int64_t)part * NC * T * 4;  // first row of the slice
    int vec_bytes = (int)(d4 << 4);                    // 16-byte part of a column; loads beyond it
    if (CUS > 1) {                                     // return 0 (buffer bounds check)
        vec_bytes -= part * NC * kStep;
        vec_bytes = vec_bytes < 0 ? 0 : (vec_bytes > NC * kStep ? NC * kStep : vec_bytes);
    }
    const int off = tid * 16;
    const __amdgpu_buffer_rsrc_t rs_v =
        __builtin_amdgcn_make_buffer_rsrc(a.v + slice, 0, vec_bytes, 0x00020000);
    float *const out = dv + (int64_t)w * dv_stride;    // this worker's private buffer
    const __amdgpu_buffer_rsrc_t rs_o =
        __builtin_amdgcn_make_buffer_rsrc(out + slice, 0, vec_bytes, 0x00020000);
    uint32_t seq = seq_base;                           // one number per coordinate of this worker
    const int nch = (int)((d4 + T - 1) / T);           // chunks per thread that cover a column
    if (EXT) {                                         // rows beyond the on-chip copy: start from v
        for (int i0 = NC; i0 < nch; i0 += 8) {
            float4 vb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) vb[u] = buffer_load4(rs_v, off, (i0 + u) * kStep);
#pragma unroll
            for (int u = 0; u < 8; ++u) buffer_store4(rs_o, off, (i0 + u) * kStep, vb[u]);
        }
    }

    float4 vr[NR > 0 ? NR : 1];                        // rows 4*(tid + i*T) .. of this worker's v
#pragma unroll
    for (int i = 0; i < NR; ++i) vr[i] = buffer_load4(rs_v, off, i * kStep);
#pragma unroll
    for (int l = 0; l < NL; ++l) vs[l * BLOCK + threadIdx.x] = buffer_load4(rs_v, off, (NR + l) * kStep);
    float vt = tid < tail ? a.v[(d4 << 2) + tid] : 0.0f;
    bool moved = false;
    int parity = 0;
    double dreg = 0.0;                                 // guard: change of the objective's terms in alpha
    const bool idle = guard_sits_out(guard, host_shift, w);      // (the same in all parts of a worker)
    unsigned int nsteps = 0;
    for (int64_t t = t_begin + w; t < t_end && !idle; t += nworkers) {
        const int j = __builtin_amdgcn_readfirstlane((int)coord_at(a, t));
        if (j < 0) continue;
        ++nsteps;
        const float *col = a.cv.col(j);
        const __amdgpu_buffer_rsrc_t rs_x =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(col + slice), 0, vec_bytes, 0x00020000);
        // the scalars of the step are requested before the column, so that nothing issued later
        // (loads complete in order) stands between the reduced dot product and the update
        const float old = a.alpha[j];
        const float qj = a.q[j];
        const float y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
        float4 x[CACHE_X ? NC : 1];
        float acc = 0.0f;
        if (CACHE_X) {
#pragma unroll
            for (int i = 0; i < NC; ++i) x[i] = column_load4<XVEC, true>(rs_x, off, i * kStep);
#pragma unroll
            for (int i = 0; i < NR; ++i) acc = dot4(x[i], vr[i], acc);
#pragma unroll
            for (int l = 0; l < NL; ++l) acc = dot4(x[NR + l], vs[l * BLOCK + threadIdx.x], acc);
        } else {
            // KB chunks of the column in flight at a time: the registers belong to v.  The
            // empty asm makes the next batch's address depend on this batch's sum, which is what
            // keeps the compiler from issuing all loads at once and spilling v.
            int offb = off;
#pragma unroll
            for (int i0 = 0; i0 < NC; i0 += KB) {
                float4 xb[KB];
#pragma unroll
                for (int u = 0; u < KB; ++u)
                    if (i0 + u < NC) xb[u] = column_load4<XVEC, true>(rs_x, offb, (i0 + u) * kStep);
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int i = i0 + u;
                    if (i < NR) acc = dot4(xb[u], vr[i < NR ? i : 0], acc);
                    else if (i < NC) acc = dot4(xb[u], vs[(i - NR) * BLOCK + threadIdx.x], acc);
                }
                asm volatile("" : "+v"(offb), "+v"(acc));
            }
            if (EXT) {
                for (int i0 = NC; i0 < nch; i0 += KB) {
                    float4 xb[KB], vb[KB];
#pragma unroll
                    for (int u = 0; u < KB; ++u) {
                        xb[u] = column_load4<XVEC, true>(rs_x, offb, (i0 + u) * kStep);
                        vb[u] = buffer_load4(rs_o, offb, (i0 + u) * kStep);
                    }
#pragma unroll
                    for (int u = 0; u < KB; ++u) acc = dot4(xb[u], vb[u], acc);
                    asm volatile("" : "+v"(offb), "+v"(acc));
                }
            }
        }
        const float xt = tid < tail ? col[(d4 << 2) + tid] : 0.0f;
        acc = fmaf(xt, vt, acc);
        float c = group_reduce<T>(acc, red, parity);
        if (CUS > 1) {
            bool failed = false;
            ++seq;
            c = partner_sum<CUS>(c, xch + (int64_t)w * 2 * CUS, part, seq, abort_flag, spin_limit, xsum, parity,
                                 failed);
            if (failed) break;                         // same decision in all threads and partners
        }
        parity ^= 1;

        const float now = cd_new_alpha<MODEL>(a.mc, c, old, qj, y);
        const float delta = now - old;
        if (delta != 0.0f) {
            int offu = off;
            float tie = 0.0f;
#pragma unroll
            for (int i0 = 0; i0 < NC; i0 += KB) {
                float4 xb[KB];
#pragma unroll
                for (int u = 0; u < KB; ++u)
                    if (i0 + u < NC)
                        xb[u] = CACHE_X ? x[CACHE_X ? i0 + u : 0] : column_load4<XVEC, false>(rs_x, offu, (i0 + u) * kStep);
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int i = i0 + u;
                    if (i < NR) {
                        float4 &vv = vr[i < NR ? i : 0];
                        vv.x = fmaf(xb[u].x, delta, vv.x);
                        vv.y = fmaf(xb[u].y, delta, vv.y);
                        vv.z = fmaf(xb[u].z, delta, vv.z);
                        vv.w = fmaf(xb[u].w, delta, vv.w);
                    } else if (i < NC) {
                        float4 vv = vs[(i - NR) * BLOCK + threadIdx.x];
                        vv.x = fmaf(xb[u].x, delta, vv.x);
                        vv.y = fmaf(xb[u].y, delta, vv.y);
                        vv.z = fmaf(xb[u].z, delta, vv.z);
                        vv.w = fmaf(xb[u].w, delta, vv.w);
                        vs[(i - NR) * BLOCK + threadIdx.x] = vv;
                        tie = vv.x;
                    }
                    if (i < NR) tie = vr[i < NR ? i : 0].x;
                }
                if (!CACHE_X) asm volatile("" : "+v"(offu), "+v"(tie));
            }
            if (EXT) {
                for (int i0 = NC; i0 < nch; i0 += KB) {
                    float4 xb[KB], vb[KB];
#pragma unroll
                    for (int u = 0; u < KB; ++u) {
                        xb[u] = column_load4<XVEC, false>(rs_x, offu, (i0 + u) * kStep);
                        vb[u] = buffer_load4(rs_o, offu, (i0 + u) * kStep);
                    }
#pragma unroll
                    for (int u = 0; u < KB; ++u) {
                        vb[u].x = fmaf(xb[u].x, delta, vb[u].x);
                        vb[u].y = fmaf(xb[u].y, delta, vb[u].y);
                        vb[u].z = fmaf(xb[u].z, delta, vb[u].z);
                        vb[u].w = fmaf(xb[u].w, delta, vb[u].w);
                        buffer_store4(rs_o, offu, (i0 + u) * kStep, vb[u]);   // beyond the end: dropped
                    }
                    asm volatile("" : "+v"(offu));
                }
            }
            vt = fmaf(xt, delta, vt);
            moved = true;
            if (tid == 0 && part == 0) {
                a.alpha[j] = now;
                if (alpha_old) {                       // what undoing the pass needs, and what it is judged by
                    alpha_old[t] = ((uint64_t)stamp << 32) | __float_as_uint(old);
                    dreg += objective_term_change<MODEL>(a.mc, now, old, y);
                }
            }
        }
    }
    // the worker's books for the guard: what its steps changed in the objective's terms in alpha, and
    // how many it took (one slot per worker, added up by the merge: thousands of atomic adds on one
    // word at the end of a kernel cost more than the whole merge)
    if (wbook && tid == 0 && part == 0) wbook[w] = make_double2(dreg, (double)nsteps);
    if (moved) {                                       // this worker's change of v
        int offo = off;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            float4 base = buffer_load4(rs_v, offo, i * kStep);
            const float4 mine = i < NR ? vr[i < NR ? i : 0] : vs[(i < NR ? 0 : i - NR) * BLOCK + threadIdx.x];
            buffer_store4(rs_o, offo, i * kStep,
                          make_float4(mine.x - base.x, mine.y - base.y, mine.z - base.z,
                                      mine.w - base.w));                   // beyond the end: dropped
            if (!CACHE_X && (i & 3) == 3) asm volatile("" : "+v"(offo), "+v"(base.x));
        }
        if (EXT) {                                     // the copy in the buffer becomes a difference
            for (int i0 = NC; i0 < nch; i0 += 4) {
                float4 base[4], mine[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    base[u] = buffer_load4(rs_v, offo, (i0 + u) * kStep);
                    mine[u] = buffer_load4(rs_o, offo, (i0 + u) * kStep);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    buffer_store4(rs_o, offo, (i0 + u) * kStep,
                                  make_float4(mine[u].x - base[u].x, mine[u].y - base[u].y,
                                              mine[u].z - base[u].z, mine[u].w - base[u].w));
                asm volatile("" : "+v"(offo));
            }
        }
        if (tid < tail) out[(d4 << 2) + tid] = vt - a.v[(d4 << 2) + tid];
    }
    if (tid == 0 && part == 0) dirty[w] = moved ? 1 : 0;
}

// v += sum over workers of their stored changes, in a fixed order (reproducible).  A workgroup
// owns 256 consecutive elements of v as 64 chunks of 16 bytes; each of its 16 wavefronts adds up
// every 16th worker's buffer for those chunks (eight independent 1 KB loads in flight), then the
// 16 partial sums are added in wavefront order.  dirty[] is uniform, so skipping a clean worker is
// a scalar branch.  The buffers' rows are dv_stride (a multiple of 64) floats apart and hold
// nothing meaningful past d, so the last chunk is cut to d when it is added.
// The guard rides on this kernel.  The first merge of a pass keeps v as it was (snap) and its sum of
// squares; the last merge adds up <snap, v - snap> and ||v - snap||^2, and the workgroup that finishes
// last judges the pass from them and from the change of the terms in alpha that the workers
// accumulated (see GuardState).  A pass that overshot is scaled back to its best point on the line
// from the old iterate -- v and the pass's alpha_j are blended with their old values -- and counts a
// trip, which the host reads (without waiting) before its next pass and halves its bound on
// concurrent steps.
struct MergeGuard {
    GuardState *st;            // nullptr: no guard
    double *part;              // per workgroup: [0, blocks) old sums of squares, then <snap, dv>, then ||dv||^2
    float *snap;               // v at the start of the pass
    const uint64_t *alpha_old; // per position of the visiting order: (stamp of the pass that moved alpha_j, its old value)
    uint32_t stamp;            // this pass's stamp: older entries belong to coordinates that did not move now
    uint32_t *host_trips;      // host-visible copy of st->trips
    double quad;               // factor of ||v||^2 in the objective
    double tol;                // a rise below tol * (objective's magnitude) is taken for rounding
    double per_step;           // roundings that one coordinate step causes per element of v, on average
    int first, last;           // this merge ends the first / the last sub-pass of the pass
    int host_shift;            // halvings the host had applied when it cut the pass into sub-passes
    double2 *wbook;            // per worker: (change of the objective's terms in alpha, steps taken) in the sub-pass
};

// The judgement of a pass, by one thread; returns the factor theta by which the pass is to be kept
// (1: as it is, 0: undone).  o = ||v_old||^2, pd = <v_old, dv>, pq = ||dv||^2, dreg = change of the
// terms in alpha.  v is held in fp32: every step rounds it, so <v_old, dv> carries noise of about
// eps/2 * o * sqrt(roundings per element / d), and theta* is only read when ||dv||^2 stands well
// above that; a pass too small to tell leaves the books as they are (the bound found while the steps
// were large stays).  Keeps the guard's books: a pass with theta* < 0.55 is damped, counted, and asks
// for half as many concurrent steps (shift + 1); `need` passes with theta* >= 0.8 and no damped one
// between them ask for twice as many again, and need doubles with every damped pass.  trips and shift are mirrored into host-visible
// memory, which the host reads without waiting before it enqueues a pass.
__device__ __forceinline__ double guard_verdict(GuardState *st, uint32_t *host_words, const MergeGuard &g, double inv_d,
                                                double o, double pd, double pq, double dreg, unsigned long long steps)
{
    const double lin = 2.0 * g.quad * pd + dreg, curv = g.quad * pq;
    const double delta = lin + curv;                              // the objective's change at theta = 1
    const double rounds = fmax(1.0, (double)steps * g.per_step);
    const double noise = 0.5 * 1.1920929e-7 * o * sqrt(rounds * inv_d);
    double theta = 1.0;
    bool told = false;
    if (!(fabs(lin) < 1e300) || !(curv < 1e300)) {
        theta = 0.0;                                              // not a number, or infinite
    } else if (pq > 16.0 * noise) {
        told = true;
        theta = fmin(1.0, fmax(0.0, -lin / (2.0 * curv)));
    } else if (delta > g.tol * (g.quad * o + fabs(dreg))) {
        theta = 0.0;                                              // a rise that rounding does not explain
    }
    st->last_delta = delta;
    st->last_theta = theta;
    st->dreg = 0.0;
    st->arrived = 0;
    st->steps_pass = 0;
    const bool damp = theta < 0.55;
    // credit towards a larger bound: a pass that was seen to step about right -- or, while no pass
    // has ever been damped, any pass (the halved bound of the start is then only a precaution)
    const bool credit = told ? theta >= 0.8 : st->trips == 0;
    if (!damp) theta = 1.0;                                       // (past 1/2 the full step still descends)
    if (theta > 0.0) st->steps_kept += steps;
    uint32_t shift = st->shift;
    const uint32_t need = st->need ? st->need : 4u;
    if (damp) {
        const uint32_t trips = st->trips + 1;
        st->trips = trips;
        __hip_atomic_store(host_words, trips, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (shift < 30) ++shift;
        st->clean = 0;
        st->need = need < 1024u ? 2u * need : need;
    } else if (credit && shift > 0 && ++st->clean >= need) {
        --shift;
        st->clean = 0;
    }
    if (shift != st->shift) {
        __hip_atomic_store(&st->shift, shift, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(host_words + 1, shift, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return theta;
}

__device__ __forceinline__ void guard_finish(const MergeGuard &g, const CdArgs &a, float *v, int64_t d)
{
    // (entered by every thread of the last workgroup to finish; all other workgroups' device-scope
    // writes of v, snap and their partial sums were complete before their arrival was counted)
    __shared__ double red[3][16];
    __shared__ double verdict;
    const int nb = gridDim.x;
    double so = 0.0, sd = 0.0, sq = 0.0;
    for (int i = threadIdx.x; i < nb; i += 1024) {
        so += __hip_atomic_load(&g.part[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sd += __hip_atomic_load(&g.part[nb + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sq += __hip_atomic_load(&g.part[2 * nb + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    so = wave_sum(so);
    sd = wave_sum(sd);
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = so; red[1][threadIdx.x >> 6] = sd; red[2][threadIdx.x >> 6] = sq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double o = 0.0, pd = 0.0, pq = 0.0;
        for (int w = 0; w < 16; ++w) { o += red[0][w]; pd += red[1][w]; pq += red[2][w]; }
        const double dreg = __hip_atomic_load(&g.st->dreg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long steps = __hip_atomic_load(&g.st->steps_pass, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        verdict = guard_verdict(g.st, g.host_trips, g, 1.0 / (double)d, o, pd, pq, dreg, steps);
    }
    __syncthreads();
    const float theta = (float)verdict;
    if (theta >= 1.0f) return;
    for (int64_t i = threadIdx.x; i < d; i += 1024) {
        const float was = __hip_atomic_load(&g.snap[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float is = __hip_atomic_load(&v[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&v[i], theta > 0.0f ? fmaf(theta, is - was, was) : was, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int64_t t = threadIdx.x; t < a.count; t += 1024) {
        const uint64_t e = g.alpha_old[t];
        if ((uint32_t)(e >> 32) != g.stamp) continue;
        const int64_t j = coord_at(a, t);
        if (j < 0) continue;
        const float was = __uint_as_float((uint32_t)e);
        a.alpha[j] = theta > 0.0f ? fmaf(theta, a.alpha[j] - was, was) : was;
    }
}

// CH = 16 is the same for short vectors, where 256 elements per workgroup would leave most of the
// device idle: a workgroup owns 16 chunks, and the four quarters of a wavefront read four workers'
// buffers at a time (their sums meet in wavefront 0 by three more shuffles).
template <int CH>
__global__ __launch_bounds__(1024) void merge_workers_kernel(float *v, int64_t d, const float *dv,
                                                             int64_t dv_stride, const int32_t *dirty,
                                                             int nworkers, const MergeGuard g, const CdArgs a)
{
    constexpr int SUBS = 64 / CH;                                  // workers per wavefront load
    __shared__ float4 part[16][64];
    __shared__ int is_last;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int sub = lane / CH;
    const int64_t k4 = (int64_t)blockIdx.x * CH + lane % CH;       // chunk of four elements
    const bool in = 4 * k4 < d;
    const float4 *p = reinterpret_cast<const float4 *>(dv) + (in ? k4 : 0);
    const int64_t stride4 = dv_stride >> 2;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    auto add = [](float4 &x, const float4 y) { x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w; };
    constexpr int STEP = 16 * SUBS;
    int wk = w * SUBS + sub;
    for (; wk + STEP * 7 < nworkers; wk += STEP * 8) {
        float4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            t[u] = dirty[wk + STEP * u] ? p[(int64_t)(wk + STEP * u) * stride4] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 8; ++u) add(s, t[u]);
    }
    for (; wk < nworkers; wk += STEP)
        if (dirty[wk]) add(s, p[(int64_t)wk * stride4]);
    part[w][lane] = s;
    __syncthreads();
    if (w == 0) {
        double s_old = 0.0, s_lin = 0.0, s_sq = 0.0;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 16; ++u) add(t, part[u][lane]);
#pragma unroll
        for (int o = CH; o < 64; o <<= 1) {                        // the quarters hold different workers' sums
            t.x += __shfl_xor(t.x, o, 64);
            t.y += __shfl_xor(t.y, o, 64);
            t.z += __shfl_xor(t.z, o, 64);
            t.w += __shfl_xor(t.w, o, 64);
        }
        if (in && sub == 0) {
            const int64_t k = 4 * k4;
            if (!g.st) {
                if (t.x != 0.0f) v[k] += t.x;
                if (k + 1 < d && t.y != 0.0f) v[k + 1] += t.y;
                if (k + 2 < d && t.z != 0.0f) v[k + 2] += t.z;
                if (k + 3 < d && t.w != 0.0f) v[k + 3] += t.w;
            } else {
                float o[4], nw[4];
                const float tt[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool ok = k + e < d;
                    o[e] = ok ? v[k + e] : 0.0f;
                    nw[e] = o[e] + tt[e];
                    s_old += (double)o[e] * (double)o[e];
                }
                if (g.last) {
                    // against v at the start of the pass (this merge's own input if it is also the first)
                    float4 was = make_float4(o[0], o[1], o[2], o[3]);
                    if (!g.first) {
                        if (k + 3 < d) was = *reinterpret_cast<const float4 *>(g.snap + k);
                        else {
                            was.x = g.snap[k];
                            was.y = k + 1 < d ? g.snap[k + 1] : 0.0f;
                            was.z = k + 2 < d ? g.snap[k + 2] : 0.0f;
                            was.w = 0.0f;
                        }
                    }
                    const float ws[4] = {was.x, was.y, was.z, was.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const double dv_e = k + e < d ? (double)nw[e] - (double)ws[e] : 0.0;
                        s_lin += (double)ws[e] * dv_e;
                        s_sq += dv_e * dv_e;
                    }
                }
                // In the merge that ends the pass, v (and snap) go straight to device-coherent memory:
                // the workgroup that judges the pass may have to overwrite v after all others, and
                // does so without any cache-wide fence.  Whole 16-byte chunks in one store each
                // (device-scope stores of single words are partial writes to memory, eight times slower).
                const bool whole = k + 3 < d;
                if (g.last && whole) {
                    const int off = (int)(k * 4);
                    coherent_store4(__builtin_amdgcn_make_buffer_rsrc(v, 0, (int)((d >> 2) << 4), 0x00020000), off,
                                    make_float4(nw[0], nw[1], nw[2], nw[3]));
                    if (g.first)
                        coherent_store4(__builtin_amdgcn_make_buffer_rsrc(g.snap, 0, (int)((d >> 2) << 4), 0x00020000),
                                        off, make_float4(o[0], o[1], o[2], o[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (k + e >= d) continue;
                        if (g.last) {
                            __hip_atomic_store(&v[k + e], nw[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if (g.first) __hip_atomic_store(&g.snap[k + e], o[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        } else {
                            if (tt[e] != 0.0f) v[k + e] = nw[e];
                            if (g.first) g.snap[k + e] = o[e];
                        }
                    }
                }
            }
        }
        if (g.st) {
            s_old = wave_sum(s_old);
            if (g.last) {
                s_lin = wave_sum(s_lin);
                s_sq = wave_sum(s_sq);
            }
            if (lane == 0) {
                if (g.first) __hip_atomic_store(&g.part[blockIdx.x], s_old, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (g.last) {
                    __hip_atomic_store(&g.part[gridDim.x + blockIdx.x], s_lin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&g.part[2 * gridDim.x + blockIdx.x], s_sq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
    if (g.st && blockIdx.x == 0) {
        // the workers' books of this sub-pass go into the pass's totals (one workgroup per merge does
        // this, and merges follow each other, so plain arithmetic on the totals is safe; they are
        // written at device scope because another workgroup of the last merge reads them)
        __shared__ double bk[2][16];
        double dr = 0.0, st = 0.0;
        for (int i = threadIdx.x; i < nworkers; i += 1024) {
            const double2 b = g.wbook[i];
            dr += b.x;
            st += b.y;
        }
        dr = wave_sum(dr);
        st = wave_sum(st);
        if (lane == 0) { bk[0][w] = dr; bk[1][w] = st; }
        __syncthreads();
        if (threadIdx.x == 0) {
            double x = 0.0, y = 0.0;
            for (int u = 0; u < 16; ++u) { x += bk[0][u]; y += bk[1][u]; }
            __hip_atomic_store(&g.st->dreg, g.st->dreg + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&g.st->steps_pass, g.st->steps_pass + (unsigned long long)y, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (g.st && g.last) {
        // The workgroup that arrives last judges the pass.  No cache-wide fence: what one workgroup
        // writes for another (partial sums, v, snap) is written with device-scope stores, the
        // workgroup barrier lets them complete before the arrival is counted, and they are read with
        // device-scope loads.
        __syncthreads();
        if (threadIdx.x == 0)
            is_last = __hip_atomic_fetch_add(&g.st->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
        __syncthreads();
        if (is_last) guard_finish(g, a, v, d);
    }
}

// ---- concurrent, sparse: G lanes per coordinate ---------------------------------------------------
// Positions [t_begin, t_end) of the visiting order.  LIVE: the gathers of v observe the atomic
// adds of steps that finished before them (device-scope loads, served past the per-die L2); one
// launch covers the pass and a.groups bounds how many steps run without seeing each other.
// !LIVE: plain, cached gathers -- a step may miss every update made since the launch began, so
// the caller launches one sub-pass of that many coordinates at a time (kernel boundaries are what
// make the adds visible to plain loads).  Device-scope loads are the slower kind: 2e7 of them take
// longer than the 2e7 atomic adds of the same pass.
// For the sub-passes the chain of dependent round trips to memory -- order -> row -> entries -> v ->
// adds -- is cut by one: cd_csr_plan_kernel resolves order and row for the whole pass beforehand.
template <int MODEL>
__global__ __launch_bounds__(256) void cd_csr_plan_kernel(const CdArgs a, float *snap, double *part_old)
{
    if (snap) {
        // guard of the pass: keep v as it is now, and its sum of squares (one partial per workgroup)
        __shared__ double sh[4];
        double sq = 0.0;
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < a.d; i += (int64_t)gridDim.x * 256) {
            const float x = a.v[i];
            snap[i] = x;
            sq += (double)x * (double)x;
        }
        sq = wave_sum(sq);
        if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = sq;
        __syncthreads();
        if (threadIdx.x == 0) part_old[blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    }
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= a.count) return;
    const int64_t j = coord_at(a, t);
    CdPlan p;
    p.j = (int32_t)j;
    p.beg = j < 0 ? 0 : a.cv.rowptr[j];
    p.len = j < 0 ? 0 : (int32_t)(a.cv.rowptr[j + 1] - p.beg);
    p.alpha = j < 0 ? 0.0f : a.alpha[j];            // a pass visits a coordinate once: still current then
    p.q = j < 0 ? 0.0f : a.q[j];
    p.y = (MODEL == DUHL_SVM && j >= 0) ? a.target[j] : 0.0f;
    p.pad = 0.0f;
    a.plan[t] = p;
}

// The guard at the end of a sparse pass (see MergeGuard): <snap, v - snap>, ||v - snap||^2 and the
// change of the objective's terms in alpha (old values from the plan), per workgroup; the workgroup
// that finishes last judges the pass and, if it overshot, blends v and the pass's alpha_j with
// their old values.
template <int MODEL>
__global__ __launch_bounds__(1024) void cd_csr_guard_kernel(const CdArgs a, const MergeGuard g, const int nold)
{
    __shared__ double red[3][16];
    __shared__ int is_last;
    __shared__ double verdict;
    const int nb = gridDim.x;
    double sd = 0.0, sq = 0.0, dreg = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < a.d; i += (int64_t)nb * 1024) {
        const double was = (double)g.snap[i];
        const double dv = (double)a.v[i] - was;
        sd += was * dv;
        sq += dv * dv;
    }
    for (int64_t t = (int64_t)blockIdx.x * 1024 + threadIdx.x; t < a.count; t += (int64_t)nb * 1024) {
        const CdPlan p = a.plan[t];
        if (p.j >= 0) dreg += objective_term_change<MODEL>(a.mc, a.alpha[p.j], p.alpha, p.y);
    }
    sd = wave_sum(sd);
    sq = wave_sum(sq);
    dreg = wave_sum(dreg);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = sd; red[1][threadIdx.x >> 6] = sq; red[2][threadIdx.x >> 6] = dreg; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double x = 0.0, y = 0.0, z = 0.0;
        for (int w = 0; w < 16; ++w) { x += red[0][w]; y += red[1][w]; z += red[2][w]; }
        __hip_atomic_store(&g.part[nold + blockIdx.x], x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&g.part[nold + nb + blockIdx.x], y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&g.part[nold + 2 * nb + blockIdx.x], z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();                                   // (the stores have completed)
    if (threadIdx.x == 0)
        is_last = __hip_atomic_fetch_add(&g.st->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)nb - 1;
    __syncthreads();
    if (!is_last) return;
    double so = 0.0, dr = 0.0;
    sd = sq = 0.0;
    for (int i = threadIdx.x; i < nold; i += 1024) so += g.part[i];          // written by an earlier kernel
    for (int i = threadIdx.x; i < nb; i += 1024) {
        sd += __hip_atomic_load(&g.part[nold + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sq += __hip_atomic_load(&g.part[nold + nb + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        dr += __hip_atomic_load(&g.part[nold + 2 * nb + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    so = wave_sum(so);
    sd = wave_sum(sd);
    sq = wave_sum(sq);
    dr = wave_sum(dr);
    __shared__ double fin[4][16];
    if ((threadIdx.x & 63) == 0) {
        fin[0][threadIdx.x >> 6] = so;
        fin[1][threadIdx.x >> 6] = sd;
        fin[2][threadIdx.x >> 6] = sq;
        fin[3][threadIdx.x >> 6] = dr;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double o = 0.0, pd = 0.0, pq = 0.0, r = 0.0;
        for (int w = 0; w < 16; ++w) { o += fin[0][w]; pd += fin[1][w]; pq += fin[2][w]; r += fin[3][w]; }
        // (steps of a sparse pass: the positions of the plan, less the share of the groups that sat out)
        const int e = (int)g.st->shift - g.host_shift;
        verdict = guard_verdict(g.st, g.host_trips, g, 1.0 / (double)a.d, o, pd, pq, r,
                                (unsigned long long)(a.count >> (e > 0 ? e : 0)));
    }
    __syncthreads();
    const float theta = (float)verdict;
    if (theta >= 1.0f) return;
    // (other workgroups of this kernel only read v and alpha, and are done)
    for (int64_t i = threadIdx.x; i < a.d; i += 1024) {
        const float was = g.snap[i];
        a.v[i] = theta > 0.0f ? fmaf(theta, a.v[i] - was, was) : was;
    }
    for (int64_t t = threadIdx.x; t < a.count; t += 1024) {
        const CdPlan p = a.plan[t];
        if (p.j >= 0) a.alpha[p.j] = theta > 0.0f ? fmaf(theta, a.alpha[p.j] - p.alpha, p.alpha) : p.alpha;
    }
}

// One exact step on the coordinate at position t of the visiting order, by a group of G lanes.
template <int MODEL, int G, bool LIVE>
__device__ __forceinline__ void csr_step(const CdArgs &a, int64_t t, int sub, const CdPlan &p)
{
    int64_t j, beg, end;
    float old, qj, y;
    if (LIVE) {
        j = coord_at(a, t);
        if (j < 0) return;
        beg = a.cv.rowptr[j];
        end = a.cv.rowptr[j + 1];
        // the scalars of the step are requested now, not after the dot product: one round
        // trip to memory less
        old = a.alpha[j];
        qj = a.q[j];
        y = MODEL == DUHL_SVM ? a.target[j] : 0.0f;
    } else {
        j = p.j;
        if (j < 0) return;
        beg = p.beg;
        end = p.beg + p.len;
        old = p.alpha;
        qj = p.q;
        y = p.y;
    }
    float acc = 0.0f;
    // index/value loads of a batch first, then the gathers that depend on them: K gathers
    // of v in flight per lane
    constexpr int K = 8;
    int32_t ci[K];                                     // (the row's first batch stays in registers)
    float xv[K];
    for (int64_t e0 = beg + sub; e0 < end; e0 += (int64_t)G * K) {
        int32_t cj[K];
        float xj[K], vv[K];
#pragma unroll
        for (int u = 0; u < K; ++u) {
            const int64_t e = e0 + (int64_t)u * G;
            const bool in = e < end;
            cj[u] = in ? a.cv.colidx[e] : 0;
            xj[u] = in ? a.cv.val[e] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < K; ++u) vv[u] = LIVE ? live_load(a.v + cj[u]) : a.v[cj[u]];
#pragma unroll
        for (int u = 0; u < K; ++u) acc = fmaf(xj[u], vv[u], acc);
        if (e0 == beg + sub) {
#pragma unroll
            for (int u = 0; u < K; ++u) {
                ci[u] = cj[u];
                xv[u] = xj[u];
            }
        }
    }
    const float c = group_sum<G>(acc);
    const float now = cd_new_alpha<MODEL>(a.mc, c, old, qj, y);
    const float delta = now - old;
    if (delta != 0.0f) {
#pragma unroll
        for (int u = 0; u < K; ++u)                     // padding of the batch has value 0: skipped
            if (beg + sub + (int64_t)u * G < end) live_add(a.v + ci[u], xv[u] * delta);
        for (int64_t e = beg + sub + (int64_t)G * K; e < end; e += G)
            live_add(a.v + a.cv.colidx[e], a.cv.val[e] * delta);
        if (sub == 0) a.alpha[j] = now;
    }
}

template <int MODEL, int G, bool LIVE>
__global__ __launch_bounds__(256) void cd_csr_async_kernel(const CdArgs a, const int64_t t_begin, const int64_t t_end,
                                                           const GuardState *guard, const int host_shift)
{
    const int sub = threadIdx.x % G;
    const int64_t ngroups = a.groups;              // idle groups of the last workgroup leave at once
    const int64_t first = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
    if (first >= ngroups) return;
    // (the first plan record is asked for before the guard's word, so that the two loads overlap)
    int64_t t = t_begin + first;
    CdPlan p{};
    if (!LIVE && t < t_end) p = a.plan[t];
    if (guard_sits_out(guard, host_shift, first)) return;
    for (; t < t_end; t += ngroups) {
        if (!LIVE && t != t_begin + first) p = a.plan[t];
        csr_step<MODEL, G, LIVE>(a, t, sub, p);
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
        if (j < 0) continue;
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
        if (j < 0) continue;
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

// The host's view of the guard before it enqueues a pass: how many halvings of the library's bound on
// concurrent steps the device asks for, read as it stands in host-visible memory -- no wait, so it
// may lag behind the device by the passes in flight (what is missing the kernels make up for by
// letting workers sit out, see guard_sits_out).
void guard_update(duhl_ctx *c)
{
    if (!c->h_trips) return;
    // While the bound is halved -- after set_data, or after a pass was undone -- the host does not run
    // more than two passes ahead of the device: it waits for the pass before the last one, and so
    // learns within two passes that the guard has doubled the bound again.  With the full bound in
    // force nothing is waited for.
    const int slot = (int)(c->guard_passes & 1);         // where the pass before the last one left its event
    if (c->guard_shift > 0 && c->guard_passes >= 2 && c->ev_pass_no[slot] == c->guard_passes - 1)
        (void)hipEventSynchronize(c->ev_pass[slot]);
    c->guard_shift = (int)static_cast<volatile uint32_t *>(c->h_trips)[1];
}

// Marks the end of a guarded pass on the compute stream (see guard_update) -- only while the bound is
// halved: an event between two passes costs about as much as a kernel launch.
void guard_mark_pass(duhl_ctx *c)
{
    if (!c->guard) return;
    const int slot = (int)(c->guard_passes & 1);
    if (c->guard_shift > 0) {
        hipEvent_t &ev = c->ev_pass[slot];
        if (!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) ev = nullptr;
        if (ev && hipEventRecord(ev, c->compute) == hipSuccess) c->ev_pass_no[slot] = c->guard_passes + 1;
    }
    c->guard_passes++;
}

// Buffers of the guard (first use), and its arguments for a pass over `count` positions that needs
// `nparts` per-workgroup partial sums.  st == nullptr in the result: no guard.
hipError_t guard_prepare(duhl_ctx *c, int64_t count, int64_t nparts, MergeGuard *g, bool want_alpha_old = true)
{
    *g = MergeGuard{};
    if (!c->cd_guard) return hipSuccess;
    hipError_t e = hipSuccess;
    if (!c->guard) {
        e = hipMalloc(reinterpret_cast<void **>(&c->guard), sizeof(GuardState));
        if (e == hipSuccess)
            e = launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(c->guard), sizeof(GuardState) / 4, 0);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->snap_pass_v), sizeof(float) * (size_t)(c->d + 4));
        if (e == hipSuccess)
            e = hipHostMalloc(reinterpret_cast<void **>(&c->h_trips), 2 * sizeof(uint32_t), hipHostMallocMapped);
        if (e == hipSuccess) e = launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->guard->shift), 1, c->guard_shift);
        if (e == hipSuccess) {
            c->h_trips[0] = 0;
            c->h_trips[1] = (uint32_t)c->guard_shift;
            e = hipHostGetDevicePointer(reinterpret_cast<void **>(&c->h_trips_dev), c->h_trips, 0);
        }
        if (e != hipSuccess) return e;
    }
    if (nparts > c->guard_part_cap) {
        (void)hipFree(c->guard_part);
        c->guard_part = nullptr;
        c->guard_part_cap = 0;
        e = hipMalloc(reinterpret_cast<void **>(&c->guard_part), sizeof(double) * (size_t)nparts);
        if (e != hipSuccess) return e;
        c->guard_part_cap = nparts;
    }
    if (want_alpha_old && count > c->alpha_old_cap) {
        (void)hipFree(c->alpha_old);
        c->alpha_old = nullptr;
        c->alpha_old_cap = 0;
        e = hipMalloc(reinterpret_cast<void **>(&c->alpha_old), sizeof(uint64_t) * (size_t)count);
        if (e == hipSuccess) e = launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(c->alpha_old), 2 * count, 0);
        if (e != hipSuccess) return e;
        c->alpha_old_cap = count;
    }
    g->stamp = ++c->guard_stamp;
    if (g->stamp == 0) g->stamp = ++c->guard_stamp;      // 0 marks entries that were never written
    g->st = c->guard;
    g->part = c->guard_part;
    g->snap = c->snap_pass_v;
    g->alpha_old = c->alpha_old;
    g->host_trips = c->h_trips_dev;
    g->quad = quad_scale(c->mc);
    g->tol = c->guard_tol;
    // a dense step rounds every element of the worker's v once; a sparse one the elements of its row
    g->per_step = c->sparse && c->n > 0 && c->d > 0 ? (double)c->nnz / ((double)c->n * (double)c->d) : 1.0;
    g->host_shift = c->guard_shift;
    if (want_alpha_old && !c->guard_wbook) {               // dense workers: one slot each
        e = hipMalloc(reinterpret_cast<void **>(&c->guard_wbook), sizeof(double2) * (size_t)(c->dv_workers + 16));
        if (e != hipSuccess) return e;
    }
    g->wbook = c->guard_wbook;
    return hipSuccess;
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
hipError_t launch_atomic_dense_t(duhl_ctx *c, const CdArgs &a, int inflight, bool vec)
{
    constexpr int BLOCK = T == 64 ? 256 : T;
    constexpr int PER = BLOCK / T;
    if (inflight < 1) inflight = 1;
    const int64_t grid = (inflight + PER - 1) / PER;
    CdArgs b = a;
    b.groups = inflight;
    if (vec)
        hipLaunchKernelGGL((cd_dense_atomic_kernel<MODEL, T, NREG, true>), dim3(grid), dim3(BLOCK), 0,
                           c->compute, b);
    else
        hipLaunchKernelGGL((cd_dense_atomic_kernel<MODEL, T, 1, false>), dim3(grid), dim3(BLOCK), 0,
                           c->compute, b);
    return hipGetLastError();
}

template <int MODEL, int T>
hipError_t launch_atomic_dense_n(duhl_ctx *c, const CdArgs &a, int inflight, bool vec)
{
    const int64_t chunks = ((c->d >> 2) + T - 1) / T;   // float4 per thread to hold a column
    if (chunks <= 1) return launch_atomic_dense_t<MODEL, T, 1>(c, a, inflight, vec);
    if (chunks <= 2) return launch_atomic_dense_t<MODEL, T, 2>(c, a, inflight, vec);
    if (chunks <= 4) return launch_atomic_dense_t<MODEL, T, 4>(c, a, inflight, vec);
    if (chunks <= 8) return launch_atomic_dense_t<MODEL, T, 8>(c, a, inflight, vec);
    if (chunks <= 13) return launch_atomic_dense_t<MODEL, T, 13>(c, a, inflight, vec);
    return launch_atomic_dense_t<MODEL, T, 16>(c, a, inflight, vec);
}

int threads_per_coordinate(const duhl_ctx *c)
{
    if (c->cd_threads == 64 || c->cd_threads == 256 || c->cd_threads == 1024) return c->cd_threads;
    if (c->d <= 2048) return 64;
    if (c->d <= 13312) return 256;
    return 1024;
}

// Coordinates that may be solved without seeing each other.  The caller's bound if given.
// Otherwise from the data: exact steps taken concurrently on L unit-norm columns behave like a
// block-Jacobi step, governed by sigma(L), the largest eigenvalue of the block's Gram matrix.
// sigma(L) is estimated as (1 + sqrt(L/d))^2, the value for uncorrelated columns, plus
// (L - 1) * mean_corr, the rank-one part that a common direction of the columns adds (mean_corr
// is measured on a column sample when the data are set).  While sigma(L) <= 2 the concurrent
// step contracts, so a whole pass may be one group (wide rows, few selected columns).  Past
// that point 2 * count / sigma(count), and never more than a quarter of the pass, worked on
// every workload here (each worker still sees its own earlier steps); non-negative sparse rows,
// whose mean correlation is ~1e-3, diverge with four times as many concurrent steps.
int64_t inflight_limit(const duhl_ctx *c, int64_t count, int max_inflight)
{
    int64_t lim;
    if (max_inflight > 0) {
        lim = max_inflight;                              // the caller's bound, halved like the library's own
        lim >>= c->guard_shift < 40 ? c->guard_shift : 40;
    } else {
        // Two estimates, the larger wins.  (i) The largest group L whose block-Jacobi step is
        // still a contraction: sigma(L) = (1 + sqrt(L/d))^2 + (L - 1) * mean cosine <= 2 (the
        // first term is the spectral norm of an L-column Gram block of near-orthogonal unit
        // columns, the second the shift a common direction adds).  (ii) The looser empirical
        // rule 2 * count / sigma(count), never more than a quarter of the pass.
        auto sigma = [&](double L) {
            const double r = 1.0 + std::sqrt(L / (double)c->d);
            return r * r + (L - 1.0) * c->mean_corr;
        };
        int64_t lo = 1, hi = count;                      // sigma is increasing in L
        if (sigma((double)count) <= 2.0) lo = count;
        while (hi - lo > 1) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (sigma((double)mid) <= 2.0) lo = mid; else hi = mid;
        }
        int64_t loose = (int64_t)(2.0 * (double)count / sigma((double)count));
        if (loose > count / 4) loose = count / 4;
        lim = lo > loose ? lo : loose;
        // every pass that the guard had to undo halves the bound; four passes in a row that it let
        // stand double it again (see guard_update)
        lim >>= c->guard_shift < 40 ? c->guard_shift : 40;
        if (lim < 1) lim = 1;
        // equal sub-passes rather than a short last one
        if (lim >= 1 && lim < count) {
            const int64_t S = (count + lim - 1) / lim;
            lim = (count + S - 1) / S;
        }
    }
    if (lim < 1) lim = 1;
    return lim < count ? lim : count;
}

template <int MODEL>
hipError_t launch_atomic(duhl_ctx *c, const CdArgs &a, int max_inflight, bool vec)
{
    if (c->sparse) {
        const int64_t avg = c->n > 0 ? c->nnz / c->n : 0;
        const int G = avg > 256 ? 64 : 16;
        const int64_t cap = (int64_t)c->num_cu * 8 * (256 / G);
        int64_t inflight = inflight_limit(c, a.count, max_inflight);
        if (inflight > cap) inflight = cap;
        const int64_t grid = (inflight + 256 / G - 1) / (256 / G);
        CdArgs b = a;
        b.groups = inflight;
        if (G == 64)
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 64, true>), dim3(grid), dim3(256), 0, c->compute, b,
                               (int64_t)0, a.count, (const GuardState *)nullptr, 0);
        else
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 16, true>), dim3(grid), dim3(256), 0, c->compute, b,
                               (int64_t)0, a.count, (const GuardState *)nullptr, 0);
        return hipGetLastError();
    }
    const int T = threads_per_coordinate(c);
    const int64_t cap = (int64_t)c->num_cu * (2048 / T);
    int64_t inflight = inflight_limit(c, a.count, max_inflight);
    if (inflight > cap) inflight = cap;
    if (T == 64) return launch_atomic_dense_n<MODEL, 64>(c, a, (int)inflight, vec);
    if (T == 256) return launch_atomic_dense_n<MODEL, 256>(c, a, (int)inflight, vec);
    return launch_atomic_dense_n<MODEL, 1024>(c, a, (int)inflight, vec);
}

// Sparse data, mode ASYNC: sub-passes of `inflight` coordinates, one launch each, all of a
// sub-pass's steps concurrent and reading v as the previous sub-passes left it (or fresher).
template <int MODEL>
hipError_t launch_csr_subpasses(duhl_ctx *c, const CdArgs &a, int max_inflight)
{
    const int64_t avg = c->n > 0 ? c->nnz / c->n : 0;
    const int G = avg > 256 ? 64 : 16;
    const int64_t inflight = inflight_limit(c, a.count, max_inflight);
    const int64_t cap = (int64_t)c->num_cu * 8 * (256 / G);      // groups that fit the device at once
    if (a.count > c->cd_plan_cap) {
        (void)hipFree(c->cd_plan);
        c->cd_plan = nullptr;
        c->cd_plan_cap = 0;
        const hipError_t e = hipMalloc(&c->cd_plan, (size_t)a.count * sizeof(CdPlan));
        if (e != hipSuccess) return e;
        c->cd_plan_cap = a.count;
    }
    CdArgs b = a;
    b.plan = static_cast<CdPlan *>(c->cd_plan);
    // guard: the plan kernel also keeps v and its sum of squares, a last kernel judges the pass
    const int64_t plan_blocks = (a.count + 255) / 256;
    int64_t end_blocks = ((a.d > a.count ? a.d : a.count) + 1023) / 1024;
    if (end_blocks > 256) end_blocks = 256;
    if (end_blocks < 1) end_blocks = 1;
    MergeGuard g;
    const hipError_t ge = guard_prepare(c, a.count, plan_blocks + 3 * end_blocks, &g, false);
    if (ge != hipSuccess) return ge;
    hipLaunchKernelGGL(cd_csr_plan_kernel<MODEL>, dim3(plan_blocks), dim3(256), 0, c->compute, b,
                       g.st ? g.snap : nullptr, g.part);
    b.groups = inflight < cap ? inflight : cap;
    const int64_t grid = (b.groups + 256 / G - 1) / (256 / G);
    for (int64_t t0 = 0; t0 < a.count; t0 += inflight) {
        const int64_t t1 = t0 + inflight < a.count ? t0 + inflight : a.count;
        if (G == 64)
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 64, false>), dim3(grid), dim3(256), 0, c->compute, b, t0, t1,
                               (const GuardState *)g.st, c->guard_shift);
        else
            hipLaunchKernelGGL((cd_csr_async_kernel<MODEL, 16, false>), dim3(grid), dim3(256), 0, c->compute, b, t0, t1,
                               (const GuardState *)g.st, c->guard_shift);
    }
    if (g.st)
        hipLaunchKernelGGL(cd_csr_guard_kernel<MODEL>, dim3(end_blocks), dim3(1024), 0, c->compute, b, g, (int)plan_blocks);
    return hipGetLastError();
}

// The merge takes 64 elements per workgroup instead of 256 while that still leaves compute units idle.
inline bool merge_narrow(const duhl_ctx *c) { return (c->d + 255) / 256 < c->num_cu / 2; }
inline int64_t merge_blocks(const duhl_ctx *c) { return merge_narrow(c) ? (c->d + 63) / 64 : (c->d + 255) / 256; }
inline void launch_merge(duhl_ctx *c, int64_t mblocks, int nworkers, const MergeGuard &g, const CdArgs &a)
{
    if (merge_narrow(c))
        hipLaunchKernelGGL(merge_workers_kernel<16>, dim3(mblocks), dim3(1024), 0, c->compute, a.v, c->d, c->dv,
                           c->dv_stride, c->dirty, nworkers, g, a);
    else
        hipLaunchKernelGGL(merge_workers_kernel<64>, dim3(mblocks), dim3(1024), 0, c->compute, a.v, c->d, c->dv,
                           c->dv_stride, c->dirty, nworkers, g, a);
}

template <int MODEL, int T, int NR, int NL, bool CACHE_X, bool EXT, bool XVEC>
hipError_t launch_workers_t(duhl_ctx *c, const CdArgs &a, int64_t inflight)
{
    constexpr int BLOCK = T == 64 ? 256 : T;
    constexpr int PER = BLOCK / T;
    // Workers per sub-pass: enough to fill the chip; several coordinates per worker once the
    // sub-pass is large, which keeps the private buffers a small fraction of the traffic.
    const int64_t cap = c->dv_workers;
    const int64_t mblocks = merge_blocks(c);
    MergeGuard g;
    const hipError_t ge = guard_prepare(c, a.count, 3 * mblocks, &g);
    if (ge != hipSuccess) return ge;
    for (int64_t t0 = 0; t0 < a.count; t0 += inflight) {
        const int64_t t1 = t0 + inflight < a.count ? t0 + inflight : a.count;
        const int64_t len = t1 - t0;
        int64_t workers = len >= 4 * (int64_t)c->num_cu ? len / 4 : (len < c->num_cu ? len : c->num_cu);
        if (workers > cap) workers = cap;
        const int64_t grid = (workers + PER - 1) / PER;
        g.first = t0 == 0;
        g.last = t1 == a.count;
        hipLaunchKernelGGL((cd_dense_worker_kernel<MODEL, T, NR, NL, CACHE_X, EXT, XVEC>), dim3(grid), dim3(BLOCK), 0,
                           c->compute, a, t0, t1, c->dv, c->dv_stride, c->dirty, nullptr, 0u, nullptr, 0,
                           g.st ? c->alpha_old : nullptr, g.stamp, g.st, c->guard_shift, g.wbook);
        launch_merge(c, mblocks, (int)(grid * PER), g, a);
    }
    return hipGetLastError();
}

// The same with workers of CUS workgroups each (columns too long for one compute unit to hold a
// private v and a cached column).  All workgroups of a launch must be resident at once -- partners
// wait for each other -- so there are at most as many as compute units, fewer by the workgroups of
// the column copy that may be running beside the pass.
template <int MODEL, int NR, int NL, int CUS, bool XVEC>
hipError_t launch_multi_t(duhl_ctx *c, const CdArgs &a, int64_t inflight, int64_t workers)
{
    const int64_t mblocks = merge_blocks(c);
    MergeGuard g;
    const hipError_t ge = guard_prepare(c, a.count, 3 * mblocks, &g);
    if (ge != hipSuccess) return ge;
    for (int64_t t0 = 0; t0 < a.count; t0 += inflight) {
        const int64_t t1 = t0 + inflight < a.count ? t0 + inflight : a.count;
        const int64_t per_worker = (t1 - t0 + workers - 1) / workers;
        g.first = t0 == 0;
        g.last = t1 == a.count;
        hipLaunchKernelGGL((cd_dense_worker_kernel<MODEL, 1024, NR, NL, true, false, XVEC, CUS>),
                           dim3(workers * CUS), dim3(1024), 0, c->compute, a, t0, t1, c->dv, c->dv_stride,
                           c->dirty, c->xch, c->xseq, &c->sel->cd_abort, c->cd_spin_limit,
                           g.st ? c->alpha_old : nullptr, g.stamp, g.st, c->guard_shift, g.wbook);
        c->xseq += (uint32_t)per_worker + 2u;          // sequence numbers never repeat back to back
        launch_merge(c, mblocks, (int)workers, g, a);
    }
    return hipGetLastError();
}

template <int MODEL, int CUS, bool XVEC>
hipError_t launch_multi(duhl_ctx *c, const CdArgs &a, int64_t inflight, int64_t workers, int64_t chunks)
{
    const int64_t per = (chunks + CUS - 1) / CUS;      // chunks of a column per workgroup
    if (per <= 8) return launch_multi_t<MODEL, 8, 0, CUS, XVEC>(c, a, inflight, workers);
    if (per <= 10) return launch_multi_t<MODEL, 8, 2, CUS, XVEC>(c, a, inflight, workers);
    return launch_multi_t<MODEL, 8, 5, CUS, XVEC>(c, a, inflight, workers);
}

// Dense asynchronous pass with private-v workers; false if this shape is not covered.
template <int MODEL>
bool launch_workers(duhl_ctx *c, const CdArgs &a, int max_inflight, bool vec, hipError_t *err)
{
    const int T = threads_per_coordinate(c);
    const int64_t chunks = ((c->d >> 2) + T - 1) / T;
    // 32-bit byte offsets inside a column and a sane private-buffer size bound the extended variant
    if (chunks > 25 * 64) return false;
    if (!c->dv) {                                   // private buffers, allocated on first use
        c->dv_stride = (c->d + 63) / 64 * 64;
        int64_t workers = (int64_t)c->num_cu * (T == 1024 ? 1 : (T == 256 ? 4 : 16));
        while (workers > c->num_cu && workers * c->dv_stride * 4 > (1ll << 30)) workers /= 2;
        c->dv_workers = workers;
        *err = hipMalloc(reinterpret_cast<void **>(&c->dv), (size_t)workers * c->dv_stride * 4);
        if (*err == hipSuccess) *err = hipMalloc(reinterpret_cast<void **>(&c->dirty), (size_t)(workers + 4) * 4);
        if (*err != hipSuccess) return true;
    }
    const int64_t inflight = inflight_limit(c, a.count, max_inflight);
    // Columns of 53,249 to 425,984 entries: two, four or eight compute units per worker, everything on chip
    if (T == 1024 && chunks > 13 && chunks <= 104 && c->cd_units != 1) {
        const int cus = c->cd_units == 2 || c->cd_units == 4 || c->cd_units == 8
                            ? c->cd_units : (chunks <= 26 ? 2 : (chunks <= 52 ? 4 : 8));
        const int64_t avail = c->num_cu - (c->res == DUHL_RESIDENT_HOST ? c->copy_blocks : 0);
        const int64_t workers = avail / (8 * cus) * 8;
        if (workers >= 8 && workers <= c->dv_workers && chunks <= 13 * cus) {
            if (!c->xch) {
                *err = hipMalloc(reinterpret_cast<void **>(&c->xch), (size_t)c->dv_workers * 16 * sizeof(uint64_t));
                if (*err == hipSuccess)
                    *err = hipMemsetAsync(c->xch, 0, (size_t)c->dv_workers * 16 * sizeof(uint64_t), c->compute);
                if (*err != hipSuccess) return true;
                c->xseq = 1;
            }
            if (vec)
                *err = cus == 2   ? launch_multi<MODEL, 2, true>(c, a, inflight, workers, chunks)
                       : cus == 4 ? launch_multi<MODEL, 4, true>(c, a, inflight, workers, chunks)
                                  : launch_multi<MODEL, 8, true>(c, a, inflight, workers, chunks);
            else                                        // columns start only 4-byte aligned
                *err = cus == 2   ? launch_multi<MODEL, 2, false>(c, a, inflight, workers, chunks)
                       : cus == 4 ? launch_multi<MODEL, 4, false>(c, a, inflight, workers, chunks)
                                  : launch_multi<MODEL, 8, false>(c, a, inflight, workers, chunks);
            return true;
        }
    }
    // (T, register chunks, LDS chunks, column cached?) by column length
    // vec: columns start 16-byte aligned; otherwise their loads are split into dwords
#define DUHL_W(TT, NR, NL, CX)                                                            \
    *err = vec ? launch_workers_t<MODEL, TT, NR, NL, CX, false, true>(c, a, inflight)     \
               : launch_workers_t<MODEL, TT, NR, NL, CX, false, false>(c, a, inflight)
    if (T == 64) {
        if (chunks <= 1) DUHL_W(64, 1, 0, true);
        else if (chunks <= 2) DUHL_W(64, 2, 0, true);
        else if (chunks <= 4) DUHL_W(64, 4, 0, true);
        else DUHL_W(64, 8, 0, true);
    } else if (T == 256) {
        if (chunks <= 4) DUHL_W(256, 4, 0, true);
        else if (chunks <= 8) DUHL_W(256, 8, 0, true);
        else if (chunks <= 10) DUHL_W(256, 10, 0, true);
        else DUHL_W(256, 13, 0, true);
    } else {
        if (chunks <= 4) DUHL_W(1024, 4, 0, true);
        else if (chunks <= 8) DUHL_W(1024, 8, 0, true);
        else if (chunks <= 10) DUHL_W(1024, 8, 2, true);
        else if (chunks <= 13) DUHL_W(1024, 8, 5, true);
        else if (chunks <= 16) DUHL_W(1024, 12, 4, false);
        else if (chunks <= 20) DUHL_W(1024, 14, 6, false);
        else if (chunks <= 25) DUHL_W(1024, 16, 9, false);
        else                                            // rest of the private v in the worker's buffer
            *err = vec ? launch_workers_t<MODEL, 1024, 16, 9, false, true, true>(c, a, inflight)
                       : launch_workers_t<MODEL, 1024, 16, 9, false, true, false>(c, a, inflight);
    }
#undef DUHL_W
    return true;
}

template <int MODEL>
hipError_t launch_cd_model(duhl_ctx *c, duhl_cd_mode mode, const CdArgs &a, int max_inflight)
{
    const bool vec = !c->sparse && c->a_aligned16 && (a.cv.ld % 4 == 0) && aligned16(a.v) &&
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
    if (mode == DUHL_CD_ASYNC) guard_update(c);
    if (mode == DUHL_CD_ASYNC && c->sparse) {
        const hipError_t err = launch_csr_subpasses<MODEL>(c, a, max_inflight);
        guard_mark_pass(c);
        return err;
    }
    if (mode == DUHL_CD_ASYNC) {
        hipError_t err = hipSuccess;
        if (launch_workers<MODEL>(c, a, max_inflight, vec, &err)) {
            guard_mark_pass(c);
            return err;
        }
    }
    return launch_atomic<MODEL>(c, a, max_inflight, vec);
}

}  // namespace

// The library's own bound on concurrent steps for a pass over `count` coordinates.
int64_t default_inflight(const duhl_ctx *c, int64_t count) { return inflight_limit(c, count, 0); }

hipError_t launch_cd(duhl_ctx *c, duhl_cd_mode mode, const int32_t *order, int64_t count,
                     uint64_t seed, int max_inflight)
{
    CdArgs a;
    a.cv = c->cv;
    a.mc = c->mc;
    a.d = c->d;
    a.n = c->n;
    a.groups = 1;
    a.order = order;
    a.P = c->P_cur;
    a.count = order ? count : c->m_cur;
    a.permute = (!order && mode != DUHL_CD_SEQUENTIAL) ? 1 : 0;
    a.alpha = c->alpha;
    a.v = c->v;
    a.q = c->q;
    a.target = c->target;
    a.plan = nullptr;
    a.pbits = 1;
    while ((1ll << a.pbits) < a.count) ++a.pbits;
    uint64_t s = seed ^ (0xD1B54A32D192ED03ull * (c->pass_counter + 1));
    for (int r = 0; r < 3; ++r) {
        a.pmul[r] = (uint32_t)splitmix64(s) | 1u;     // odd: invertible modulo a power of two
        a.padd[r] = (uint32_t)splitmix64(s);
    }
    if (a.count <= 0) return hipSuccess;
    if (c->model == DUHL_LASSO) return launch_cd_model<DUHL_LASSO>(c, mode, a, max_inflight);
    if (c->model == DUHL_ELASTIC_NET) return launch_cd_model<DUHL_ELASTIC_NET>(c, mode, a, max_inflight);
    return launch_cd_model<DUHL_SVM>(c, mode, a, max_inflight);
}

}  // namespace duhl
