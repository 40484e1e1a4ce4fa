// Working-set selection: the m coordinates with the largest gap-memory entries (eq. (11)/(13)),
// ties to the smaller index, listed in ascending index order; rho of eq. (7) on the way.
//
// z is turned into order-preserving 32-bit keys.  Three histogram passes (11 + 11 + 10 bits)
// find the key of the m-th largest entry exactly; a count pass and an ordered scatter then
// write the indices.  The work is 4n bytes per pass -- negligible next to a gap pass -- so the
// design goal is few launches: one kernel of at most 128 small workgroups, all resident at once,
// which meet at five device-wide barriers; serial steps are repeated by every workgroup.
// The second half plans the column swap for host residency: which selected columns are not in
// a device slot yet and which slots may be overwritten (Algorithm 2, the step that refreshes B's memory).
#include "duhl_internal.h"

namespace duhl {

namespace {

constexpr int kChunk = 2048;      // granularity of a workgroup's chunk: eight tiles of 256 entries
constexpr int kMaxGroups = 128;   // most workgroups of the selection launch: all must be resident at
                                  // once, and a barrier costs more the more of them arrive

__device__ __forceinline__ uint32_t zkey(float z)
{
    if (!(z > 0.0f) && !(z < 0.0f)) z = 0.0f;              // +0, -0 and NaN share one key
    const uint32_t b = __float_as_uint(z);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);     // unsigned order == float order
}

template <typename T>
__device__ __forceinline__ T coherent_load(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void coherent_store(T *p, T x)
{
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Barrier over all workgroups of the launch.  ctr only grows; `target` is its value once every
// workgroup has arrived at this barrier (the host hands each launch a fresh range of values).
// No cache-wide fence is paid: everything one workgroup writes for another before a barrier is
// written with agent-scope stores or atomics (coherent_store, atomicAdd) and read after it with
// agent-scope loads (coherent_load); the workgroup barriers around the arrival order them with
// the counter.  The launch has at most kMaxGroups small
// workgroups, all resident at once, so the wait is short; it is bounded all the same: after
// spin_limit polls the workgroup reports failure, and so do all others (abort flag).
__device__ __forceinline__ bool grid_sync(uint32_t *ctr, uint32_t target, uint32_t *abort_flag, int spin_limit)
{
    __shared__ int ok;
    __syncthreads();                                     // this workgroup's stores have completed
    if (threadIdx.x == 0) {
        bool good = true;
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while ((int32_t)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            ++spins;
            if (spins > spin_limit ||
                ((spins & 255) == 0 &&
                 __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                good = false;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!good) __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = good ? 1 : 0;
    }
    __syncthreads();
    return ok != 0;
}

struct SelectArgs {
    const float *keys;     // what is ranked (z, or the scores of another rule)
    const float *zval;     // the gap memory, for the sums of eq. (7)
    int64_t n, m;
    int chunk;             // entries per workgroup, a multiple of 2048
    SelectState *st;
    uint32_t *blk_gt, *blk_eq;
    int32_t *P, *P_out;
    double *partials, *scalars;
    uint32_t bar_base;     // value of st->barrier before this launch
    int spin_limit;
};

// f(i, key value) for every position of this workgroup's chunk, the same number of calls in
// every thread (positions past n included; f checks).  KPT > 0: the chunk is KPT entries per
// thread and they are in registers (kreg), read once for all passes of the kernel; KPT == 0: a
// chunk of any length, read again each time, eight loads per thread in flight.
template <int KPT, typename F>
__device__ __forceinline__ void for_each_key(const SelectArgs &a, const float (&kreg)[KPT > 0 ? KPT : 1], F &&f)
{
    const int64_t base = (int64_t)blockIdx.x * a.chunk;
    if (KPT > 0) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) f(base + q * 256 + threadIdx.x, kreg[q]);
    } else {
        for (int it0 = 0; it0 < a.chunk / 256; it0 += 8) {
            float ki[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t i = base + (it0 + u) * 256 + threadIdx.x;
                ki[u] = i < a.n ? a.keys[i] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) f(base + (it0 + u) * 256 + threadIdx.x, ki[u]);
        }
    }
}

// Histogram of one digit of the keys of this workgroup's chunk (those whose higher digits equal
// `prefix`), flushed into the device-wide histogram.  Pass 0 also adds up the gap memory over the
// chunk (the keys themselves when the gaps are what is ranked).
template <int PASS, int KPT>
__device__ __forceinline__ void hist_pass(const SelectArgs &a, const float (&kreg)[KPT > 0 ? KPT : 1],
                                          uint32_t prefix, uint32_t *hist, double *zsum)
{
    constexpr int kBits = PASS == 2 ? 10 : 11;
    constexpr int kShift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
    constexpr int kBins = 1 << kBits;
    for (int i = threadIdx.x; i < kBins; i += 256) hist[i] = 0;
    __syncthreads();
    const bool own = a.zval == a.keys;
    double sum = 0.0;
    for_each_key<KPT>(a, kreg, [&](int64_t i, float kf) {
        if (i >= a.n) return;
        const uint32_t key = zkey(kf);
        if (PASS == 0 && own) sum += (double)kf;
        if (PASS == 0 || (key >> (kShift + kBits)) == prefix)
            atomicAdd(&hist[(key >> kShift) & (kBins - 1)], 1u);
    });
    if (PASS == 0 && !own) {                             // another rule's scores are ranked
        const int64_t base = (int64_t)blockIdx.x * a.chunk;
        for (int it0 = 0; it0 < a.chunk / 256; it0 += 8) {
            float zv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t i = base + (it0 + u) * 256 + threadIdx.x;
                zv[u] = i < a.n ? a.zval[i] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += (double)zv[u];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += 256)
        if (hist[i]) atomicAdd(&a.st->hist[PASS][i], hist[i]);
    if (PASS == 0) *zsum = sum;
}

// From the complete device-wide histogram of a pass: the digit that holds the `need`-th largest
// entry and how many entries of that bin are still needed.  Every workgroup computes this for
// itself (same inputs, same result), which saves a second barrier per pass.
template <int PASS>
__device__ __forceinline__ void find_digit(const SelectArgs &a, uint32_t &prefix, uint32_t &need,
                                           uint32_t *tsum, uint32_t *found)
{
    constexpr int kBits = PASS == 2 ? 10 : 11;
    constexpr int kBins = 1 << kBits;
    constexpr int kPer = kBins / 256;                    // consecutive bins per thread
    uint32_t mine[kPer], total = 0;
#pragma unroll
    for (int b = 0; b < kPer; ++b) {
        mine[b] = coherent_load(&a.st->hist[PASS][threadIdx.x * kPer + b]);
        total += mine[b];
    }
    // entries in bins above this thread's range: a suffix sum over the 256 threads, inside each
    // wavefront by shuffles, across the four wavefronts through tsum[0..3]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t incl = total;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_down(incl, o, kWave);
        if (lane + o < 64) incl += y;
    }
    if (lane == 0) tsum[w] = incl;
    __syncthreads();
    uint32_t above = incl - total;
    for (int q = w + 1; q < 4; ++q) above += tsum[q];
    if (above < need && need <= above + total) {
        uint32_t acc = above;
#pragma unroll
        for (int b = kPer - 1; b >= 0; --b) {
            if (acc < need && need <= acc + mine[b]) {
                found[0] = (prefix << kBits) | (uint32_t)(threadIdx.x * kPer + b);
                found[1] = need - acc;                   // still to take from that bin
            }
            acc += mine[b];
        }
    }
    __syncthreads();
    prefix = found[0];
    need = found[1];
    __syncthreads();
}

__device__ __forceinline__ double block_sum_partials(const double *partials, int count, double *dsh)
{
    double s = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) s += coherent_load(&partials[i]);
    s = wave_sum(s);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) dsh[threadIdx.x >> 6] = s;
    __syncthreads();
    return (dsh[0] + dsh[1]) + (dsh[2] + dsh[3]);
}

// The whole selection in one launch: three histogram passes find the key of the m-th largest
// entry, then a count per chunk and an ordered scatter write the indices.  Workgroups meet at five
// barriers; each owns one chunk of consecutive entries throughout.
template <int KPT>
__global__ __launch_bounds__(256) void select_fused_kernel(const SelectArgs a)
{
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t tsum[256];
    __shared__ uint32_t found[2];
    __shared__ uint32_t wg[4], we[4];
    __shared__ uint32_t tg2[2][4], te2[2][4];            // the scatter's per-tile counts, two tiles deep
    __shared__ double dsh[4];
    SelectState *st = a.st;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t G = gridDim.x;
    uint32_t bar = a.bar_base;
    uint32_t *ctr = &st->barrier;
    // the chunk's keys, requested before anything else (they arrive during the first barrier)
    float kreg[KPT > 0 ? KPT : 1];
    if (KPT > 0) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            const int64_t i = (int64_t)blockIdx.x * a.chunk + q * 256 + threadIdx.x;
            kreg[q] = i < a.n ? a.keys[i] : 0.0f;
        }
    }

    // -- the device-wide histograms are clean: the previous launch left them so (see below)
    if (blockIdx.x == 0 && threadIdx.x == 0) {           // (read by the kernels after this one)
        st->n_fill = 0;
        st->n_evict = 0;
    }

    // -- the key of the m-th largest entry, digit by digit
    uint32_t prefix = 0, need = (uint32_t)a.m;
    double zsum = 0.0;
    hist_pass<0, KPT>(a, kreg, prefix, hist, &zsum);
    zsum = wave_sum(zsum);
    if (lane == 0) dsh[w] = zsum;
    __syncthreads();
    if (threadIdx.x == 0) coherent_store(&a.partials[blockIdx.x], (dsh[0] + dsh[1]) + (dsh[2] + dsh[3]));
    bar += G;
    if (!grid_sync(ctr, bar, &st->cd_abort, a.spin_limit)) return;
    find_digit<0>(a, prefix, need, tsum, found);
    double all = 0.0;
    if (blockIdx.x == 0) {
        all = block_sum_partials(a.partials, (int)G, dsh);
        if (threadIdx.x == 0) a.scalars[S_SUM_ALL] = all;
    }
    hist_pass<1, KPT>(a, kreg, prefix, hist, nullptr);
    bar += G;
    if (!grid_sync(ctr, bar, &st->cd_abort, a.spin_limit)) return;
    find_digit<1>(a, prefix, need, tsum, found);
    hist_pass<2, KPT>(a, kreg, prefix, hist, nullptr);
    bar += G;
    if (!grid_sync(ctr, bar, &st->cd_abort, a.spin_limit)) return;
    find_digit<2>(a, prefix, need, tsum, found);
    const uint32_t thr = prefix, take_eq = need;         // full key; entries equal to it still to take
    if (blockIdx.x == 0 && threadIdx.x == 0) st->thr_key = thr;

    // -- per chunk: entries above the key, entries equal to it
    {
        uint32_t g = 0, e = 0;
        for_each_key<KPT>(a, kreg, [&](int64_t i, float kf) {
            const uint32_t key = zkey(kf);
            g += i < a.n && key > thr;
            e += i < a.n && key == thr;
        });
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            g += __shfl_xor(g, o, kWave);
            e += __shfl_xor(e, o, kWave);
        }
        if (lane == 0) { wg[w] = g; we[w] = e; }
        __syncthreads();
        if (threadIdx.x == 0) {
            coherent_store(&a.blk_gt[blockIdx.x], wg[0] + wg[1] + wg[2] + wg[3]);
            coherent_store(&a.blk_eq[blockIdx.x], we[0] + we[1] + we[2] + we[3]);
        }
    }
    bar += G;
    if (!grid_sync(ctr, bar, &st->cd_abort, a.spin_limit)) return;
    // every workgroup is through with the histograms: clean them for the next launch (which
    // saves it a barrier; the data are set with clean ones, and set again after a failed barrier)
    for (int i = blockIdx.x * 256 + threadIdx.x; i < 3 * 2048; i += G * 256)
        coherent_store(&st->hist[0][0] + i, 0u);
    // entries of both kinds in the chunks before this one (G <= kMaxGroups <= 256: one per thread)
    uint32_t gt_before = 0, eq_before = 0;
    {
        uint32_t g = 0, e = 0;
        if (threadIdx.x < blockIdx.x) {
            g = coherent_load(&a.blk_gt[threadIdx.x]);
            e = coherent_load(&a.blk_eq[threadIdx.x]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            g += __shfl_xor(g, o, kWave);
            e += __shfl_xor(e, o, kWave);
        }
        __syncthreads();
        if (lane == 0) { wg[w] = g; we[w] = e; }
        __syncthreads();
        gt_before = wg[0] + wg[1] + wg[2] + wg[3];
        eq_before = we[0] + we[1] + we[2] + we[3];
        __syncthreads();
    }

    // -- ordered scatter: entry i goes to position (#selected entries with a smaller index)
    // (the counts of consecutive tiles alternate between two buffers, so one barrier per tile
    // is enough: a buffer is rewritten two tiles later, with the next tile's barrier in between)
    double ssel = 0.0;
    const bool own = a.zval == a.keys;
    int tile = 0;
    for_each_key<KPT>(a, kreg, [&](int64_t i, float kf) {
        uint32_t *cg = tg2[tile & 1], *ce = te2[tile & 1];
        ++tile;
        bool g = false, e = false;
        if (i < a.n) {
            const uint32_t key = zkey(kf);
            g = key > thr;
            e = key == thr;
        }
        const unsigned long long mg = __ballot(g), me = __ballot(e);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (lane == 0) { cg[w] = __popcll(mg); ce[w] = __popcll(me); }
        __syncthreads();
        uint32_t og = gt_before + __popcll(mg & below), oe = eq_before + __popcll(me & below);
        uint32_t tg = 0, te = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q < w) { og += cg[q]; oe += ce[q]; }
            tg += cg[q];
            te += ce[q];
        }
        if (g || (e && oe < take_eq)) {
            const uint32_t pos = og + (oe < take_eq ? oe : take_eq);
            a.P[pos] = (int32_t)i;
            if (a.P_out) a.P_out[pos] = (int32_t)i;
            ssel += own ? (double)kf : (double)a.zval[i];
        }
        gt_before += tg;
        eq_before += te;
    });
    ssel = wave_sum(ssel);
    if (lane == 0) dsh[w] = ssel;
    __syncthreads();
    if (threadIdx.x == 0) coherent_store(&a.partials[blockIdx.x], (dsh[0] + dsh[1]) + (dsh[2] + dsh[3]));
    bar += G;
    if (!grid_sync(ctr, bar, &st->cd_abort, a.spin_limit)) return;
    if (blockIdx.x == 0) {
        const double sel = block_sum_partials(a.partials, (int)G, dsh);
        if (threadIdx.x == 0) {
            a.scalars[S_SUM_SEL] = sel;
            // eq. (7): (mean of z over P) / (mean of z over all coordinates)
            a.scalars[S_RHO] = all > 0.0 ? (sel / (double)a.m) / (all / (double)a.n) : 1.0;
        }
    }
}

// ---- other selection rules, as scores fed to the same top-m machinery ---------------------------
// Uniformly random subset (the random reference scheme of Section 5.1): score = a hash of
// (seed, i) mapped to a positive float; the m largest scores are a uniform sample.  Contiguous block (the
// sequential reference scheme of Section 5.2): score 1 on {start + k mod n, k < m}, else 0.
__global__ void score_random_kernel(float *score, int64_t n, uint64_t seed)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t x = seed + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1);
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    x ^= x >> 31;
    // one of the 254 * 2^23 positive normal floats, chosen uniformly by bit pattern (order is all that
    // matters): almost 31 random bits, so even for n ~ 1e6 equal scores -- which fall to the smaller
    // index -- are rare enough (n^2 / 2^32 pairs) not to bias the subset
    const uint32_t pick = (uint32_t)__umul64hi(x, 254ull << 23);
    score[i] = __uint_as_float(0x00800000u + pick);
}
__global__ void score_block_kernel(float *score, int64_t n, int64_t start, int64_t m)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t rel = i >= start ? i - start : i + n - start;
    score[i] = rel < m ? 1.0f : 0.0f;
}

// ---- swap planning (host residency) ------------------------------------------------------------
__global__ void mark_clear_kernel(uint8_t *mark, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) mark[i] = 0;
}
__global__ void mark_set_kernel(uint8_t *mark, const int32_t *list, int64_t count)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) mark[list[k]] = 1;
}
// Device residency: how many selected coordinates were not in the current set (marked).
__global__ __launch_bounds__(256) void count_new_kernel(const int32_t *P, int64_t m, const uint8_t *mark,
                                                        SelectState *st)
{
    __shared__ uint32_t part[4];
    uint32_t mine = 0;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < m; k += (int64_t)gridDim.x * 256)
        mine += mark[P[k]] == 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, kWave);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {                      // one atomic per workgroup on the shared counter
        const uint32_t t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(&st->n_fill, t);
    }
}
// Selected columns that are in no device slot.
__global__ void find_fill_kernel(const int32_t *P, int64_t m, const int32_t *col_slot,
                                 SelectState *st, int32_t *fill_col)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < m && col_slot[P[k]] < 0) fill_col[atomicAdd(&st->n_fill, 1u)] = P[k];
}
// Slots that are empty (occupied == false) or hold a column outside the marked (protected) sets
// (occupied == true): launched for the empty ones first, so that no column is given up while a slot
// is free.
__global__ void find_evict_kernel(const int32_t *slot_col, int64_t budget, const uint8_t *mark,
                                  SelectState *st, int32_t *evict_slot, bool occupied)
{
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s < budget) {
        const int32_t j = slot_col[s];
        if (occupied ? (j >= 0 && mark[j] == 0) : j < 0) evict_slot[atomicAdd(&st->n_evict, 1u)] = (int32_t)s;
    }
}
// Pair the k-th missing column with the k-th evictable slot.  The evicted column loses its slot
// at once (later reads of it go to host memory); the new column gains it only when published.
__global__ void apply_plan_kernel(SelectState *st, const int32_t *fill_col,
                                  const int32_t *evict_slot, int32_t *fill_slot, int32_t *slot_col,
                                  int32_t *col_slot, int64_t limit)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= limit || k >= (int64_t)st->n_fill) return;
    if (k >= (int64_t)st->n_evict) { atomicOr(&st->error, 1u); return; }   // cannot happen
    const int32_t s = evict_slot[k];
    const int32_t old = slot_col[s];
    if (old >= 0) col_slot[old] = -1;
    slot_col[s] = fill_col[k];
    fill_slot[k] = s;
}
__global__ void publish_kernel(const SelectState *st, const int32_t *fill_col,
                               const int32_t *fill_slot, int32_t *col_slot, int64_t limit)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < limit && k < (int64_t)st->n_fill) col_slot[fill_col[k]] = fill_slot[k];
}

// Host -> device copy of the planned columns by a few workgroups reading the device-mapped
// pinned matrix directly; the list and its length stay on the device, so no host round trip.
// Eight workgroups (64 KB of reads in flight each) already saturate the host link (56 GB/s
// measured); more of them only slow the concurrent coordinate-descent pass down (5x with 32).
template <bool VEC4>
__global__ __launch_bounds__(256) void copy_columns_kernel(const float *src, int64_t ld,
                                                           const float *const *chunk, uint32_t chunk_cols,
                                                           float *slots, int64_t ld_s, int64_t d,
                                                           const SelectState *st,
                                                           const int32_t *fill_col,
                                                           const int32_t *fill_slot)
{
    const int64_t count = st->n_fill;
    for (int64_t k = blockIdx.x; k < count; k += gridDim.x) {
        const uint32_t j = (uint32_t)fill_col[k];
        const uint32_t piece = chunk ? j / chunk_cols : 0u;          // the matrix may come in pieces
        const float *s = (chunk ? chunk[piece] : src) + (int64_t)(j - piece * chunk_cols) * ld;
        float *t = slots + (int64_t)fill_slot[k] * ld_s;
        int64_t done = 0;
        if (VEC4) {
            const int64_t d4 = d >> 2;
            const float4 *s4 = reinterpret_cast<const float4 *>(s);
            float4 *t4 = reinterpret_cast<float4 *>(t);
            int64_t r = threadIdx.x;
            for (; r + 768 < d4; r += 1024) {
                const float4 a0 = s4[r], a1 = s4[r + 256], a2 = s4[r + 512], a3 = s4[r + 768];
                t4[r] = a0; t4[r + 256] = a1; t4[r + 512] = a2; t4[r + 768] = a3;
            }
            for (; r < d4; r += 256) t4[r] = s4[r];
            done = d4 << 2;
        }
        for (int64_t r = done + threadIdx.x; r < d; r += 256) t[r] = s[r];
    }
}

// The same copy for a batch of columns that host threads staged in pinned memory: column k of the
// batch goes to the slot planned for the (k0 + k)-th missing column.
__global__ __launch_bounds__(256) void copy_staged_kernel(const float4 *stage, int64_t lds4, float *slots,
                                                          int64_t ld_s, int64_t d4ceil, const int32_t *fill_slot,
                                                          int64_t count)
{
    for (int64_t k = blockIdx.x; k < count; k += gridDim.x) {
        const float4 *s4 = stage + k * lds4;
        float4 *t4 = reinterpret_cast<float4 *>(slots + (int64_t)fill_slot[k] * ld_s);
        int64_t r = threadIdx.x;
        for (; r + 768 < d4ceil; r += 1024) {
            const float4 a0 = s4[r], a1 = s4[r + 256], a2 = s4[r + 512], a3 = s4[r + 768];
            t4[r] = a0; t4[r + 256] = a1; t4[r + 512] = a2; t4[r + 768] = a3;
        }
        for (; r < d4ceil; r += 256) t4[r] = s4[r];
    }
}

// While the first pass over a staged matrix has a batch on hand (its gaps are just out), the columns
// whose gap reaches tau go into free device slots -- one workgroup per column claims the next slot
// until `limit` are taken -- so that the first working sets find most of their columns already on
// the device instead of crossing the host link a second time.
__global__ __launch_bounds__(256) void keep_staged_kernel(const float4 *stage, int64_t lds4, float *slots, int64_t ld_s,
                                                          int64_t d4ceil, const float *z, int64_t first, int64_t count,
                                                          float tau, SelectState *st, uint32_t limit,
                                                          int32_t *slot_col, int32_t *col_slot)
{
    __shared__ int claimed;
    for (int64_t k = blockIdx.x; k < count; k += gridDim.x) {
        const int64_t i = first + k;
        if (threadIdx.x == 0) {
            int s = -1;
            // (the counter may run past the limit; claims beyond it are void)
            const float zi = z[i];                  // (a gap of exactly zero never qualifies: most of a Lasso's are)
            if (zi >= tau && zi > 0.0f && st->n_kept < limit) {
                const uint32_t got = atomicAdd(&st->n_kept, 1u);
                if (got < limit) s = (int)got;
            }
            claimed = s;
        }
        __syncthreads();
        const int s = claimed;
        __syncthreads();
        if (s < 0) continue;
        const float4 *s4 = stage + k * lds4;
        float4 *t4 = reinterpret_cast<float4 *>(slots + (int64_t)s * ld_s);
        int64_t r = threadIdx.x;
        for (; r + 768 < d4ceil; r += 1024) {
            const float4 a0 = s4[r], a1 = s4[r + 256], a2 = s4[r + 512], a3 = s4[r + 768];
            t4[r] = a0; t4[r + 256] = a1; t4[r + 512] = a2; t4[r + 768] = a3;
        }
        for (; r < d4ceil; r += 256) t4[r] = s4[r];
        if (threadIdx.x == 0) {
            slot_col[s] = (int32_t)i;
            col_slot[i] = s;
        }
    }
}

}  // namespace

hipError_t launch_keep_batch(duhl_ctx *c, const StageBatch &b, int64_t first, float tau)
{
    hipLaunchKernelGGL(keep_staged_kernel, dim3(c->copy_blocks * 4), dim3(256), 0, c->compute,
                       reinterpret_cast<const float4 *>(b.stage), b.lds / 4, c->slots, c->ld_s, (c->d + 3) / 4, c->z,
                       first + b.k0, b.count, tau, c->sel, (uint32_t)c->budget, c->slot_col, c->col_slot);
    return hipGetLastError();
}

// Staged columns are 16-byte aligned and padded to a multiple of four floats, and so are the slots
// (ld_s is a multiple of 64), so whole 16-byte chunks are copied: ceil(d/4) of them.
hipError_t launch_copy_batch(duhl_ctx *c, const StageBatch &b)
{
    hipLaunchKernelGGL(copy_staged_kernel, dim3(c->copy_blocks), dim3(256), 0, c->copy,
                       reinterpret_cast<const float4 *>(b.stage), b.lds / 4, c->slots, c->ld_s, (c->d + 3) / 4,
                       c->fill_slot + b.k0, b.count);
    return hipGetLastError();
}

hipError_t launch_score(duhl_ctx *c, int scheme, int64_t m, uint64_t arg)
{
    const int T = 256;
    const int64_t n = c->n;
    if (scheme == DUHL_SELECT_RANDOM)
        hipLaunchKernelGGL(score_random_kernel, dim3((n + T - 1) / T), dim3(T), 0, c->compute, c->score, n, arg);
    else
        hipLaunchKernelGGL(score_block_kernel, dim3((n + T - 1) / T), dim3(T), 0, c->compute, c->score, n,
                           (int64_t)((arg % (uint64_t)((n + m - 1) / m)) * (uint64_t)m % (uint64_t)n), m);
    return hipGetLastError();
}

hipError_t launch_select(duhl_ctx *c, int64_t m, int32_t *P_out, const float *keys)
{
    const int64_t n = c->n;
    int64_t groups = c->select_groups > 0 && c->select_groups < kMaxGroups ? c->select_groups : kMaxGroups;
    int64_t chunk = ((n + groups - 1) / groups + kChunk - 1) / kChunk * kChunk;   // whole 8-tile batches
    if (chunk < kChunk) chunk = kChunk;
    const int64_t nb = (n + chunk - 1) / chunk;
    SelectArgs a;
    a.keys = keys;
    a.zval = c->z;
    a.n = n;
    a.m = m;
    a.chunk = (int)chunk;
    a.st = c->sel;
    a.blk_gt = c->blk_gt;
    a.blk_eq = c->blk_eq;
    a.P = c->P_next;
    a.P_out = P_out;
    a.partials = c->partials;
    a.scalars = c->scalars;
    a.bar_base = c->sel_bar;
    a.spin_limit = c->select_spin_limit;                 // default: seconds; the barriers take microseconds
    // chunks of up to 8,192 entries stay in registers for the whole kernel
    switch (chunk / 256) {
    case 8: hipLaunchKernelGGL(select_fused_kernel<8>, dim3(nb), dim3(256), 0, c->compute, a); break;
    case 16: hipLaunchKernelGGL(select_fused_kernel<16>, dim3(nb), dim3(256), 0, c->compute, a); break;
    case 24: hipLaunchKernelGGL(select_fused_kernel<24>, dim3(nb), dim3(256), 0, c->compute, a); break;
    case 32: hipLaunchKernelGGL(select_fused_kernel<32>, dim3(nb), dim3(256), 0, c->compute, a); break;
    default: hipLaunchKernelGGL(select_fused_kernel<0>, dim3(nb), dim3(256), 0, c->compute, a); break;
    }
    const hipError_t e = hipGetLastError();
    // five barriers of nb arrivals each: the device counter only moves if the kernel really runs
    if (e == hipSuccess) c->sel_bar += 5u * (uint32_t)nb;
    return e;
}

hipError_t launch_plan_swap(duhl_ctx *c, bool overlap_safe, bool want_count)
{
    hipStream_t s = c->compute;
    const int T = 256;
    const int64_t m = c->m_next;
    // device residency: nothing to copy, only count what changed -- and only if someone asks
    if (c->res != DUHL_RESIDENT_HOST && !want_count) return hipSuccess;
    hipLaunchKernelGGL(mark_clear_kernel, dim3((c->n + T - 1) / T), dim3(T), 0, s, c->mark, c->n);
    if (c->res != DUHL_RESIDENT_HOST) {
        if (c->m_cur > 0)
            hipLaunchKernelGGL(mark_set_kernel, dim3((c->m_cur + T - 1) / T), dim3(T), 0, s, c->mark,
                               c->P_cur, c->m_cur);
        int64_t cgrid = (m + 2047) / 2048;
        if (cgrid > kMaxGroups) cgrid = kMaxGroups;
        hipLaunchKernelGGL(count_new_kernel, dim3(cgrid), dim3(256), 0, s, c->P_next, m, c->mark, c->sel);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(mark_set_kernel, dim3((m + T - 1) / T), dim3(T), 0, s, c->mark, c->P_next, m);
    if (overlap_safe && c->m_cur > 0)
        hipLaunchKernelGGL(mark_set_kernel, dim3((c->m_cur + T - 1) / T), dim3(T), 0, s, c->mark,
                           c->P_cur, c->m_cur);
    hipLaunchKernelGGL(find_fill_kernel, dim3((m + T - 1) / T), dim3(T), 0, s, c->P_next, m,
                       c->col_slot, c->sel, c->fill_col);
    hipLaunchKernelGGL(find_evict_kernel, dim3((c->budget + T - 1) / T), dim3(T), 0, s, c->slot_col,
                       c->budget, c->mark, c->sel, c->evict_slot, false);
    hipLaunchKernelGGL(find_evict_kernel, dim3((c->budget + T - 1) / T), dim3(T), 0, s, c->slot_col,
                       c->budget, c->mark, c->sel, c->evict_slot, true);
    hipLaunchKernelGGL(apply_plan_kernel, dim3((m + T - 1) / T), dim3(T), 0, s, c->sel, c->fill_col,
                       c->evict_slot, c->fill_slot, c->slot_col, c->col_slot, m);
    return hipGetLastError();
}

hipError_t launch_copy_columns(duhl_ctx *c)
{
    const bool vec = c->a_aligned16 && (c->cv.ld % 4 == 0);
    if (vec)
        hipLaunchKernelGGL(copy_columns_kernel<true>, dim3(c->copy_blocks), dim3(256), 0, c->copy,
                           c->cv.base, c->cv.ld, c->cv.chunk, c->cv.chunk_cols, c->slots, c->ld_s, c->d,
                           c->sel, c->fill_col, c->fill_slot);
    else
        hipLaunchKernelGGL(copy_columns_kernel<false>, dim3(c->copy_blocks), dim3(256), 0, c->copy,
                           c->cv.base, c->cv.ld, c->cv.chunk, c->cv.chunk_cols, c->slots, c->ld_s, c->d,
                           c->sel, c->fill_col, c->fill_slot);
    return hipGetLastError();
}

hipError_t launch_publish(duhl_ctx *c)
{
    const int T = 256;
    const int64_t m = c->m_next;
    hipLaunchKernelGGL(publish_kernel, dim3((m + T - 1) / T), dim3(T), 0, c->compute, c->sel,
                       c->fill_col, c->fill_slot, c->col_slot, m);
    return hipGetLastError();
}

}  // namespace duhl
