// Internal declarations shared by the translation units of libduhl (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "duhl.h"

struct duhl_host_sampler;   // host-thread gap sampler (host_sampler.hip)
struct duhl_stager;         // pinned staging of a matrix in pageable host memory (host_stage.hip)

namespace duhl {

constexpr int kWave = 64;

// How a kernel finds the non-zeros of column a_j (the paper's A = [a_1 .. a_n], Section 2).
struct ColView {
    // dense
    const float *base;        // column j at base + j*ld (device memory, or device-mapped host memory)
    int64_t ld;
    // host matrix given in pieces: column j in piece j / chunk_cols, at chunk[..] + (j % chunk_cols)*ld;
    // base is then the first piece (non-null marks dense data)
    const float *const *chunk;
    uint32_t chunk_cols;
    const int32_t *col_slot;  // host residency: device slot holding column j, or -1; else nullptr
    const float *slots;       // slot s at slots + s*ld_s
    int64_t ld_s;
    // sparse (CSR over coordinates); used when base == nullptr
    const int64_t *rowptr;
    const int32_t *colidx;
    const float *val;

    __device__ __forceinline__ const float *col(int64_t j) const
    {
        if (col_slot) {
            const int32_t s = col_slot[j];
            if (s >= 0) return slots + (int64_t)s * ld_s;
        }
        if (chunk) {
            const uint32_t k = (uint32_t)j / chunk_cols;
            return chunk[k] + (int64_t)((uint32_t)j - k * chunk_cols) * ld;
        }
        return base + j * ld;
    }
};

// Constants of the model formulas (Appendix C, D, E), rounded once to fp32.
struct ModelConst {
    int model;        // duhl_model
    float Lam;        // Lasso: lambda * d
    float B;          // Lasso: Lipschitzing bound ||b||^2 / (2 lambda d)
    float inv_d;      // Lasso: 1/d
    float lam_n;      // SVM: lambda * n
    float inv_lam_n;  // SVM: 1/(lambda n)
    float inv_n;      // SVM: 1/n
    float lam_eta;    // elastic net: lambda d eta
    float lam_l1;     // elastic net: lambda d (1 - eta)
    float inv_2lam_eta;  // elastic net: 1 / (2 lambda d eta)
};

// The constants from the problem's sizes and parameters; B is the Lipschitzing bound of the Lasso
// (Appendix E: ||b||^2 / (2 lambda d)), eta the elastic-net mix.
inline ModelConst model_constants(int model, int64_t d_, int64_t n_, double lambda, double eta, double B)
{
    ModelConst mc{};
    mc.model = model;
    const double d = (double)d_, n = (double)n_;
    if (model == DUHL_LASSO) {
        mc.Lam = (float)(lambda * d);
        mc.B = (float)B;
        mc.inv_d = (float)(1.0 / d);
    } else if (model == DUHL_ELASTIC_NET) {
        mc.Lam = (float)(lambda * d);
        mc.lam_eta = (float)(lambda * d * eta);
        mc.lam_l1 = (float)(lambda * d * (1.0 - eta));
        mc.inv_2lam_eta = (float)(1.0 / (2.0 * lambda * d * eta));
        mc.inv_d = (float)(1.0 / d);
    } else {
        mc.lam_n = (float)(lambda * n);
        mc.inv_lam_n = (float)(1.0 / (lambda * n));
        mc.inv_n = (float)(1.0 / n);
    }
    return mc;
}

// Columns per wavefront of the dense gap pass: several amortise the reads of v, but a problem of
// few columns needs one wavefront per column to put enough of them on every compute unit.
inline int default_gap_cols(int64_t d, int64_t n, int num_cu)
{
    int cols = d < 4096 ? 8 : 4;
    while (cols > 1 && n / cols < 8 * (int64_t)num_cu) cols /= 2;
    return cols;
}

// Coordinate gap from c = a_i^T v (Appendix E), clamped at 0 (Section 2: the gap is non-negative).
template <int MODEL>
__device__ __forceinline__ float gap_value(const ModelConst &mc, float c, float alpha, float y)
{
    float z;
    if (MODEL == DUHL_LASSO) {
        const float over = fmaxf(fabsf(c) - mc.Lam, 0.0f);
        z = (fmaf(alpha, c, mc.Lam * fabsf(alpha)) + mc.B * over) * mc.inv_d;
    } else if (MODEL == DUHL_ELASTIC_NET) {
        const float over = fmaxf(fabsf(c) - mc.lam_l1, 0.0f);
        const float reg = fmaf(0.5f * mc.lam_eta * alpha, alpha, mc.lam_l1 * fabsf(alpha));
        z = (fmaf(alpha, c, reg) + over * over * mc.inv_2lam_eta) * mc.inv_d;
    } else {
        const float s = c * mc.inv_lam_n;
        const float hinge = fmaxf(1.0f - y * s, 0.0f);
        z = (fmaf(alpha, s, hinge) - y * alpha) * mc.inv_n;
    }
    return z > 0.0f ? z : 0.0f;
}

// Exact minimiser over coordinate j given c = a_j^T v, q = ||a_j||^2 (Appendix D).
template <int MODEL>
__device__ __forceinline__ float cd_new_alpha(const ModelConst &mc, float c, float alpha, float q,
                                              float y)
{
    if (MODEL == DUHL_LASSO) {
        if (!(q > 0.0f)) return 0.0f;
        const float gamma = alpha - c / q;
        const float mag = fabsf(gamma) - mc.Lam / q;
        return mag > 0.0f ? copysignf(mag, gamma) : 0.0f;
    } else if (MODEL == DUHL_ELASTIC_NET) {
        const float den = q + mc.lam_eta;
        const float gamma = fmaf(alpha, q, -c) / den;
        const float mag = fabsf(gamma) - mc.lam_l1 / den;
        return mag > 0.0f ? copysignf(mag, gamma) : 0.0f;
    } else {
        if (!(q > 0.0f)) return y;
        const float step = (y - c * mc.inv_lam_n) * (mc.lam_n / q);
        const float t = fminf(fmaxf(y * (alpha + step), 0.0f), 1.0f);
        return y * t;
    }
}

// The terms of the objective that depend on alpha_j alone (Appendix C / D): lambda |alpha| (Lasso),
// lambda (eta/2 alpha^2 + (1-eta)|alpha|) (elastic net), -(1/n) y alpha (SVM dual).
template <int MODEL>
__device__ __forceinline__ float objective_term(const ModelConst &mc, float alpha, float y)
{
    if (MODEL == DUHL_LASSO) return mc.Lam * mc.inv_d * fabsf(alpha);
    if (MODEL == DUHL_ELASTIC_NET)
        return mc.inv_d * fmaf(0.5f * mc.lam_eta * alpha, alpha, mc.lam_l1 * fabsf(alpha));
    return -mc.inv_n * y * alpha;
}
// objective_term(now) - objective_term(old) without the cancellation of two rounded terms.
template <int MODEL>
__device__ __forceinline__ double objective_term_change(const ModelConst &mc, float now, float old, float y)
{
    const double dn = (double)now, dol = (double)old;
    if (MODEL == DUHL_LASSO) return (double)mc.Lam * (double)mc.inv_d * (fabs(dn) - fabs(dol));
    if (MODEL == DUHL_ELASTIC_NET)
        return (double)mc.inv_d * (0.5 * (double)mc.lam_eta * (dn - dol) * (dn + dol) + (double)mc.lam_l1 * (fabs(dn) - fabs(dol)));
    return -(double)mc.inv_n * (double)y * (dn - dol);
}
// Factor of ||v||^2 in the objective: 1/(2d), or 1/(2 lambda n^2) for the SVM dual.
inline double quad_scale(const ModelConst &mc)
{
    return mc.model == DUHL_SVM ? 0.5 * (double)mc.inv_lam_n * (double)mc.inv_n : 0.5 * (double)mc.inv_d;
}

// 16-byte load of matrix data that is read once per pass: the non-temporal hint keeps the stream
// from displacing v and the other small arrays in the caches (measured: 6.7-7.0 TB/s against
// 6.0-6.3 TB/s for plain loads on a 32 GB read).
typedef float duhl_v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float4 *p)
{
    const duhl_v4f t = __builtin_nontemporal_load(reinterpret_cast<const duhl_v4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

// Cross-lane moves as DPP modifiers of ordinary vector instructions (full rate) rather than trips
// through the LDS crossbar.  Controls: quad_perm patterns (one byte, two bits per lane of a
// quad), row_ror:n = 0x120 + n (rotation inside a row of 16 lanes), row_half_mirror = 0x141.
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    return x + __int_as_float(dpp_mov<CTRL>(__float_as_int(x)));
}
template <int CTRL>
__device__ __forceinline__ int64_t dpp_mov64(int64_t x)
{
    const int lo = dpp_mov<CTRL>((int)(uint32_t)x), hi = dpp_mov<CTRL>((int)(x >> 32));
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
template <int CTRL>
__device__ __forceinline__ double dpp_add(double x)
{
    return x + __longlong_as_double(dpp_mov64<CTRL>(__double_as_longlong(x)));
}

// Sum over the 64 lanes of a wavefront; every lane receives the result.  All lanes must be
// active.  Rotations by 8, 4, 2, 1 give every lane the sum of its row of 16; the four row sums
// are then read from one lane each.
template <typename F>
__device__ __forceinline__ F row_sum16(F x)
{
    x = dpp_add<0x128>(x);
    x = dpp_add<0x124>(x);
    x = dpp_add<0x122>(x);
    x = dpp_add<0x121>(x);
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
    const int r = __float_as_int(row_sum16(x));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(r, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(r, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(r, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(r, 48));
    return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ double wave_sum(double x)
{
    const int64_t r = __double_as_longlong(row_sum16(x));
    const int lo = (int)(uint32_t)r, hi = (int)(r >> 32);
    double part[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t l = (uint32_t)__builtin_amdgcn_readlane(lo, 16 * k);
        const uint32_t h = (uint32_t)__builtin_amdgcn_readlane(hi, 16 * k);
        part[k] = __longlong_as_double((int64_t)(((uint64_t)h << 32) | l));
    }
    return (part[0] + part[1]) + (part[2] + part[3]);
}
// Sum over aligned groups of G lanes (G a power of two <= 64).
template <int G>
__device__ __forceinline__ float group_sum(float x)
{
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}

// Slots of the device scalar block (doubles), results of reductions.
enum Scalar { S_GAP_SUM = 0, S_SUM_ALL, S_SUM_SEL, S_RHO, S_OBJ_SQ, S_OBJ_LIN, S_BSQ, S_CORR, S_SINK, S_COUNT };

// Scratch of the selection kernels (device memory, one per context).
struct SelectState {
    uint32_t hist[3][2048];
    uint32_t barrier;    // arrivals at the selection kernel's barriers, only ever incremented
    uint32_t thr_key;    // key of the smallest selected entry of the last selection
    uint32_t reserved[8];
    uint32_t n_fill;     // columns to copy (host residency)
    uint32_t n_evict;    // evictable slots found
    uint32_t error;      // validation flags
    uint32_t cd_abort;   // set by a workgroup that gave up waiting for others (selection barrier, CD partners)
    uint32_t n_kept;     // slots claimed by the columns kept during the first pass over a staged matrix
    uint32_t pad;
};

// Device state of the guard of the concurrent passes.  Exact coordinate steps never raise the
// objective; steps taken at once on columns that are alike overshoot together.  The guard looks at
// the pass as one step from (alpha, v) to (alpha + D, v + Dv): along that line the objective is
// bounded by  theta * lin + theta^2 * curv  above its old value (the quadratic part exactly, the
// convex terms in alpha by their chord), which is smallest at theta* = -lin / (2 curv).  theta* >= 1
// is what sequential steps give; theta* near 1/k means k-fold overshoot, and below 1/2 the pass
// has raised the objective.
struct GuardState {
    double dreg;            // the pass so far: change of the objective's terms in alpha (regulariser / linear term)
    double last_delta;      // objective change of the last guarded pass (as measured, before any damping)
    double last_theta;      // theta* of the last guarded pass (1 when too small a step to tell)
    uint32_t arrived;       // workgroups of the finishing kernel that are done (the last one decides)
    uint32_t trips;         // passes damped (scaled back to theta* < 1, or undone) since the data were set
    uint32_t shift;         // halvings of the bound on concurrent steps now asked for: +1 per damped pass,
    uint32_t clean;         // -1 after `need` passes in a row (counted here) with theta* near 1
    uint32_t need;          // 0 stands for 4; doubles with every damped pass (a level that failed is tried again later and later)
    uint32_t pad;
    unsigned long long steps_pass;   // coordinate steps taken by the pass so far
    unsigned long long steps_kept;   // coordinate steps of all passes that were not undone, since the data were set
};

}  // namespace duhl

struct duhl_ctx {
    duhl_model model;
    int64_t d, n, budget;
    int device;
    hipStream_t compute, copy;
    int num_cu;

    bool have_data;
    bool sparse;
    duhl_residency res;
    double lambda;
    duhl::ModelConst mc;
    duhl::ColView cv;
    const float *target;   // b (Lasso) or y (SVM), device, borrowed
    int64_t nnz;

    // owned device state
    float *alpha, *v, *z, *q;
    int32_t *P_cur, *P_next;
    int64_t m_cur, m_next;
    bool pending;          // a selected set waits for duhl_commit_swap
    bool swap_exclusive;   // the pending copies reuse slots of the current set
    uint64_t pass_counter;
    double mean_corr;      // mean cosine between columns, estimated on a sample (>= 0)
    double eta;            // elastic-net mix requested through duhl_set_eta
    double eta_active;     // the mix the current data were set with

    double *scalars;            // S_COUNT doubles
    double *partials;           // per-block partial sums
    int64_t partials_cap;
    duhl::SelectState *sel;
    uint32_t *blk_gt, *blk_eq;  // per-chunk counts of the selection scatter
    int64_t blk_cap;

    float *score;               // scores of the non-gap selection rules (allocated on first use)

    // sparse data: copy of the matrix blocked by ranges of v, for the full gap pass (cb_R == 0: none)
    int64_t *cb_soff;        // slice starts
    int32_t *cb_perm;        // rows by position
    int64_t cb_slices;       // slices per range
    uint16_t *cb_idx;
    float *cb_val, *cb_partial;
    int cb_R, cb_W;

    // private buffers of the asynchronous dense workers (allocated on first use)
    float *dv;
    int64_t dv_stride, dv_workers;
    int32_t *dirty;
    uint32_t sel_bar;           // value the selection kernel's barrier counter has before its next launch
    uint64_t *xch;              // exchange slots of workers that span several compute units
    float *snap_alpha, *snap_v; // duhl_run's last good iterate (allocated on first use)
    // guard of the concurrent passes (allocated on first use)
    duhl::GuardState *guard;
    double *guard_part;         // per-workgroup partial sums of ||v||^2 before and after the pass
    int64_t guard_part_cap;
    float *snap_pass_v;         // v at the start of the pass
    double2 *guard_wbook;       // per dense worker: its books of the sub-pass (see MergeGuard)
    uint64_t *alpha_old;        // per position of the visiting order: (stamp of the pass, alpha_j before it moved)
    uint32_t guard_stamp;       // stamp of the last guarded pass; never reset while the context lives
    int64_t alpha_old_cap;
    uint32_t *h_trips;          // pinned, device-writable: GuardState::trips and ::shift as the host may read
    uint32_t *h_trips_dev;      // them without waiting ([0], [1])
    int keep_first_pass;        // 0: the first pass over a staged matrix keeps no columns (DUHL_KEEP_FIRST_PASS)
    int64_t kept_first_pass;    // columns that pass left in device slots
    bool z_fresh;               // device residency: every z_i is the gap at the current (alpha, v) -- true from
    double z_fresh_sum;         // set_data's pass until alpha, v or z change -- and this is their sum
    bool ptr_escaped;           // the caller holds a device pointer to alpha, v or z: never assume z fresh
    int gap_lds;                // 0: the dense gap pass never keeps v on chip (DUHL_GAP_LDS)
    int64_t gap_lds_min_parts, gap_lds_max_count;   // where it does (DUHL_GAP_LDS_MIN_PARTS, DUHL_GAP_LDS_MAX_COUNT)
    float *gap_pdot;            // partial dot products of that pass when v takes several parts
    int64_t gap_pdot_cap;
    int cd_guard;               // 0: guard switched off (DUHL_CD_GUARD)
    double guard_tol;           // relative rise of the objective that still counts as rounding
    int guard_start;            // halvings of the bound in force right after set_data
    int guard_shift;            // halvings of the library's bound on concurrent steps that the host applies
    hipEvent_t ev_pass[2];      // behind the last two guarded passes: while the bound is halved the host stays
    uint64_t guard_passes;      // at most two passes ahead of the device, so that it sees the bound recover
    uint64_t ev_pass_no[2];     // 1 + the number of the pass each event was recorded behind (0: none)
    void *cd_plan;              // sparse sub-passes: one record per position of the visiting order
    int64_t cd_plan_cap;
    uint32_t xseq;              // next free sequence number for those slots

    // host residency
    std::vector<const float *> host_chunks;   // the caller's host addresses of the matrix: its pieces, or one entry
    int64_t chunk_cols;         // columns per piece (n when the matrix is one piece)
    int64_t host_ld;            // floats between the columns of the host matrix
    const float **chunk_tab;    // device table of the pieces' device addresses (nullptr: one piece)
    bool a_aligned16;           // every piece (or the matrix) starts on a 16-byte boundary
    duhl_host_sampler *sampler; // unit A's gap sampler, created on first use
    bool pageable;              // the host matrix is in ordinary memory that the device cannot read:
                                // every column crosses the link through pinned staging buffers
    duhl_stager *stager;        // those buffers, their copy threads and the background swap job
    float *slots;
    int64_t ld_s;
    int32_t *col_slot, *slot_col;
    uint8_t *mark;
    int32_t *fill_col, *fill_slot, *evict_slot;
    hipEvent_t ev_plan, ev_copy;
    hipEvent_t ev_copy_begin;   // on the copy stream, before the first column copy of a selection (timing)
    bool swap_timed;            // ev_copy_begin / ev_copy bracket a finished or running swap

    double *h_scalars;          // pinned staging for scalar read-back
    uint32_t *h_u32;

    // tuning knobs (environment, read at creation)
    int gap_cols;      // columns per wavefront in the dense gap kernel
    int cd_threads;    // threads per coordinate in the async dense kernel (0 = by d)
    int copy_blocks;   // workgroups of the column-copy kernel
    int cd_units;      // compute units per dense CD worker for long columns (0 = by d, 1 = never more than one)
    int cd_spin_limit; // polls a workgroup waits for a partner's partial sum before it gives up
    int select_spin_limit;   // polls a workgroup of the selection kernel waits at a barrier
    int select_groups;       // most workgroups of the selection kernel (0: the kernel's own limit)
    int csr_blocked;         // build and use the blocked copy of sparse data
    int csr_blocked_waves;   // workgroups per compute unit launched by its pass
    int csr_blocked_list_min;   // shortest index list evaluated from the blocked copy (< 0: n/4)

    std::string err;
};

namespace duhl {

// Host address of column j of a host-resident dense matrix.
inline const float *host_col(const duhl_ctx *c, int64_t j)
{
    const int64_t k = j / c->chunk_cols;
    return c->host_chunks[(size_t)k] + (j - k * c->chunk_cols) * c->host_ld;
}

// ---- launchers (each enqueues on the given stream and returns the launch status) ----------
hipError_t launch_gap(duhl_ctx *c, const int32_t *idx, int64_t count, bool slot_list,
                      bool with_norms);
hipError_t launch_select(duhl_ctx *c, int64_t m, int32_t *P_out, const float *keys);
hipError_t launch_score(duhl_ctx *c, int scheme, int64_t m, uint64_t arg);
hipError_t launch_plan_swap(duhl_ctx *c, bool overlap_safe, bool want_count);
hipError_t launch_copy_columns(duhl_ctx *c);
hipError_t launch_publish(duhl_ctx *c);
hipError_t launch_cd(duhl_ctx *c, duhl_cd_mode mode, const int32_t *order, int64_t count,
                     uint64_t seed, int max_inflight);
int64_t default_inflight(const duhl_ctx *c, int64_t count);
hipError_t launch_objective(duhl_ctx *c);
hipError_t launch_init_v(duhl_ctx *c);
hipError_t launch_accumulate_v(duhl_ctx *c);
hipError_t launch_corr_sample(duhl_ctx *c, float *u, int samples);
hipError_t launch_validate(duhl_ctx *c);
hipError_t launch_check_norms(duhl_ctx *c);
hipError_t launch_stream_read(duhl_ctx *c, const void *dev, int64_t bytes, float *sink);
hipError_t launch_scatter_add(duhl_ctx *c, int64_t ops, int64_t *done);
hipError_t launch_fill_i32(hipStream_t s, int32_t *p, int64_t n, int32_t value);
hipError_t launch_fill_f32(hipStream_t s, float *p, int64_t n, float value);
hipError_t launch_sum_partials(duhl_ctx *c, int64_t count, int scalar_slot);
void host_sampler_destroy(duhl_ctx *c);
int64_t host_sampler_prefix(const duhl_ctx *c);   // leading list entries the last host sampling round refreshed
// ---- pageable host matrix (host_stage.hip) -------------------------------------------------------
// One batch of staged columns: column k of the batch is at stage + k*lds (device-readable pinned
// memory, 16-byte aligned columns); it is list entry k0 + k of the pass.
struct StageBatch {
    const float *stage;
    int64_t lds, k0, count;
};
hipError_t stager_create(duhl_ctx *c);
void stager_destroy(duhl_ctx *c);
// The gap pass over columns read from host memory: the listed coordinates (device list idx of `count`
// entries), or first .. first+count-1 when idx == nullptr.  Waits for the compute stream.
hipError_t staged_gap(duhl_ctx *c, const int32_t *idx, int64_t first, int64_t count, bool with_norms);
hipError_t staged_corr_sample(duhl_ctx *c, float *u, int samples);
hipError_t staged_accumulate_v(duhl_ctx *c);
// Column swap: reads the plan back, then a background thread stages the missing columns and
// enqueues their copies into the slots on the copy stream; stager_swap_join waits until all of them
// are enqueued and ev_copy is recorded.
hipError_t stager_swap_begin(duhl_ctx *c);
hipError_t stager_swap_join(duhl_ctx *c);
bool stager_swap_done(duhl_ctx *c);
// Host residency: are the column copies of the pending selection still running?
bool swap_in_flight(duhl_ctx *c);
// kernels of other files that the staged passes launch
hipError_t launch_gap_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx, int64_t first, bool with_norms,
                            bool first_batch);
hipError_t launch_corr_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx, float *u);
hipError_t launch_accumulate_batch(duhl_ctx *c, const StageBatch &b, const int32_t *idx);
hipError_t launch_copy_batch(duhl_ctx *c, const StageBatch &b);
hipError_t launch_keep_batch(duhl_ctx *c, const StageBatch &b, int64_t first, float tau);

hipError_t csr_blocked_build(duhl_ctx *c);
void csr_blocked_free(duhl_ctx *c);
hipError_t launch_gap_csr_blocked(duhl_ctx *c, const int32_t *idx, int64_t count, int64_t *grid_out);

}  // namespace duhl
