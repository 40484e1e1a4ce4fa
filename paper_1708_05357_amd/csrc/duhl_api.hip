// Host side of libduhl: the extern "C" entry points declared in duhl.h.
// Argument checks, memory, stream/event choreography; all arithmetic is in the kernels.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "duhl_internal.h"

using namespace duhl;

namespace {

duhl_status fail(duhl_ctx *c, duhl_status st, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return st;
}

#define HIPCHK(c, expr)                                                                       \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail((c), e_ == hipErrorOutOfMemory ? DUHL_ENOMEM : DUHL_EHIP, "%s: %s",   \
                        #expr, hipGetErrorString(e_));                                        \
    } while (0)

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return (s && *s) ? atoi(s) : dflt;
}

template <typename T>
hipError_t dev_alloc(T **p, int64_t count)
{
    *p = nullptr;
    return hipMalloc(reinterpret_cast<void **>(p), (size_t)(count > 0 ? count : 1) * sizeof(T));
}

void free_host_residency(duhl_ctx *c)
{
    host_sampler_destroy(c);
    stager_destroy(c);
    c->pageable = false;
    csr_blocked_free(c);
    c->host_chunks.clear();
    (void)hipFree(c->chunk_tab); c->chunk_tab = nullptr;
    (void)hipFree(c->slots); c->slots = nullptr;
    (void)hipFree(c->col_slot); c->col_slot = nullptr;
    (void)hipFree(c->slot_col); c->slot_col = nullptr;
    (void)hipFree(c->fill_col); c->fill_col = nullptr;
    (void)hipFree(c->fill_slot); c->fill_slot = nullptr;
    (void)hipFree(c->evict_slot); c->evict_slot = nullptr;
    if (c->ev_plan) { (void)hipEventDestroy(c->ev_plan); c->ev_plan = nullptr; }
    if (c->ev_copy) { (void)hipEventDestroy(c->ev_copy); c->ev_copy = nullptr; }
    if (c->ev_copy_begin) { (void)hipEventDestroy(c->ev_copy_begin); c->ev_copy_begin = nullptr; }
    c->swap_timed = false;
}

// Read `count` doubles of the device scalar block after the compute stream has drained.
duhl_status read_scalars(duhl_ctx *c, int first, int count)
{
    HIPCHK(c, hipMemcpyAsync(c->h_scalars + first, c->scalars + first, sizeof(double) * count,
                             hipMemcpyDeviceToHost, c->compute));
    HIPCHK(c, hipMemcpyAsync(c->h_u32 + 2, &c->sel->cd_abort, sizeof(uint32_t), hipMemcpyDeviceToHost,
                             c->compute));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    if (c->h_u32[2] != 0)
        return fail(c, DUHL_EHIP,
                    "a device-side wait between workgroups timed out (selection or coordinate descent); "
                    "the working set, alpha and v are undefined, set the data again");
    return DUHL_OK;
}

// Everything set_data does after the matrix view is in place.
duhl_status finish_set_data(duhl_ctx *c, const float *target, double lambda)
{
    c->target = target;
    c->lambda = lambda;
    c->cv.col_slot = c->col_slot;
    c->cv.slots = c->slots;
    c->cv.ld_s = c->ld_s;

    HIPCHK(c, launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->sel->error), 2, 0));   // and cd_abort
    // the selection kernel expects clean histograms and leaves them clean, unless a barrier failed
    HIPCHK(c, launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->sel->hist[0][0]), 3 * 2048, 0));
    // a selection that gave up at a barrier (or was never launched) leaves the device's arrival
    // counter behind the host's account of it: both start again from zero
    HIPCHK(c, launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->sel->barrier), 1, 0));
    c->sel_bar = 0;
    HIPCHK(c, launch_validate(c));
    HIPCHK(c, hipMemcpyAsync(c->h_u32, &c->sel->error, sizeof(uint32_t), hipMemcpyDeviceToHost,
                             c->compute));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    const uint32_t flags = c->h_u32[0];
    if (flags & 1u) return fail(c, DUHL_EINVAL, "labels must be +1 or -1");
    if (flags & 8u) return fail(c, DUHL_EINVAL, "target vector holds a non-finite value");
    if (flags & 2u) return fail(c, DUHL_EINVAL, "rowptr must start at 0, be non-decreasing and end at rowptr[n]");
    if (flags & 4u)
        return fail(c, DUHL_EINVAL,
                    "column indices must lie in [0,d) and increase strictly inside a row");

    HIPCHK(c, launch_fill_f32(c->compute, c->alpha, c->n, 0.0f));
    HIPCHK(c, launch_fill_f32(c->compute, c->z, c->n, 0.0f));
    HIPCHK(c, launch_init_v(c));

    double bound = 0.0;
    if (c->model == DUHL_LASSO) {
        duhl_status st = read_scalars(c, S_BSQ, 1);
        if (st != DUHL_OK) return st;
        bound = c->h_scalars[S_BSQ] / (2.0 * lambda * (double)c->d);   // Appendix E: ||b||^2/(2 lambda d)
    } else if (c->model == DUHL_ELASTIC_NET) {
        c->eta_active = c->eta;
    }
    const ModelConst mc = model_constants(c->model, c->d, c->n, lambda, c->eta, bound);
    c->mc = mc;
    c->m_cur = c->m_next = 0;
    c->pending = c->swap_exclusive = false;
    c->pass_counter = 0;
    if (c->guard) {                                 // a new problem: the bound on concurrent steps starts afresh
        HIPCHK(c, launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(c->guard), sizeof(GuardState) / 4, 0));
        // (the first passes from alpha = 0 are the ones in which every coordinate moves, and steps
        // collide most: they start with half the bound, which the guard doubles after four passes)
        HIPCHK(c, launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->guard->shift), 1, c->guard_start));
        c->h_trips[0] = 0;
        c->h_trips[1] = (uint32_t)c->guard_start;
    }
    c->guard_shift = c->cd_guard ? c->guard_start : 0;
    c->have_data = true;
    // column norms and a first full gap pass in one read of the matrix
    HIPCHK(c, launch_gap(c, nullptr, c->n, false, true));
    // a NaN or an infinity anywhere in the matrix shows in its column's norm
    HIPCHK(c, launch_check_norms(c));
    HIPCHK(c, hipMemcpyAsync(c->h_u32, &c->sel->error, sizeof(uint32_t), hipMemcpyDeviceToHost, c->compute));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    if (c->h_u32[0] & 16u) {
        c->have_data = false;
        return fail(c, DUHL_EINVAL, "the matrix holds a non-finite value (a column norm is not finite)");
    }
    // how strongly the columns share a direction, from up to 1024 evenly spaced columns; it sets
    // the default bound on concurrent coordinate steps
    c->mean_corr = 0.0;
    const int samples = (int)(c->n < 1024 ? c->n : 1024);
    if (samples > 1) {
        float *u = nullptr;
        HIPCHK(c, dev_alloc(&u, c->d));
        hipError_t e = launch_corr_sample(c, u, samples);
        duhl_status st = e == hipSuccess ? read_scalars(c, S_CORR, 1) : DUHL_EHIP;
        (void)hipFree(u);
        if (st != DUHL_OK) return fail(c, st, "column correlation estimate failed");
        const double uu = c->h_scalars[S_CORR];
        const double mc_ = (uu / samples - 1.0) / (samples - 1.0);
        c->mean_corr = mc_ > 0.0 ? mc_ : 0.0;
    }
    HIPCHK(c, hipStreamSynchronize(c->compute));
    HIPCHK(c, hipGetLastError());
    // the first pass has left every gap at alpha = 0 in z: a full duhl_gap before anything moves
    // would only compute the same again
    c->z_fresh = false;
    if (c->res == DUHL_RESIDENT_DEVICE && !c->ptr_escaped) {
        duhl_status st = read_scalars(c, S_GAP_SUM, 1);
        if (st != DUHL_OK) return st;
        c->z_fresh_sum = c->h_scalars[S_GAP_SUM];
        c->z_fresh = true;
    }
    return DUHL_OK;
}

duhl_status check_common(duhl_ctx *c, const void *target, double lambda)
{
    if (!c) return DUHL_EINVAL;
    if (!target) return fail(c, DUHL_EINVAL, "target is NULL");
    if (!(lambda > 0.0) || !std::isfinite(lambda)) return fail(c, DUHL_EINVAL, "lambda must be finite and > 0");
    return DUHL_OK;
}

// Dense data: one piece in device or host memory, or several pieces in host memory.
duhl_status set_data_dense_pieces(duhl_ctx *c, const float *const *pieces, int64_t n_pieces,
                                         int64_t piece_cols, int64_t ld, duhl_residency res,
                                         const float *target, double lambda)
{
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    HIPCHK(c, hipStreamSynchronize(c->copy));       // column copies of a pending selection
    c->have_data = false;
    free_host_residency(c);
    c->sparse = false;
    const bool pageable = res == DUHL_RESIDENT_HOST_PAGEABLE;
    if (pageable) res = DUHL_RESIDENT_HOST;         // host residency in every other respect
    c->pageable = pageable;
    c->res = res;
    c->nnz = c->d * c->n;
    c->cv = ColView{};
    c->cv.ld = ld;
    c->host_ld = ld;
    c->chunk_cols = piece_cols;
    c->a_aligned16 = true;
    for (int64_t k = 0; k < n_pieces; ++k)
        c->a_aligned16 = c->a_aligned16 && (reinterpret_cast<uintptr_t>(pieces[k]) & 15) == 0;
    if (res == DUHL_RESIDENT_DEVICE) {
        c->cv.base = pieces[0];
        c->ld_s = 0;
    } else {
        std::vector<const float *> dev(n_pieces);
        for (int64_t k = 0; k < n_pieces && !pageable; ++k) {
            void *dptr = nullptr;
            if (hipHostGetDevicePointer(&dptr, const_cast<float *>(pieces[k]), 0) != hipSuccess || !dptr) {
                (void)hipGetLastError();
                return fail(c, DUHL_EINVAL, "host-resident A must be pinned, device-mapped host memory");
            }
            dev[k] = static_cast<const float *>(dptr);
            c->a_aligned16 = c->a_aligned16 && (reinterpret_cast<uintptr_t>(dptr) & 15) == 0;
        }
        c->cv.base = dev[0];
        c->host_chunks.assign(pieces, pieces + n_pieces);
        if (n_pieces > 1 && !pageable) {
            HIPCHK(c, dev_alloc(&c->chunk_tab, n_pieces));
            HIPCHK(c, hipMemcpy(c->chunk_tab, dev.data(), sizeof(float *) * (size_t)n_pieces, hipMemcpyHostToDevice));
            c->cv.chunk = c->chunk_tab;
            c->cv.chunk_cols = (uint32_t)piece_cols;
        }
        c->ld_s = (c->d + 63) / 64 * 64;
        HIPCHK(c, dev_alloc(&c->slots, c->budget * c->ld_s));
        HIPCHK(c, dev_alloc(&c->col_slot, c->n));
        HIPCHK(c, dev_alloc(&c->slot_col, c->budget));
        HIPCHK(c, dev_alloc(&c->fill_col, c->budget));
        HIPCHK(c, dev_alloc(&c->fill_slot, c->budget));
        HIPCHK(c, dev_alloc(&c->evict_slot, c->budget));
        HIPCHK(c, hipEventCreateWithFlags(&c->ev_plan, hipEventDisableTiming));
        HIPCHK(c, hipEventCreate(&c->ev_copy));             // these two also time the copies
        HIPCHK(c, hipEventCreate(&c->ev_copy_begin));
        HIPCHK(c, launch_fill_i32(c->compute, c->col_slot, c->n, -1));
        HIPCHK(c, launch_fill_i32(c->compute, c->slot_col, c->budget, -1));
        if (pageable) {
            // no kernel may follow a host address: a column that is in no slot is only ever read from
            // a staging buffer.  The view keeps a harmless device address for coordinates without a
            // slot (slot 0, stride 0), so that a caller's list that names one reads valid memory.
            c->cv.base = c->slots;
            c->cv.ld = 0;
            c->a_aligned16 = true;
            HIPCHK(c, stager_create(c));
        }
    }
    return finish_set_data(c, target, lambda);
}

}  // namespace

namespace duhl {
bool swap_in_flight(duhl_ctx *c)
{
    if (!c->pending || c->res != DUHL_RESIDENT_HOST || !c->ev_copy) return false;
    // (pageable memory: the background thread records the event only after its last batch)
    if (c->pageable && c->stager && !stager_swap_done(c)) return true;
    return hipEventQuery(c->ev_copy) == hipErrorNotReady;
}
}  // namespace duhl

extern "C" {

duhl_status duhl_create(duhl_ctx **out, duhl_model model, int64_t d, int64_t n, int64_t budget_cols,
                        int device, void *compute_stream, void *copy_stream)
{
    if (!out) return DUHL_EINVAL;
    if (model != DUHL_LASSO && model != DUHL_SVM && model != DUHL_ELASTIC_NET) return DUHL_EINVAL;
    // n: coordinates are int32.  d: kernels address a column and v with 32-bit byte offsets.
    if (d <= 0 || n <= 0 || budget_cols <= 0 || n > 0x7fffffffll || d >= (1ll << 29)) return DUHL_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return DUHL_EHIP;
    if (hipSetDevice(device) != hipSuccess) return DUHL_EHIP;
    duhl_ctx *c = new (std::nothrow) duhl_ctx();
    if (!c) return DUHL_ENOMEM;
    c->model = model;
    c->d = d;
    c->n = n;
    c->budget = budget_cols < n ? budget_cols : n;
    c->device = device;
    c->eta = c->eta_active = 1.0;
    c->compute = reinterpret_cast<hipStream_t>(compute_stream);
    c->copy = reinterpret_cast<hipStream_t>(copy_stream);
    c->num_cu = 256;
    (void)hipDeviceGetAttribute(&c->num_cu, hipDeviceAttributeMultiprocessorCount, device);
    const int gap_cols = default_gap_cols(d, n, c->num_cu);
    c->gap_cols = env_int("DUHL_GAP_COLS", gap_cols);
    if (c->gap_cols != 1 && c->gap_cols != 2 && c->gap_cols != 4 && c->gap_cols != 8) c->gap_cols = gap_cols;
    c->cd_threads = env_int("DUHL_CD_THREADS", 0);
    c->copy_blocks = env_int("DUHL_COPY_BLOCKS", 8);
    if (c->copy_blocks < 1) c->copy_blocks = 1;
    c->cd_units = env_int("DUHL_CD_UNITS", 0);
    c->cd_spin_limit = env_int("DUHL_CD_SPIN_LIMIT", 1 << 22);
    if (c->cd_spin_limit < 0) c->cd_spin_limit = 0;
    c->gap_lds = env_int("DUHL_GAP_LDS", 1);
    c->gap_lds_min_parts = env_int("DUHL_GAP_LDS_MIN_PARTS", 2);
    if (c->gap_lds_min_parts < 2) c->gap_lds_min_parts = 2;   // (one part: the formula would belong in the same kernel)
    c->gap_lds_max_count = env_int("DUHL_GAP_LDS_MAX_COUNT", 49152);
    c->cd_guard = env_int("DUHL_CD_GUARD", 1);
    c->keep_first_pass = env_int("DUHL_KEEP_FIRST_PASS", 1);
    c->guard_tol = 1e-6;
    // From alpha = 0 every coordinate of a Lasso moves, by steps of any size, and the first concurrent
    // pass is the one that overshoots: it starts with half the bound.  The steps of the SVM dual are
    // clipped to the box and its first passes were never seen to overshoot: full bound.
    c->guard_start = env_int("DUHL_GUARD_START", model == DUHL_SVM ? 0 : 1);
    c->select_spin_limit = env_int("DUHL_SELECT_SPIN_LIMIT", 1 << 22);
    if (c->select_spin_limit < 0) c->select_spin_limit = 0;
    c->select_groups = env_int("DUHL_SELECT_GROUPS", 0);
    c->csr_blocked = env_int("DUHL_CSR_BLOCKED", 1);
    c->csr_blocked_waves = env_int("DUHL_CSR_BLOCKED_WAVES", 2);
    if (c->csr_blocked_waves < 1) c->csr_blocked_waves = 1;
    c->csr_blocked_list_min = env_int("DUHL_CSR_BLOCKED_LIST_MIN", -1);

    c->partials_cap = n / 4 + 4096;
    c->blk_cap = (n + 2047) / 2048 + 1;
    hipError_t e = hipSuccess;
    auto ok = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    ok(dev_alloc(&c->alpha, n));
    ok(dev_alloc(&c->v, d + 4));
    ok(dev_alloc(&c->z, n));
    ok(dev_alloc(&c->q, n));
    ok(dev_alloc(&c->P_cur, c->budget));
    ok(dev_alloc(&c->P_next, c->budget));
    ok(dev_alloc(&c->scalars, (int64_t)S_COUNT));
    ok(dev_alloc(&c->partials, c->partials_cap));
    ok(dev_alloc(&c->sel, (int64_t)1));
    ok(dev_alloc(&c->blk_gt, c->blk_cap));
    ok(dev_alloc(&c->blk_eq, c->blk_cap));
    ok(dev_alloc(&c->mark, n));
    ok(hipHostMalloc(reinterpret_cast<void **>(&c->h_scalars), sizeof(double) * S_COUNT, hipHostMallocDefault));
    ok(hipHostMalloc(reinterpret_cast<void **>(&c->h_u32), sizeof(uint32_t) * 4, hipHostMallocDefault));
    if (e == hipSuccess) e = hipMemset(c->sel, 0, sizeof(SelectState));
    // working-set lists only ever hold coordinates: zero now, and a selection that ends early (a
    // device-side wait that timed out) leaves older valid entries behind, never garbage
    if (e == hipSuccess) e = hipMemset(c->P_cur, 0, sizeof(int32_t) * (size_t)c->budget);
    if (e == hipSuccess) e = hipMemset(c->P_next, 0, sizeof(int32_t) * (size_t)c->budget);
    if (e != hipSuccess) {
        duhl_destroy(c);
        return e == hipErrorOutOfMemory ? DUHL_ENOMEM : DUHL_EHIP;
    }
    *out = c;
    return DUHL_OK;
}

duhl_status duhl_set_eta(duhl_ctx *c, double eta)
{
    if (!c) return DUHL_EINVAL;
    if (c->model != DUHL_ELASTIC_NET) return fail(c, DUHL_EINVAL, "eta applies to DUHL_ELASTIC_NET only");
    if (!(eta > 0.0) || !(eta <= 1.0)) return fail(c, DUHL_EINVAL, "eta must be in (0, 1]");
    c->eta = eta;
    c->z_fresh = false;
    return DUHL_OK;
}

duhl_status duhl_set_wait_limit(duhl_ctx *c, int64_t polls)
{
    if (!c) return DUHL_EINVAL;
    if (polls < 0 || polls > 0x7fffffffll) return fail(c, DUHL_EINVAL, "polls must be in [0, 2^31)");
    c->cd_spin_limit = c->select_spin_limit = (int)polls;
    return DUHL_OK;
}

duhl_status duhl_set_data_dense(duhl_ctx *c, const float *A, int64_t ld, duhl_residency res,
                                const float *target, double lambda)
{
    duhl_status st = check_common(c, target, lambda);
    if (st != DUHL_OK) return st;
    if (!A) return fail(c, DUHL_EINVAL, "A is NULL");
    if (ld < c->d) return fail(c, DUHL_EINVAL, "ld (%lld) < d (%lld)", (long long)ld, (long long)c->d);
    if (res != DUHL_RESIDENT_DEVICE && res != DUHL_RESIDENT_HOST && res != DUHL_RESIDENT_HOST_PAGEABLE)
        return fail(c, DUHL_EINVAL, "bad residency");
    return set_data_dense_pieces(c, &A, 1, c->n, ld, res, target, lambda);
}

duhl_status duhl_set_data_dense_chunks(duhl_ctx *c, const float *const *chunks, int64_t n_chunks,
                                       int64_t cols_per_chunk, int64_t ld, const float *target,
                                       double lambda)
{
    duhl_status st = check_common(c, target, lambda);
    if (st != DUHL_OK) return st;
    if (!chunks) return fail(c, DUHL_EINVAL, "chunks is NULL");
    if (ld < c->d) return fail(c, DUHL_EINVAL, "ld (%lld) < d (%lld)", (long long)ld, (long long)c->d);
    if (cols_per_chunk < 1 || n_chunks < 1 || n_chunks != (c->n + cols_per_chunk - 1) / cols_per_chunk)
        return fail(c, DUHL_EINVAL, "need cols_per_chunk >= 1 and n_chunks == ceil(n / cols_per_chunk)");
    for (int64_t k = 0; k < n_chunks; ++k)
        if (!chunks[k]) return fail(c, DUHL_EINVAL, "chunk %lld is NULL", (long long)k);
    return set_data_dense_pieces(c, chunks, n_chunks, cols_per_chunk, ld, DUHL_RESIDENT_HOST, target, lambda);
}

duhl_status duhl_set_data_csr(duhl_ctx *c, const int64_t *rowptr, const int32_t *colidx,
                              const float *val, duhl_residency res, const float *target, double lambda)
{
    duhl_status st = check_common(c, target, lambda);
    if (st != DUHL_OK) return st;
    if (!rowptr || !colidx || !val) return fail(c, DUHL_EINVAL, "CSR array is NULL");
    if (res != DUHL_RESIDENT_DEVICE)
        return fail(c, DUHL_EINVAL, "sparse data must be device-resident");
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    HIPCHK(c, hipStreamSynchronize(c->copy));       // column copies of a pending selection
    c->have_data = false;
    free_host_residency(c);
    c->sparse = true;
    c->res = res;
    c->cv = ColView{};
    c->cv.rowptr = rowptr;
    c->cv.colidx = colidx;
    c->cv.val = val;
    c->ld_s = 0;
    int64_t last = 0;
    HIPCHK(c, hipMemcpy(&last, rowptr + c->n, sizeof(int64_t), hipMemcpyDeviceToHost));
    if (last < 0) return fail(c, DUHL_EINVAL, "rowptr[n] is negative");
    c->nnz = last;
    st = finish_set_data(c, target, lambda);
    if (st != DUHL_OK) return st;
    HIPCHK(c, csr_blocked_build(c));
    return DUHL_OK;
}

duhl_status duhl_gap(duhl_ctx *c, const int32_t *idx, int64_t count, double *gap_sum)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    if (idx && (count < 0 || count > c->n)) return fail(c, DUHL_EINVAL, "count out of range");
    if (!idx && c->z_fresh) {                       // nothing has moved since set_data's own full pass
        if (gap_sum) *gap_sum = c->z_fresh_sum;
        return DUHL_OK;
    }
    HIPCHK(c, hipSetDevice(c->device));
    if (idx)
        HIPCHK(c, launch_gap(c, idx, count, false, false));
    else if (c->res == DUHL_RESIDENT_HOST)
        HIPCHK(c, launch_gap(c, nullptr, c->budget, true, false));
    else
        HIPCHK(c, launch_gap(c, nullptr, c->n, false, false));
    if (gap_sum) {
        duhl_status st = read_scalars(c, S_GAP_SUM, 1);
        if (st != DUHL_OK) return st;
        *gap_sum = c->h_scalars[S_GAP_SUM];
    }
    return DUHL_OK;
}

duhl_status duhl_select_rule_apply(duhl_ctx *c, duhl_select_rule rule, uint64_t arg, int64_t m,
                                   int32_t *P_out, int64_t *n_swapped, double *rho)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    if (rule != DUHL_SELECT_GAP && rule != DUHL_SELECT_RANDOM && rule != DUHL_SELECT_BLOCK)
        return fail(c, DUHL_EINVAL, "unknown selection rule");
    if (m < 1 || m > c->n) return fail(c, DUHL_EINVAL, "m must be in [1, n]");
    if (m > c->budget) return fail(c, DUHL_EBUDGET, "m (%lld) exceeds the column budget (%lld)",
                                   (long long)m, (long long)c->budget);
    const bool host = c->res == DUHL_RESIDENT_HOST;
    if (host && c->pending)
        return fail(c, DUHL_ESTATE, "the previous selection has not been committed");
    HIPCHK(c, hipSetDevice(c->device));
    const float *keys = c->z;
    if (rule != DUHL_SELECT_GAP) {
        if (!c->score) HIPCHK(c, dev_alloc(&c->score, c->n));
        HIPCHK(c, launch_score(c, (int)rule, m, arg));
        keys = c->score;
    }
    HIPCHK(c, launch_select(c, m, P_out, keys));
    c->m_next = m;
    c->pending = true;
    const bool overlap_safe = c->budget >= c->m_cur + m;
    c->swap_exclusive = host && !overlap_safe;
    HIPCHK(c, launch_plan_swap(c, host ? overlap_safe : true, n_swapped != nullptr));
    if (host) {
        HIPCHK(c, hipEventRecord(c->ev_plan, c->compute));
        HIPCHK(c, hipStreamWaitEvent(c->copy, c->ev_plan, 0));
        HIPCHK(c, hipEventRecord(c->ev_copy_begin, c->copy));
        c->swap_timed = true;
        if (c->pageable) {
            // the host must gather the columns: the plan comes back (this waits for the compute
            // stream), then a background thread stages them and enqueues the copies
            HIPCHK(c, stager_swap_begin(c));
        } else {
            HIPCHK(c, launch_copy_columns(c));
            HIPCHK(c, hipEventRecord(c->ev_copy, c->copy));
        }
    }
    if (n_swapped || rho) {
        HIPCHK(c, hipMemcpyAsync(c->h_u32, &c->sel->n_fill, sizeof(uint32_t), hipMemcpyDeviceToHost,
                                 c->compute));
        static_assert(S_SUM_SEL == S_SUM_ALL + 1 && S_RHO == S_SUM_ALL + 2, "read back as one block");
        duhl_status st = read_scalars(c, S_SUM_ALL, 3);      // sum of all keys' gaps, of the set's, rho
        if (st != DUHL_OK) return st;
        if (n_swapped) *n_swapped = (int64_t)c->h_u32[0];
        if (rho) *rho = c->h_scalars[S_RHO];
    }
    return DUHL_OK;
}

duhl_status duhl_select(duhl_ctx *c, int64_t m, int32_t *P_out, int64_t *n_swapped, double *rho)
{
    return duhl_select_rule_apply(c, DUHL_SELECT_GAP, 0, m, P_out, n_swapped, rho);
}

duhl_status duhl_commit_swap(duhl_ctx *c)
{
    if (!c) return DUHL_EINVAL;
    if (!c->pending) return fail(c, DUHL_ESTATE, "no selection is pending");
    HIPCHK(c, hipSetDevice(c->device));
    if (c->res == DUHL_RESIDENT_HOST) {
        if (c->pageable) HIPCHK(c, stager_swap_join(c));   // every copy is enqueued, ev_copy recorded
        HIPCHK(c, hipStreamWaitEvent(c->compute, c->ev_copy, 0));
        HIPCHK(c, launch_publish(c));
    }
    int32_t *t = c->P_cur;
    c->P_cur = c->P_next;
    c->P_next = t;
    c->m_cur = c->m_next;
    c->pending = c->swap_exclusive = false;
    return DUHL_OK;
}

duhl_status duhl_cd_epoch(duhl_ctx *c, duhl_cd_mode mode, const int32_t *order, int64_t n_order,
                          uint64_t seed, int max_inflight)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    if (mode != DUHL_CD_SEQUENTIAL && mode != DUHL_CD_ASYNC && mode != DUHL_CD_ATOMIC)
        return fail(c, DUHL_EINVAL, "bad mode");
    if (c->m_cur <= 0) return fail(c, DUHL_ESTATE, "no working set: call duhl_select and duhl_commit_swap");
    if (c->pending && c->swap_exclusive)
        return fail(c, DUHL_ESTATE, "the working set is being replaced in place: call duhl_commit_swap first");
    if (order && n_order < 0) return fail(c, DUHL_EINVAL, "n_order is negative");
    if (max_inflight < 0) return fail(c, DUHL_EINVAL, "max_inflight is negative");
    HIPCHK(c, hipSetDevice(c->device));
    c->z_fresh = false;
    HIPCHK(c, launch_cd(c, mode, order, n_order, seed, max_inflight));
    c->pass_counter++;
    return DUHL_OK;
}

duhl_status duhl_cd_stats(duhl_ctx *c, int64_t *passes_damped, int64_t *inflight_now, int64_t *steps_kept,
                          double *last_theta)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    if (passes_damped) *passes_damped = c->h_trips ? (int64_t)*static_cast<volatile uint32_t *>(c->h_trips) : 0;
    if (inflight_now) *inflight_now = c->m_cur > 0 ? default_inflight(c, c->m_cur) : 0;
    if (steps_kept) *steps_kept = 0;
    if (last_theta) *last_theta = 1.0;
    if ((steps_kept || last_theta) && c->guard) {
        GuardState gs;
        HIPCHK(c, hipMemcpy(&gs, c->guard, sizeof gs, hipMemcpyDeviceToHost));
        if (steps_kept) *steps_kept = (int64_t)gs.steps_kept;
        if (last_theta && gs.steps_kept + gs.trips > 0) *last_theta = gs.last_theta;
    }
    return DUHL_OK;
}

duhl_status duhl_objective(duhl_ctx *c, double *objective)
{
    if (!c) return DUHL_EINVAL;
    if (!objective) return fail(c, DUHL_EINVAL, "objective is NULL");
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, launch_objective(c));
    duhl_status st = read_scalars(c, S_OBJ_SQ, 2);
    if (st != DUHL_OK) return st;
    const double sq = c->h_scalars[S_OBJ_SQ], lin = c->h_scalars[S_OBJ_LIN];
    const double d = (double)c->d, n = (double)c->n;
    if (c->model != DUHL_SVM)
        *objective = sq / (2.0 * d) + c->lambda * lin;             // Appendix C (a), (b); Appendix D
    else
        *objective = -lin / n + sq / (2.0 * c->lambda * n * n);    // Appendix C (c)
    return DUHL_OK;
}

duhl_status duhl_recompute_v(duhl_ctx *c)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    HIPCHK(c, hipSetDevice(c->device));
    c->z_fresh = false;
    HIPCHK(c, launch_init_v(c));
    HIPCHK(c, launch_accumulate_v(c));
    return DUHL_OK;
}

duhl_status duhl_probe_stream_read(duhl_ctx *c, const void *dev, int64_t bytes, int reps, double *best_ms)
{
    if (!c) return DUHL_EINVAL;
    if (!dev || !best_ms || bytes <= 0 || bytes % 16 != 0 || reps < 1 ||
        (reinterpret_cast<uintptr_t>(dev) & 15) != 0)
        return fail(c, DUHL_EINVAL, "probe: need a 16-byte aligned device pointer, bytes % 16 == 0, reps >= 1");
    HIPCHK(c, hipSetDevice(c->device));
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0));
    HIPCHK(c, hipEventCreate(&e1));
    float *sink = reinterpret_cast<float *>(c->scalars + S_SINK);
    double best = 0.0;
    duhl_status st = DUHL_OK;
    for (int r = 0; r <= reps && st == DUHL_OK; ++r) {         // first launch is a warm-up
        hipError_t e = hipEventRecord(e0, c->compute);
        if (e == hipSuccess) e = launch_stream_read(c, dev, bytes, sink);
        if (e == hipSuccess) e = hipEventRecord(e1, c->compute);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) st = fail(c, DUHL_EHIP, "probe: %s", hipGetErrorString(e));
        else if (r > 0 && (best == 0.0 || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st == DUHL_OK) *best_ms = best;
    return st;
}

duhl_status duhl_probe_scatter_add(duhl_ctx *c, int64_t ops, int reps, double *adds_per_s)
{
    if (!c) return DUHL_EINVAL;
    if (!adds_per_s || ops < 1 || reps < 1) return fail(c, DUHL_EINVAL, "probe: need ops >= 1, reps >= 1 and a result pointer");
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data set");
    HIPCHK(c, hipSetDevice(c->device));
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0));
    HIPCHK(c, hipEventCreate(&e1));
    double best = 0.0;
    int64_t done = 0;
    duhl_status st = DUHL_OK;
    for (int r = 0; r <= reps && st == DUHL_OK; ++r) {         // first launch is a warm-up
        hipError_t e = hipEventRecord(e0, c->compute);
        if (e == hipSuccess) e = launch_scatter_add(c, ops, &done);
        if (e == hipSuccess) e = hipEventRecord(e1, c->compute);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) st = fail(c, DUHL_EHIP, "probe: %s", hipGetErrorString(e));
        else if (r > 0 && (best == 0.0 || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st == DUHL_OK) *adds_per_s = best > 0.0 ? (double)done / (best * 1e-3) : 0.0;
    return st;
}

static duhl_status locate(duhl_ctx *c, duhl_what what, void **ptr, int64_t *len, size_t *elem)
{
    *elem = 4;
    switch (what) {
    case DUHL_ALPHA: *ptr = c->alpha; *len = c->n; break;
    case DUHL_V: *ptr = c->v; *len = c->d; break;
    case DUHL_Z: *ptr = c->z; *len = c->n; break;
    case DUHL_SQNORM: *ptr = c->q; *len = c->n; break;
    case DUHL_P: *ptr = c->P_cur; *len = c->m_cur; break;
    default: return fail(c, DUHL_EINVAL, "unknown array id");
    }
    return DUHL_OK;
}

duhl_status duhl_get(duhl_ctx *c, duhl_what what, void *dst, int64_t len)
{
    if (!c) return DUHL_EINVAL;
    if (!dst) return fail(c, DUHL_EINVAL, "dst is NULL");
    void *p; int64_t n; size_t el;
    duhl_status st = locate(c, what, &p, &n, &el);
    if (st != DUHL_OK) return st;
    if (len != n) return fail(c, DUHL_EINVAL, "len (%lld) must be %lld", (long long)len, (long long)n);
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    if (n > 0) HIPCHK(c, hipMemcpy(dst, p, el * (size_t)n, hipMemcpyDeviceToHost));
    return DUHL_OK;
}

duhl_status duhl_set(duhl_ctx *c, duhl_what what, const void *src, int64_t len)
{
    if (!c) return DUHL_EINVAL;
    if (!src) return fail(c, DUHL_EINVAL, "src is NULL");
    if (what != DUHL_ALPHA && what != DUHL_V && what != DUHL_Z)
        return fail(c, DUHL_EINVAL, "only alpha, v and z can be set");
    void *p; int64_t n; size_t el;
    duhl_status st = locate(c, what, &p, &n, &el);
    if (st != DUHL_OK) return st;
    if (len != n) return fail(c, DUHL_EINVAL, "len (%lld) must be %lld", (long long)len, (long long)n);
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    c->z_fresh = false;
    HIPCHK(c, hipMemcpy(p, src, el * (size_t)n, hipMemcpyHostToDevice));
    return DUHL_OK;
}

duhl_status duhl_device_ptr(duhl_ctx *c, duhl_what what, void **ptr)
{
    if (!c) return DUHL_EINVAL;
    if (!ptr) return fail(c, DUHL_EINVAL, "ptr is NULL");
    void *p; int64_t n; size_t el;
    duhl_status st = locate(c, what, &p, &n, &el);
    if (st != DUHL_OK) return st;
    if (what == DUHL_ALPHA || what == DUHL_V || what == DUHL_Z) {   // the caller may write through it
        c->ptr_escaped = true;
        c->z_fresh = false;
    }
    *ptr = p;
    return DUHL_OK;
}

int64_t duhl_working_set_size(const duhl_ctx *c) { return c ? c->m_cur : 0; }

duhl_status duhl_swap_stats(duhl_ctx *c, int64_t *columns, double *copy_ms)
{
    if (!c) return DUHL_EINVAL;
    if (!columns || !copy_ms) return fail(c, DUHL_EINVAL, "columns or copy_ms is NULL");
    if (!c->have_data || c->res != DUHL_RESIDENT_HOST) return fail(c, DUHL_ESTATE, "no host-resident data");
    if (c->pending) return fail(c, DUHL_ESTATE, "a selection is pending: call duhl_commit_swap first");
    if (!c->swap_timed) return fail(c, DUHL_ESTATE, "no selection yet");
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->copy));
    uint32_t n_fill = 0;
    HIPCHK(c, hipMemcpyAsync(&n_fill, &c->sel->n_fill, sizeof(n_fill), hipMemcpyDeviceToHost, c->compute));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    float ms = 0.0f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->ev_copy_begin, c->ev_copy));
    *columns = (int64_t)n_fill;
    *copy_ms = (double)ms;
    return DUHL_OK;
}

duhl_status duhl_resident_columns(duhl_ctx *c, int64_t *count)
{
    if (!c) return DUHL_EINVAL;
    if (!count) return fail(c, DUHL_EINVAL, "count is NULL");
    if (!c->have_data) return fail(c, DUHL_ESTATE, "no data");
    if (c->res != DUHL_RESIDENT_HOST) {
        *count = c->n;
        return DUHL_OK;
    }
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    int32_t *host = static_cast<int32_t *>(malloc((size_t)c->budget * sizeof(int32_t)));
    if (!host) return fail(c, DUHL_ENOMEM, "host allocation failed");
    const hipError_t e = hipMemcpy(host, c->slot_col, (size_t)c->budget * sizeof(int32_t), hipMemcpyDeviceToHost);
    int64_t used = 0;
    for (int64_t s = 0; e == hipSuccess && s < c->budget; ++s) used += host[s] >= 0;
    free(host);
    HIPCHK(c, e);
    *count = used;
    return DUHL_OK;
}

duhl_status duhl_selection_threshold(duhl_ctx *c, float *threshold)
{
    if (!c) return DUHL_EINVAL;
    if (!threshold) return fail(c, DUHL_EINVAL, "threshold is NULL");
    if (!c->have_data || (!c->pending && c->m_cur == 0)) return fail(c, DUHL_ESTATE, "no selection yet");
    HIPCHK(c, hipSetDevice(c->device));
    uint32_t key = 0;
    HIPCHK(c, hipMemcpyAsync(&key, &c->sel->thr_key, sizeof(key), hipMemcpyDeviceToHost, c->compute));
    HIPCHK(c, hipStreamSynchronize(c->compute));
    // keys order floats as unsigned integers: sign bit set for non-negative values, all bits
    // inverted for negative ones
    const uint32_t bits = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    float out;
    memcpy(&out, &bits, sizeof(out));
    *threshold = out;
    return DUHL_OK;
}

const char *duhl_last_error(const duhl_ctx *c) { return c ? c->err.c_str() : "null context"; }

void duhl_destroy(duhl_ctx *c)
{
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->compute);
    (void)hipStreamSynchronize(c->copy);
    free_host_residency(c);
    (void)hipFree(c->alpha); (void)hipFree(c->v); (void)hipFree(c->z); (void)hipFree(c->q);
    (void)hipFree(c->P_cur); (void)hipFree(c->P_next);
    (void)hipFree(c->scalars); (void)hipFree(c->partials); (void)hipFree(c->sel);
    (void)hipFree(c->blk_gt); (void)hipFree(c->blk_eq); (void)hipFree(c->mark);
    (void)hipFree(c->dv); (void)hipFree(c->dirty); (void)hipFree(c->score); (void)hipFree(c->xch);
    (void)hipFree(c->cd_plan);
    (void)hipFree(c->guard_wbook);
    (void)hipFree(c->gap_pdot);
    (void)hipFree(c->guard); (void)hipFree(c->guard_part); (void)hipFree(c->snap_pass_v); (void)hipFree(c->alpha_old);
    if (c->h_trips) (void)hipHostFree(c->h_trips);
    for (hipEvent_t ev : c->ev_pass)
        if (ev) (void)hipEventDestroy(ev);
    (void)hipFree(c->snap_alpha); (void)hipFree(c->snap_v);
    if (c->h_scalars) (void)hipHostFree(c->h_scalars);
    if (c->h_u32) (void)hipHostFree(c->h_u32);
    delete c;
}

}  // extern "C"
