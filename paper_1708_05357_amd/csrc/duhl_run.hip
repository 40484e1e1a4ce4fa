// The outer loop (Algorithm 1; Algorithm 2 when the gap memory is allowed to go stale): rounds of
// gap refresh -> working-set selection -> passes over the working set, driven from native code so
// that nothing but kernel launches sits between the steps.  It only sequences the library's own
// entry points; all arithmetic stays in their kernels.
#include <chrono>
#include <cmath>

#include "duhl_internal.h"

namespace {

duhl_status set_error(duhl_ctx *c, duhl_status st, const char *text)
{
    c->err = text;
    return st;
}

// Every gap at the current point, wherever the column lives (slot, device or host memory), and
// their sum: the duality gap of eq. (2).  With host residency this is a pass over the host link.
duhl_status refresh_all(duhl_ctx *c, double *total)
{
    hipError_t e = duhl::launch_gap(c, nullptr, c->n, false, false);
    if (e == hipSuccess)
        e = hipMemcpyAsync(c->h_scalars + duhl::S_GAP_SUM, c->scalars + duhl::S_GAP_SUM, sizeof(double),
                           hipMemcpyDeviceToHost, c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) return set_error(c, DUHL_EHIP, hipGetErrorString(e));
    *total = c->h_scalars[duhl::S_GAP_SUM];
    return DUHL_OK;
}

// Keep (restore == false) or bring back (restore == true) the iterate: alpha and v, on the compute stream.
duhl_status snapshot(duhl_ctx *c, bool restore)
{
    hipError_t e = hipSuccess;
    if (!c->snap_alpha) e = hipMalloc(reinterpret_cast<void **>(&c->snap_alpha), sizeof(float) * (size_t)c->n);
    if (e == hipSuccess && !c->snap_v) e = hipMalloc(reinterpret_cast<void **>(&c->snap_v), sizeof(float) * (size_t)c->d);
    if (e == hipSuccess)
        e = hipMemcpyAsync(restore ? c->alpha : c->snap_alpha, restore ? c->snap_alpha : c->alpha,
                           sizeof(float) * (size_t)c->n, hipMemcpyDeviceToDevice, c->compute);
    if (e == hipSuccess)
        e = hipMemcpyAsync(restore ? c->v : c->snap_v, restore ? c->snap_v : c->v, sizeof(float) * (size_t)c->d,
                           hipMemcpyDeviceToDevice, c->compute);
    if (e != hipSuccess) return set_error(c, e == hipErrorOutOfMemory ? DUHL_ENOMEM : DUHL_EHIP, hipGetErrorString(e));
    if (restore) c->z_fresh = false;
    return DUHL_OK;
}

// Entries [start, start + len) of a list of `total` entries, wrapping at the end: at most two runs.
template <typename F>
duhl_status for_window(int64_t total, int64_t start, int64_t len, F &&f)
{
    start %= total;
    const int64_t first = len < total - start ? len : total - start;
    duhl_status st = f(start, first);
    if (st == DUHL_OK && len > first) st = f(0, len - first);
    return st;
}

}  // namespace

extern "C" duhl_status duhl_run(duhl_ctx *c, const duhl_run_opts *o, duhl_run_stats *out)
{
    if (!c) return DUHL_EINVAL;
    if (!o || !out) return set_error(c, DUHL_EINVAL, "options or statistics pointer is NULL");
    if (!c->have_data) return set_error(c, DUHL_ESTATE, "no data set");
    if (o->passes < 0 || o->max_rounds < 0 || o->check_every < 0 || o->max_inflight < 0 || o->max_extra_passes < 0)
        return set_error(c, DUHL_EINVAL,
                         "passes >= 0, max_rounds >= 0, check_every >= 0, max_inflight >= 0, max_extra_passes >= 0 required");
    if (std::isnan(o->gap_tol)) return set_error(c, DUHL_EINVAL, "gap_tol is NaN");
    const bool host = c->res == DUHL_RESIDENT_HOST;
    const bool threads = o->host_threads > 0;
    if (threads && (!host || !o->sample_host))
        return set_error(c, DUHL_EINVAL, "host threads need DUHL_RESIDENT_HOST data and sample_host");
    const bool sampled = threads ? true : o->sample_dev != nullptr;
    if (sampled && (o->sample_len < 1 || o->sample_per_round < 1 || o->sample_per_round > o->sample_len ||
                    o->sample_len > c->n))
        return set_error(c, DUHL_EINVAL, "need 1 <= sample_per_round <= sample_len <= n");
    if (c->pending) return set_error(c, DUHL_ESTATE, "a selection is pending: call duhl_commit_swap first");
    const int check_every = o->check_every > 0 ? o->check_every : 1;

    duhl_run_stats s{};
    const auto t0 = std::chrono::steady_clock::now();
    duhl_status st = DUHL_OK;
    int64_t cursor = 0;                                     // where the next sample window starts
    int64_t swept = 0;                                      // list entries refreshed since the last full refresh
    int inflight = o->max_inflight;                         // 0: the library's own bound
    double good_objective = 0.0;
    bool have_good = false;
    // passes per round; 0 in the options: one in the first round, whose two phases are timed, then
    // by the rule stated with the options (host residency: 8, the passes are also the time unit A's
    // threads and the column copies have)
    int passes = o->passes > 0 ? o->passes : (host ? 8 : 1);
    bool timing = o->passes == 0 && !host;
    struct Events {                                         // destroyed on every way out
        hipEvent_t e[3] = {nullptr, nullptr, nullptr};
        ~Events()
        {
            for (hipEvent_t x : e)
                if (x) (void)hipEventDestroy(x);
        }
    } events;
    hipEvent_t *ev = events.e;
    if (timing)
        for (int k = 0; k < 3; ++k)
            if (hipEventCreate(&ev[k]) != hipSuccess) timing = false;
    for (int64_t rnd = 0; rnd < o->max_rounds; ++rnd) {
        if (timing && rnd == 0 && hipEventRecord(ev[0], c->compute) != hipSuccess) timing = false;
        // -- guard of the concurrent passes ----------------------------------------------------
        // Exact coordinate steps never raise the objective; steps taken concurrently can, when the
        // columns worked on at once are more alike than the bound on their number assumed (e.g. a
        // selection that gathers near-duplicate columns).  So the objective is looked at on every
        // checked round: if it rose, the iterate goes back to the last good one and the bound is halved.
        if (o->adapt_inflight && o->mode != DUHL_CD_SEQUENTIAL && rnd % check_every == 0) {
            double obj = 0.0;
            st = duhl_objective(c, &obj);
            if (st != DUHL_OK) return st;
            const bool fine = !have_good || (std::isfinite(obj) && obj <= good_objective + 1e-6 * std::fabs(good_objective) + 1e-30);
            if (fine) {
                st = snapshot(c, false);
                good_objective = obj;
                have_good = true;
            } else {
                st = snapshot(c, true);
                const int64_t now = inflight > 0 ? inflight : duhl::default_inflight(c, o->m);
                inflight = (int)(now / 2 > 1 ? now / 2 : 1);
                s.inflight_halvings++;
            }
            if (st != DUHL_OK) return st;
        }
        // -- refresh the gap memory (Section 4.1) --------------------------------------------
        if (!host && !sampled) {
            st = duhl_gap(c, nullptr, 0, nullptr);          // every coordinate: eq. (11) exactly
        } else {
            // what was just worked on, from device memory: residents / the current working set
            if (host) st = duhl_gap(c, nullptr, 0, nullptr);
            else if (c->m_cur > 0) st = duhl_gap(c, c->P_cur, c->m_cur, nullptr);
            else st = duhl_gap(c, nullptr, 0, nullptr);     // first round: no set yet, all are fresh
            if (st == DUHL_OK && sampled && !threads) {
                st = for_window(o->sample_len, cursor, o->sample_per_round, [&](int64_t a, int64_t len) {
                    return duhl_gap(c, o->sample_dev + a, len, nullptr);
                });
                cursor = (cursor + o->sample_per_round) % o->sample_len;
                swept += o->sample_per_round;
            }
        }
        if (st != DUHL_OK) return st;

        // -- select; the sum of the gap memory comes with it ---------------------------------
        const bool check = rnd % check_every == 0;
        int64_t nsw = 0;
        double rho = 1.0;
        st = duhl_select_rule_apply(c, o->rule, o->seed + (uint64_t)rnd, o->m, nullptr,
                                    check ? &nsw : nullptr, check ? &rho : nullptr);
        if (st != DUHL_OK) return st;
        if (check) {
            s.gap_memory_sum = c->h_scalars[duhl::S_SUM_ALL];   // read back together with rho
            s.rho = rho;
            s.columns_swapped += nsw;
            // With a stale gap memory the sum is only an estimate, and a poor one before every
            // listed entry has been refreshed at least once: entries still hold their values from
            // the starting point (for the Lasso most of those are exactly zero).
            bool reached = s.gap_memory_sum <= o->gap_tol && (!sampled || swept >= o->sample_len);
            // host residency without a sample list: only the columns in device slots are ever
            // refreshed, the rest keep the values of the starting point, so the sum says nothing
            // about them -- it is always confirmed by a full refresh before the loop ends on it
            const bool must_confirm = sampled ? o->confirm != 0 : host;
            if (reached && must_confirm) {
                // make every entry fresh at the current point and test the true total gap
                st = duhl_commit_swap(c);
                if (st != DUHL_OK) return st;
                double total = 0.0;
                st = refresh_all(c, &total);
                if (st != DUHL_OK) return st;
                s.confirmations++;
                s.gap_memory_sum = total;
                swept = sampled ? o->sample_len : 0;
                if (total <= o->gap_tol) {
                    s.converged = 1;
                    break;
                }
                continue;                                   // next round selects from the fresh memory
            }
            if (reached) {
                // done: the selection just made becomes the current set, nothing stays pending
                st = duhl_commit_swap(c);
                if (st != DUHL_OK) return st;
                s.converged = 1;
                break;
            }
        }
        // -- passes over the working set, next to the column copies when they may overlap ----
        if (timing && rnd == 0 && hipEventRecord(ev[1], c->compute) != hipSuccess) timing = false;
        const bool overlap = host && c->m_cur > 0 && !c->swap_exclusive;
        if (!overlap) {
            st = duhl_commit_swap(c);
            if (st != DUHL_OK) return st;
        }
        int64_t begun = 0;
        if (threads) {
            begun = o->sample_per_round;
            if (cursor + begun > o->sample_len) begun = o->sample_len - cursor;   // no wrap inside a round
            st = duhl_host_sample_begin(c, o->sample_host + cursor, begun, o->host_threads);
            if (st != DUHL_OK) return st;
        }
        for (int k = 0; k < passes && st == DUHL_OK; ++k)
            st = duhl_cd_epoch(c, o->mode, nullptr, 0, o->seed + (uint64_t)(rnd * 64 + k), inflight);
        if (timing && rnd == 0 && st == DUHL_OK) {
            float g_ms = 0.0f, c_ms = 0.0f;
            if (hipEventRecord(ev[2], c->compute) == hipSuccess && hipEventSynchronize(ev[2]) == hipSuccess &&
                hipEventElapsedTime(&g_ms, ev[0], ev[1]) == hipSuccess &&
                hipEventElapsedTime(&c_ms, ev[1], ev[2]) == hipSuccess && c_ms > 0.0f) {
                const long t = std::lround(std::sqrt((double)g_ms / (double)c_ms)) + 1;
                passes = (int)(t < 1 ? 1 : (t > 8 ? 8 : t));
            }
            timing = false;
        }
        // theta sized to the copy: unit B works on while its next working set is still arriving.  One
        // pass at a time, each waited for, so that the host does not enqueue passes for longer than
        // the copies last.
        int extra = 0;
        while (overlap && st == DUHL_OK && extra < o->max_extra_passes) {
            if (hipStreamSynchronize(c->compute) != hipSuccess) { st = DUHL_EHIP; break; }
            if (!duhl::swap_in_flight(c)) break;
            st = duhl_cd_epoch(c, o->mode, nullptr, 0,
                               (o->seed ^ 0x9e3779b97f4a7c15ull) + (uint64_t)(rnd * 1024 + extra), inflight);
            ++extra;
        }
        if (threads) {
            // unit A samples for as long as unit B works (Algorithm 2): until the passes and the copies are done
            if (st == DUHL_OK && hipStreamSynchronize(c->compute) != hipSuccess) st = DUHL_EHIP;
            if (st == DUHL_OK && hipStreamSynchronize(c->copy) != hipSuccess) st = DUHL_EHIP;
            int64_t done = 0;
            const duhl_status st2 = duhl_host_sample_end(c, o->host_wait_all ? 1 : 0, &done);
            if (st == DUHL_OK) st = st2;
            // the threads take the window's entries in order, so all but the few they were working
            // on when stopped form a prefix: the next window starts where that prefix ends
            int64_t adv = duhl::host_sampler_prefix(c);
            if (adv > begun) adv = begun;
            cursor = (cursor + adv) % o->sample_len;
            swept += adv;
            s.host_sampled += done;
        }
        if (st != DUHL_OK) return st;
        if (overlap) {
            st = duhl_commit_swap(c);
            if (st != DUHL_OK) return st;
        }
        s.rounds = rnd + 1;
        s.passes += (rnd == 0 && o->passes == 0 && !host ? 1 : passes) + extra;
    }
    if (hipStreamSynchronize(c->compute) != hipSuccess) return set_error(c, DUHL_EHIP, "stream synchronisation failed");
    s.inflight_last = inflight;
    s.passes_per_round = passes;
    s.seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    *out = s;
    return DUHL_OK;
}
