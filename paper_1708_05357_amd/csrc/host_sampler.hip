// Unit A's side of Algorithm 2 (its loop next to unit B's update step): while the GPU works on the
// current block, host threads refresh entries of the gap memory z from the matrix in host memory.
//
// duhl_host_sample_begin snapshots alpha and v at the current point of the compute stream (the
// iterate alpha^(t) of the listing), then starts threads that evaluate gap_j for the listed
// coordinates straight from the pinned host matrix -- the host link stays free for the column
// swap.  duhl_host_sample_end stops them (unit A samples only while unit B works), uploads what was refreshed and
// scatters it into z on the compute stream.  The arithmetic is single precision with eight
// partial sums per dot product, like the device kernels; the formulas are those of Appendix E.
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "duhl_internal.h"

struct duhl_host_sampler {
    // A pool of threads that lives as long as the context: a thread's first HIP call costs
    // milliseconds, far more than one sampling round, so threads are not created per round.
    std::vector<std::thread> threads;
    std::mutex mu;
    std::condition_variable cv_start, cv_done;
    int generation = 0, finished = 0;
    bool quit = false;
    std::atomic<int> stop{0};
    std::atomic<int64_t> next{0};   // next list entry to hand out: entries are claimed in list order
    int64_t prefix = 0;             // after a round: leading entries of the list that were all refreshed
    hipEvent_t snap = nullptr;
    float *h_alpha = nullptr, *h_v = nullptr, *h_target = nullptr;   // pinned snapshots
    float *h_z = nullptr;                                            // pinned results, one per list entry
    int32_t *h_idx = nullptr;                                        // pinned: coordinate, or -1 if not done
    float *d_z = nullptr;
    int32_t *d_idx = nullptr;
    int64_t cap = 0, count = 0;
    bool active = false;
    std::vector<const float *> touched;   // host pieces of the matrix whose pages were touched once
    std::vector<int32_t> *list = nullptr;   // coordinates of the running round
};

namespace duhl {

namespace {

__global__ void scatter_z_kernel(float *z, const int32_t *idx, const float *val, int64_t count)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count && idx[k] >= 0) z[idx[k]] = val[k];
}

// a^T v with eight independent partial sums (vectorises; fixed summation order).
float host_dot(const float *a, const float *v, int64_t d)
{
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int64_t k = 0;
    for (; k + 8 <= d; k += 8)
        for (int u = 0; u < 8; ++u) s[u] += a[k + u] * v[k + u];
    float t = 0.0f;
    for (; k < d; ++k) t += a[k] * v[k];
    return ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7])) + t;
}

// The coordinate gap of Appendix E from c = a_i^T v (same expressions as the device epilogue).
float host_gap_value(const ModelConst &mc, float c, float alpha, float y)
{
    float z;
    if (mc.model == DUHL_LASSO) {
        const float over = std::fmax(std::fabs(c) - mc.Lam, 0.0f);
        z = (std::fma(alpha, c, mc.Lam * std::fabs(alpha)) + mc.B * over) * mc.inv_d;
    } else if (mc.model == DUHL_ELASTIC_NET) {
        const float over = std::fmax(std::fabs(c) - mc.lam_l1, 0.0f);
        const float reg = std::fma(0.5f * mc.lam_eta * alpha, alpha, mc.lam_l1 * std::fabs(alpha));
        z = (std::fma(alpha, c, reg) + over * over * mc.inv_2lam_eta) * mc.inv_d;
    } else {
        const float s = c * mc.inv_lam_n;
        const float hinge = std::fmax(1.0f - y * s, 0.0f);
        z = (std::fma(alpha, s, hinge) - y * alpha) * mc.inv_n;
    }
    return z > 0.0f ? z : 0.0f;
}

// `seen`: the round counter at the time the thread was created; it works on later rounds only.
void sampler_thread(duhl_ctx *c, duhl_host_sampler *hs, int tid, int nthreads, int seen)
{
    (void)hipSetDevice(c->device);
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(hs->mu);
            hs->cv_start.wait(lk, [&] { return hs->quit || hs->generation != seen; });
            if (hs->quit) return;
            seen = hs->generation;
        }
        if (hipEventSynchronize(hs->snap) == hipSuccess) {        // snapshots are in host memory now
            const int64_t d = c->d;
            const std::vector<int32_t> &list = *hs->list;
            // entries are claimed one by one from a shared counter, so what is refreshed when the
            // round is stopped early is a prefix of the list but for the (at most one per thread)
            // entries still being worked on
            (void)tid;
            (void)nthreads;
            for (;;) {
                if (hs->stop.load(std::memory_order_relaxed)) break;
                const int64_t k = hs->next.fetch_add(1, std::memory_order_relaxed);
                if (k >= hs->count) break;
                const int32_t j = list[k];
                const float cj = host_dot(host_col(c, j), hs->h_v, d);
                const float y = c->model == DUHL_SVM ? hs->h_target[j] : 0.0f;
                hs->h_z[k] = host_gap_value(c->mc, cj, hs->h_alpha[j], y);
                hs->h_idx[k] = j;                                 // marks the entry as refreshed
            }
        }
        {
            std::lock_guard<std::mutex> lk(hs->mu);
            hs->finished++;
        }
        hs->cv_done.notify_all();
    }
}

// The CPU's first access to a page of pinned memory that only the GPU has written so far takes a
// minor page fault (measured: 2.5 GB/s per thread on first touch, >100 GB/s afterwards), so the
// matrix is touched once, one word per page, before the first sampling round.
void prefault(const float *A, int64_t floats, int nthreads)
{
    std::vector<std::thread> th;
    std::vector<float> sink(nthreads, 0.0f);
    const int64_t step = 4096 / sizeof(float);
    const int64_t pages = (floats + step - 1) / step;
    for (int t = 0; t < nthreads; ++t)
        th.emplace_back([=, &sink] {
            float s = 0.0f;
            const volatile float *p = A;
            for (int64_t g = pages * t / nthreads; g < pages * (t + 1) / nthreads; ++g) s += p[g * step];
            sink[t] = s;
        });
    for (auto &x : th) x.join();
}

void stop_pool(duhl_host_sampler *hs)
{
    {
        std::lock_guard<std::mutex> lk(hs->mu);
        hs->quit = true;
    }
    hs->cv_start.notify_all();
    for (auto &t : hs->threads) t.join();
    hs->threads.clear();
    hs->quit = false;
}

}  // namespace

int64_t host_sampler_prefix(const duhl_ctx *c) { return c->sampler ? c->sampler->prefix : 0; }

void host_sampler_destroy(duhl_ctx *c)
{
    duhl_host_sampler *hs = c->sampler;
    if (!hs) return;
    hs->stop.store(1);
    if (hs->active) {
        std::unique_lock<std::mutex> lk(hs->mu);
        hs->cv_done.wait(lk, [&] { return hs->finished == (int)hs->threads.size(); });
    }
    stop_pool(hs);
    if (hs->snap) (void)hipEventDestroy(hs->snap);
    if (hs->h_alpha) (void)hipHostFree(hs->h_alpha);
    if (hs->h_v) (void)hipHostFree(hs->h_v);
    if (hs->h_target) (void)hipHostFree(hs->h_target);
    if (hs->h_z) (void)hipHostFree(hs->h_z);
    if (hs->h_idx) (void)hipHostFree(hs->h_idx);
    (void)hipFree(hs->d_z);
    (void)hipFree(hs->d_idx);
    delete hs->list;
    delete hs;
    c->sampler = nullptr;
}

}  // namespace duhl

using namespace duhl;

#define HS_CHK(c, expr)                                                                        \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) {                                                                \
            (c)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                      \
            return e_ == hipErrorOutOfMemory ? DUHL_ENOMEM : DUHL_EHIP;                        \
        }                                                                                      \
    } while (0)

extern "C" duhl_status duhl_host_sample_begin(duhl_ctx *c, const int32_t *idx_host, int64_t count,
                                              int nthreads)
{
    if (!c) return DUHL_EINVAL;
    if (!c->have_data) { c->err = "no data set"; return DUHL_ESTATE; }
    if (c->sparse || c->res != DUHL_RESIDENT_HOST) {
        c->err = "the host sampler needs a dense matrix in host memory (DUHL_RESIDENT_HOST)";
        return DUHL_EINVAL;
    }
    if (!idx_host || count < 0 || nthreads < 1 || nthreads > 256) { c->err = "bad argument"; return DUHL_EINVAL; }
    for (int64_t k = 0; k < count; ++k)
        if (idx_host[k] < 0 || idx_host[k] >= c->n) { c->err = "coordinate out of range"; return DUHL_EINVAL; }
    HS_CHK(c, hipSetDevice(c->device));
    duhl_host_sampler *hs = c->sampler;
    if (hs && hs->active) { c->err = "a host sampling round is already running"; return DUHL_ESTATE; }
    if (!hs) {
        hs = new (std::nothrow) duhl_host_sampler();
        if (!hs) return DUHL_ENOMEM;
        c->sampler = hs;
        hs->list = new std::vector<int32_t>();
        hipError_t e = hipEventCreateWithFlags(&hs->snap, hipEventDisableTiming);
        if (e == hipSuccess)
            e = hipHostMalloc(reinterpret_cast<void **>(&hs->h_alpha), sizeof(float) * c->n, hipHostMallocDefault);
        if (e == hipSuccess)
            e = hipHostMalloc(reinterpret_cast<void **>(&hs->h_v), sizeof(float) * c->d, hipHostMallocDefault);
        if (e == hipSuccess && c->model == DUHL_SVM) {
            e = hipHostMalloc(reinterpret_cast<void **>(&hs->h_target), sizeof(float) * c->n, hipHostMallocDefault);
            if (e == hipSuccess)
                e = hipMemcpy(hs->h_target, c->target, sizeof(float) * c->n, hipMemcpyDeviceToHost);
        }
        if (e != hipSuccess) {                       // leave no half-built sampler behind
            host_sampler_destroy(c);
            c->err = std::string("host sampler set-up: ") + hipGetErrorString(e);
            return e == hipErrorOutOfMemory ? DUHL_ENOMEM : DUHL_EHIP;
        }
    }
    if (hs->touched != c->host_chunks) {
        hs->touched = c->host_chunks;
        for (size_t k = 0; k < hs->touched.size(); ++k) {
            const int64_t first = (int64_t)k * c->chunk_cols;
            const int64_t cols = c->n - first < c->chunk_cols ? c->n - first : c->chunk_cols;
            prefault(hs->touched[k], c->host_ld * (cols - 1) + c->d, nthreads);
        }
    }
    if (count > hs->cap) {
        if (hs->h_z) (void)hipHostFree(hs->h_z);
        if (hs->h_idx) (void)hipHostFree(hs->h_idx);
        (void)hipFree(hs->d_z);
        (void)hipFree(hs->d_idx);
        hs->h_z = nullptr; hs->h_idx = nullptr; hs->d_z = nullptr; hs->d_idx = nullptr; hs->cap = 0;
        HS_CHK(c, hipHostMalloc(reinterpret_cast<void **>(&hs->h_z), sizeof(float) * count, hipHostMallocDefault));
        HS_CHK(c, hipHostMalloc(reinterpret_cast<void **>(&hs->h_idx), sizeof(int32_t) * count, hipHostMallocDefault));
        HS_CHK(c, hipMalloc(reinterpret_cast<void **>(&hs->d_z), sizeof(float) * count));
        HS_CHK(c, hipMalloc(reinterpret_cast<void **>(&hs->d_idx), sizeof(int32_t) * count));
        hs->cap = count;
    }
    hs->count = count;
    hs->list->assign(idx_host, idx_host + count);
    for (int64_t k = 0; k < count; ++k) hs->h_idx[k] = -1;
    // alpha^(t) and v at this point of the compute stream
    HS_CHK(c, hipMemcpyAsync(hs->h_alpha, c->alpha, sizeof(float) * c->n, hipMemcpyDeviceToHost, c->compute));
    HS_CHK(c, hipMemcpyAsync(hs->h_v, c->v, sizeof(float) * c->d, hipMemcpyDeviceToHost, c->compute));
    HS_CHK(c, hipEventRecord(hs->snap, c->compute));
    hs->stop.store(0);
    hs->next.store(0);
    if ((int)hs->threads.size() != nthreads) {                    // (re)build the pool
        stop_pool(hs);
        for (int t = 0; t < nthreads; ++t)
            hs->threads.emplace_back(sampler_thread, c, hs, t, nthreads, hs->generation);
    }
    {
        std::lock_guard<std::mutex> lk(hs->mu);
        hs->finished = 0;
        hs->generation++;
    }
    hs->cv_start.notify_all();
    hs->active = true;
    return DUHL_OK;
}

extern "C" duhl_status duhl_host_sample_end(duhl_ctx *c, int wait_all, int64_t *n_done)
{
    if (!c) return DUHL_EINVAL;
    duhl_host_sampler *hs = c->sampler;
    if (!hs || !hs->active) { c->err = "no host sampling round is running"; return DUHL_ESTATE; }
    HS_CHK(c, hipSetDevice(c->device));
    if (!wait_all) hs->stop.store(1);            // unit B is done: stop sampling
    {
        std::unique_lock<std::mutex> lk(hs->mu);
        hs->cv_done.wait(lk, [&] { return hs->finished == (int)hs->threads.size(); });
    }
    hs->active = false;
    int64_t done = 0, prefix = 0;
    for (int64_t k = 0; k < hs->count; ++k) done += hs->h_idx[k] >= 0;
    while (prefix < hs->count && hs->h_idx[prefix] >= 0) ++prefix;
    hs->prefix = prefix;
    if (hs->count > 0) {
        HS_CHK(c, hipMemcpyAsync(hs->d_idx, hs->h_idx, sizeof(int32_t) * hs->count, hipMemcpyHostToDevice, c->compute));
        HS_CHK(c, hipMemcpyAsync(hs->d_z, hs->h_z, sizeof(float) * hs->count, hipMemcpyHostToDevice, c->compute));
        hipLaunchKernelGGL(scatter_z_kernel, dim3((hs->count + 255) / 256), dim3(256), 0, c->compute, c->z,
                           hs->d_idx, hs->d_z, hs->count);
        HS_CHK(c, hipGetLastError());
        // the pinned staging buffers are reused by the next round: wait until they were read
        HS_CHK(c, hipStreamSynchronize(c->compute));
    }
    if (n_done) *n_done = done;
    return DUHL_OK;
}
