// A matrix in ordinary (pageable) host memory: unit A's memory on a machine that cannot pin all of
// it (Assumption 1 of Section 3: unit A holds the whole matrix, unit B only a working set).  The
// device cannot read such memory, so every column that has to cross the host link is first copied
// by host threads into one of a few pinned, device-readable staging buffers, and a kernel reads it
// from there: the gap pass computes its dot products straight from the staged batch (no device
// copy), the column swap of Algorithm 2 copies the batch into the planned device slots.
//
// Two independent lanes, each with its own buffers and copy threads: the caller's thread drives the
// staged passes (first pass of set_data, duhl_gap over a list, the full refresh of duhl_run) on the
// compute stream; a background thread drives the column swap on the copy stream, so that
// duhl_select returns at once and the passes on the current working set overlap the copies (Figure 2).
// A buffer is refilled only after the kernel that read it has finished (one event per buffer).
#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "duhl_internal.h"

namespace {

constexpr int kBufs = 3;

// Fork-join over the jobs 0 .. njobs-1 by a fixed set of threads plus the caller.
class CopyPool {
public:
    void start(int nthreads)
    {
        for (int t = 0; t < nthreads; ++t) threads_.emplace_back([this] { worker(); });
    }
    ~CopyPool()
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            quit_ = true;
        }
        cv_go_.notify_all();
        for (auto &t : threads_) t.join();
    }
    void run(int64_t njobs, const std::function<void(int64_t)> &fn)
    {
        if (njobs <= 0) return;
        {
            std::lock_guard<std::mutex> lk(mu_);
            fn_ = &fn;
            njobs_ = njobs;
            next_.store(0);
            busy_ = (int)threads_.size();
            ++generation_;
        }
        cv_go_.notify_all();
        drain();
        std::unique_lock<std::mutex> lk(mu_);
        cv_done_.wait(lk, [this] { return busy_ == 0; });
        fn_ = nullptr;
    }

private:
    void drain()
    {
        for (;;) {
            const int64_t k = next_.fetch_add(1, std::memory_order_relaxed);
            if (k >= njobs_) break;
            (*fn_)(k);
        }
    }
    void worker()
    {
        int seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_go_.wait(lk, [&] { return quit_ || generation_ != seen; });
                if (quit_) return;
                seen = generation_;
            }
            drain();
            {
                std::lock_guard<std::mutex> lk(mu_);
                --busy_;
            }
            cv_done_.notify_all();
        }
    }
    std::vector<std::thread> threads_;
    std::mutex mu_;
    std::condition_variable cv_go_, cv_done_;
    const std::function<void(int64_t)> *fn_ = nullptr;
    std::atomic<int64_t> next_{0};
    int64_t njobs_ = 0;
    int generation_ = 0, busy_ = 0;
    bool quit_ = false;
};

struct Lane {
    float *host[kBufs] = {nullptr, nullptr, nullptr};     // pinned
    const float *dev[kBufs] = {nullptr, nullptr, nullptr};   // the same memory as the device sees it
    hipEvent_t done[kBufs] = {nullptr, nullptr, nullptr};    // the kernel that read the buffer has finished
    bool used[kBufs] = {false, false, false};
    CopyPool pool;
    int next = 0;
};

}  // namespace

struct duhl_stager {
    int64_t lds = 0;            // floats between staged columns: d rounded up to four
    int64_t cols_per_buf = 0;
    Lane fg, bg;
    int32_t *idx_dev = nullptr; // device copy of a host-made list (n entries)
    std::vector<int32_t> list;  // host copy of the caller's list
    // background swap job
    std::thread swap_thread;
    std::mutex mu;
    std::condition_variable cv;
    bool job_pending = false, job_done = true, quit = false;
    std::vector<int32_t> fill;  // coordinates whose columns the job copies, in plan order
    hipError_t job_status = hipSuccess;
};

namespace duhl {

namespace {

hipError_t lane_create(Lane &L, size_t bytes, int threads)
{
    for (int b = 0; b < kBufs; ++b) {
        hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&L.host[b]), bytes, hipHostMallocMapped);
        if (e != hipSuccess) return e;
        void *dptr = nullptr;
        e = hipHostGetDevicePointer(&dptr, L.host[b], 0);
        if (e != hipSuccess) return e;
        L.dev[b] = static_cast<const float *>(dptr);
        e = hipEventCreateWithFlags(&L.done[b], hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    L.pool.start(threads);
    return hipSuccess;
}

void lane_destroy(Lane &L)
{
    for (int b = 0; b < kBufs; ++b) {
        if (L.done[b]) {
            (void)hipEventSynchronize(L.done[b]);
            (void)hipEventDestroy(L.done[b]);
        }
        if (L.host[b]) (void)hipHostFree(L.host[b]);
        L.host[b] = nullptr;
        L.done[b] = nullptr;
    }
}

// Copy the columns of list entries [k0, k0 + count) into a staging buffer: entry k names coordinate
// list[k] (or first + k when list == nullptr); entries outside [0, n) are left out (the kernels skip
// them as well).  Columns are padded with zeros to lds floats.
void fill_buffer(const duhl_ctx *c, Lane &L, float *dst, const int32_t *list, int64_t first, int64_t k0,
                 int64_t count)
{
    const int64_t d = c->d, lds = c->stager->lds;
    const bool contiguous = !list && c->host_ld == lds && c->host_chunks.size() == 1;
    if (contiguous) {                                   // one run of memory: split it into 2 MB jobs
        const char *src = reinterpret_cast<const char *>(host_col(c, first + k0));
        char *out = reinterpret_cast<char *>(dst);
        const int64_t bytes = count * lds * 4, piece = 2 << 20;
        L.pool.run((bytes + piece - 1) / piece, [&](int64_t job) {
            const int64_t off = job * piece;
            memcpy(out + off, src + off, (size_t)(bytes - off < piece ? bytes - off : piece));
        });
        return;
    }
    L.pool.run(count, [&](int64_t k) {
        const int64_t j = list ? (int64_t)list[k0 + k] : first + k0 + k;
        if (j < 0 || j >= c->n) return;
        float *out = dst + k * lds;
        memcpy(out, host_col(c, j), (size_t)d * 4);
        for (int64_t r = d; r < lds; ++r) out[r] = 0.0f;
    });
}

// Batches of a pass over `count` list entries through the lane's buffers: fill (host threads), then
// `launch` enqueues the kernels that read the batch on `stream`.
template <typename F>
hipError_t staged_pass(duhl_ctx *c, Lane &L, hipStream_t stream, const int32_t *list, int64_t first,
                       int64_t count, F &&launch)
{
    duhl_stager *st = c->stager;
    for (int64_t k0 = 0; k0 < count; k0 += st->cols_per_buf) {
        const int64_t cnt = count - k0 < st->cols_per_buf ? count - k0 : st->cols_per_buf;
        const int b = L.next;
        L.next = (L.next + 1) % kBufs;
        if (L.used[b]) {
            const hipError_t e = hipEventSynchronize(L.done[b]);
            if (e != hipSuccess) return e;
        }
        fill_buffer(c, L, L.host[b], list, first, k0, cnt);
        StageBatch batch{L.dev[b], st->lds, k0, cnt};
        hipError_t e = launch(batch);
        if (e == hipSuccess) e = hipEventRecord(L.done[b], stream);
        if (e != hipSuccess) return e;
        L.used[b] = true;
    }
    return hipSuccess;
}

// The background thread: waits for a swap job, stages the missing columns and enqueues their
// copies on the copy stream, records ev_copy behind the last of them.
void swap_worker(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    (void)hipSetDevice(c->device);
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(st->mu);
            st->cv.wait(lk, [&] { return st->quit || st->job_pending; });
            if (st->quit) return;
            st->job_pending = false;
        }
        hipError_t e = staged_pass(c, st->bg, c->copy, st->fill.data(), 0, (int64_t)st->fill.size(),
                                   [&](const StageBatch &b) { return launch_copy_batch(c, b); });
        if (e == hipSuccess) e = hipEventRecord(c->ev_copy, c->copy);
        {
            std::lock_guard<std::mutex> lk(st->mu);
            st->job_status = e;
            st->job_done = true;
        }
        st->cv.notify_all();
    }
}

int env_or(const char *name, int dflt)
{
    const char *s = getenv(name);
    const int v = (s && *s) ? atoi(s) : dflt;
    return v > 0 ? v : dflt;
}

}  // namespace

hipError_t stager_create(duhl_ctx *c)
{
    duhl_stager *st = new (std::nothrow) duhl_stager();
    if (!st) return hipErrorOutOfMemory;
    c->stager = st;
    st->lds = (c->d + 3) / 4 * 4;
    // buffer size: DUHL_STAGE_MB megabytes (64 by default), at least one column
    size_t bytes = (size_t)env_or("DUHL_STAGE_MB", 64) << 20;
    const size_t col = (size_t)st->lds * 4;
    if (bytes < col) bytes = col;
    st->cols_per_buf = (int64_t)(bytes / col);
    bytes = (size_t)st->cols_per_buf * col;
    const int threads = env_or("DUHL_STAGE_THREADS", 6);
    hipError_t e = lane_create(st->fg, bytes, threads);
    if (e == hipSuccess) e = lane_create(st->bg, bytes, threads);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&st->idx_dev), sizeof(int32_t) * (size_t)c->n);
    if (e != hipSuccess) return e;
    st->swap_thread = std::thread(swap_worker, c);
    return hipSuccess;
}

void stager_destroy(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    if (!st) return;
    if (st->swap_thread.joinable()) {
        {
            std::unique_lock<std::mutex> lk(st->mu);
            st->cv.wait(lk, [&] { return st->job_done && !st->job_pending; });
            st->quit = true;
        }
        st->cv.notify_all();
        st->swap_thread.join();
    }
    (void)hipStreamSynchronize(c->compute);
    (void)hipStreamSynchronize(c->copy);
    lane_destroy(st->fg);
    lane_destroy(st->bg);
    (void)hipFree(st->idx_dev);
    delete st;
    c->stager = nullptr;
}

hipError_t staged_gap(duhl_ctx *c, const int32_t *idx, int64_t first, int64_t count, bool with_norms)
{
    duhl_stager *st = c->stager;
    const int32_t *list = nullptr;
    if (idx) {                                          // the host needs the list to gather the columns
        st->list.resize((size_t)count);
        hipError_t e = hipMemcpyAsync(st->list.data(), idx, sizeof(int32_t) * (size_t)count, hipMemcpyDeviceToHost,
                                      c->compute);
        if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
        if (e != hipSuccess) return e;
        list = st->list.data();
    }
    // The first pass over the whole matrix (set_data) also fills the device slots: once the gaps of
    // the first twentieth of the columns are out, their (1 - f)-quantile is taken for the threshold
    // above which a fraction f of all columns lies -- f chosen to fill about 0.9 of the slots -- and
    // every later batch leaves its columns above it on the device (launch_keep_batch).
    const bool keep = with_norms && !idx && first == 0 && count == c->n && c->keep_first_pass && c->slots;
    const int64_t probe = keep ? std::max<int64_t>(std::min<int64_t>(c->n, 2048), c->n / 20) : 0;
    bool have_tau = false;
    float tau = 0.0f;
    if (keep) {
        hipError_t e = launch_fill_i32(c->compute, reinterpret_cast<int32_t *>(&c->sel->n_kept), 1, 0);
        if (e != hipSuccess) return e;
    }
    bool first_batch = true;
    hipError_t e = staged_pass(c, st->fg, c->compute, list, first, count, [&](const StageBatch &b) {
        hipError_t e = hipSuccess;
        if (keep && !have_tau && b.k0 >= probe && c->n > b.k0) {
            std::vector<float> zs((size_t)b.k0);
            e = hipMemcpyAsync(zs.data(), c->z, sizeof(float) * zs.size(), hipMemcpyDeviceToHost, c->compute);
            if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
            if (e != hipSuccess) return e;
            double f = 0.9 * (double)c->budget / (double)(c->n - b.k0);
            if (f > 1.0) f = 1.0;
            size_t rank = (size_t)((1.0 - f) * (double)zs.size());
            if (rank >= zs.size()) rank = zs.size() - 1;
            std::nth_element(zs.begin(), zs.begin() + (std::ptrdiff_t)rank, zs.end());
            tau = zs[rank];
            have_tau = true;
        }
        e = launch_gap_batch(c, b, idx, first, with_norms, first_batch);
        first_batch = false;
        if (e == hipSuccess && have_tau) e = launch_keep_batch(c, b, first, tau);
        return e;
    });
    if (e == hipSuccess && keep) {
        e = hipMemcpyAsync(c->h_u32 + 3, &c->sel->n_kept, sizeof(uint32_t), hipMemcpyDeviceToHost, c->compute);
        if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
        if (e == hipSuccess) c->kept_first_pass = c->h_u32[3] < (uint32_t)c->budget ? c->h_u32[3] : c->budget;
    }
    return e;
}

// A host-made list of coordinates, also put on the device for the kernels.
static hipError_t upload_list(duhl_ctx *c, const std::vector<int32_t> &list)
{
    if (list.empty()) return hipSuccess;
    hipError_t e = hipMemcpyAsync(c->stager->idx_dev, list.data(), sizeof(int32_t) * list.size(), hipMemcpyHostToDevice,
                                  c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);   // list.data() is pageable: it may be reused
    return e;
}

// u += a_j / ||a_j|| for `samples` evenly spaced columns (u is cleared and summed up by the caller).
hipError_t staged_corr_sample(duhl_ctx *c, float *u, int samples)
{
    duhl_stager *st = c->stager;
    st->list.clear();
    for (int64_t s = 0; s < samples; ++s) st->list.push_back((int32_t)(s * (c->n / samples)));
    const hipError_t e = upload_list(c, st->list);
    if (e != hipSuccess) return e;
    return staged_pass(c, st->fg, c->compute, st->list.data(), 0, (int64_t)st->list.size(),
                       [&](const StageBatch &b) { return launch_corr_batch(c, b, st->idx_dev, u); });
}

hipError_t staged_accumulate_v(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    std::vector<float> alpha((size_t)c->n);
    hipError_t e = hipMemcpyAsync(alpha.data(), c->alpha, sizeof(float) * (size_t)c->n, hipMemcpyDeviceToHost, c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) return e;
    st->list.clear();
    for (int64_t j = 0; j < c->n; ++j)
        if (alpha[(size_t)j] != 0.0f) st->list.push_back((int32_t)j);
    e = upload_list(c, st->list);
    if (e != hipSuccess) return e;
    return staged_pass(c, st->fg, c->compute, st->list.data(), 0, (int64_t)st->list.size(),
                       [&](const StageBatch &b) { return launch_accumulate_batch(c, b, st->idx_dev); });
}

hipError_t stager_swap_begin(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    // the plan was made on the device: bring the list of missing columns to the host
    hipError_t e = hipMemcpyAsync(c->h_u32 + 3, &c->sel->n_fill, sizeof(uint32_t), hipMemcpyDeviceToHost, c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e != hipSuccess) return e;
    int64_t n_fill = c->h_u32[3];
    if (n_fill > c->m_next) n_fill = c->m_next;
    {
        std::unique_lock<std::mutex> lk(st->mu);
        st->cv.wait(lk, [&] { return st->job_done; });       // (the previous job was joined by commit)
    }
    st->fill.resize((size_t)n_fill);
    if (n_fill > 0) {
        e = hipMemcpy(st->fill.data(), c->fill_col, sizeof(int32_t) * (size_t)n_fill, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return e;
    }
    {
        std::lock_guard<std::mutex> lk(st->mu);
        st->job_done = false;
        st->job_pending = true;
        st->job_status = hipSuccess;
    }
    st->cv.notify_all();
    return hipSuccess;
}

bool stager_swap_done(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    std::lock_guard<std::mutex> lk(st->mu);
    return st->job_done;
}

hipError_t stager_swap_join(duhl_ctx *c)
{
    duhl_stager *st = c->stager;
    std::unique_lock<std::mutex> lk(st->mu);
    st->cv.wait(lk, [&] { return st->job_done; });
    return st->job_status;
}

}  // namespace duhl
