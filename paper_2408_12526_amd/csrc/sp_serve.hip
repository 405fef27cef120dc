// Real-time replay of an arrival list against a loaded student group: dispatcher thread (the caller) + one worker
// thread per student group (see sp_dispatch.h).  Host code; the only GPU work is what sp_forward enqueues and the
// copies of token ids / offsets / logits around it.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "sp_dispatch.h"
#include "sp_internal.h"

namespace {

// Offsets and token ids of one element: from the worker's pinned staging buffer (which the GPU can read in place) into
// its device buffer, as a kernel on the worker's own stream: for about a kilobyte a launch on the compute queue is
// cheaper than a copy command and the hand-over between the copy engine and that queue.  On the way back there is
// nothing to copy: the forward writes its few logits straight into pinned host memory.  (Measured on the replay of the
// bursty arrival process: p50 latency 240 -> 225 us against two copy commands per element.)
__global__ void stage_inputs_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = src[i];
}

struct Job {
    int32_t count = 0, bin_len = 0, k = 0;
    std::vector<int64_t> ids;
    std::vector<int32_t> lens;
};

struct Shared;

struct Worker {
    int index = 0;
    std::thread th;
    hipStream_t stream = nullptr;
    int32_t *h_ids = nullptr, *h_cu = nullptr, *d_ids = nullptr, *d_cu = nullptr;
    int32_t* h_cu_dev = nullptr;        // the staging buffer as the GPU addresses it
    float *h_logits = nullptr, *h_logits_dev = nullptr;   // pinned; the forward writes them in place
    void* d_ws = nullptr;
    std::mutex mu;
    std::condition_variable cv;
    bool has_job = false, stop = false;
    std::atomic<bool> flag{false};      // set with has_job / stop: lets the worker spin without the lock
    Job job;
};

struct Shared {
    const sp_model* model = nullptr;
    const sp_serve_config* cfg = nullptr;
    const int32_t* token_ids = nullptr;
    const int64_t* id_offsets = nullptr;
    int64_t* done_us = nullptr;
    float* logits = nullptr;
    int device = 0, classes = 0, cu_room = 0;    // cu_room: ints reserved for the offsets in front of the ids
    size_t ws_bytes = 0;
    std::chrono::steady_clock::time_point t0;
    std::mutex cq_mu;
    std::condition_variable cq_cv;
    std::vector<int> cq;                 // workers that finished an element (room for all of them reserved up front)
    std::atomic<int> cq_count{0};
    std::atomic<int> error{0};
};

inline int64_t now_us(const Shared& S)
{
    return std::chrono::duration_cast<std::chrono::microseconds>(std::chrono::steady_clock::now() - S.t0).count();
}

void worker_main(Shared* S, Worker* w)
{
    if (hipSetDevice(S->device) != hipSuccess) S->error.store(SP_EHIP);
    const sp_serve_config& c = *S->cfg;
    for (;;) {
        {
            // a short spin first: waking a sleeping thread costs more than a small forward's launches
            for (int spin = 0; spin < 2000 && !w->flag.load(std::memory_order_acquire); ++spin) std::this_thread::yield();
            std::unique_lock<std::mutex> lk(w->mu);
            w->cv.wait(lk, [&] { return w->has_job || w->stop; });
            if (w->stop) return;
            w->has_job = false;
            w->flag.store(false, std::memory_order_release);
        }
        const Job& j = w->job;             // the dispatcher does not touch it again before this worker reports back
        int32_t total = 0, longest = 0;
        w->h_cu[0] = 0;
        for (int32_t i = 0; i < j.count; ++i) {
            const int32_t len = j.lens[i], out_len = c.padded ? j.bin_len : len;
            const int32_t* src = S->token_ids + S->id_offsets[j.ids[i]];
            memcpy(w->h_ids + total, src, sizeof(int32_t) * (size_t)len);
            for (int32_t t = len; t < out_len; ++t) w->h_ids[total + t] = c.pad_id;
            total += out_len;
            w->h_cu[i + 1] = total;
            longest = out_len > longest ? out_len : longest;
        }
        int rc = SP_OK;
        // offsets and ids share one staging buffer (offsets first): one small kernel brings both to the device
        const int nstage = S->cu_room + total;
        hipLaunchKernelGGL(stage_inputs_kernel, dim3((unsigned)((nstage + 255) / 256)), dim3(256), 0, w->stream,
                           (const int32_t*)w->h_cu_dev, w->d_cu, nstage);
        if (hipGetLastError() != hipSuccess) rc = SP_EHIP;
        if (rc == SP_OK)
            rc = sp_forward(S->model, w->d_ids, w->d_cu, j.count, total, longest, j.k, w->d_ws, S->ws_bytes, w->h_logits_dev,
                            w->stream);
        if (hipStreamSynchronize(w->stream) != hipSuccess) rc = SP_EHIP;
        const int64_t t = now_us(*S);
        for (int32_t i = 0; i < j.count; ++i) {
            S->done_us[j.ids[i]] = t;
            memcpy(S->logits + (size_t)j.ids[i] * S->classes, w->h_logits + (size_t)i * S->classes, sizeof(float) * (size_t)S->classes);
        }
        if (rc != SP_OK) S->error.store(rc);
        {
            std::lock_guard<std::mutex> lk(S->cq_mu);
            S->cq.push_back(w->index);
            S->cq_count.fetch_add(1);
        }
        S->cq_cv.notify_one();
    }
}

void release(Worker& w)
{
    if (w.h_cu) (void)hipHostFree(w.h_cu);           // (h_ids / d_ids point into the same allocations)
    if (w.h_logits) (void)hipHostFree(w.h_logits);
    if (w.d_cu) (void)hipFree(w.d_cu);
    if (w.d_ws) (void)hipFree(w.d_ws);
    if (w.stream) (void)hipStreamDestroy(w.stream);
}

}  // namespace

extern "C" int sp_serve_replay(const sp_model* model, const sp_serve_config* cfg, const int64_t* arrival_us,
                               const int32_t* token_ids, const int64_t* id_offsets, int64_t n, int64_t* dispatch_us,
                               int64_t* done_us, int32_t* k_used, int64_t* element, int32_t* elem_size,
                               int64_t* n_elements, float* logits, int64_t* refused, int32_t* k_final)
{
    if (!model || !cfg || !arrival_us || !token_ids || !id_offsets || !dispatch_us || !done_us || !k_used || !element ||
        !elem_size || !n_elements || !logits || !refused || !k_final)
        return SP_EINVAL;
    const sp_config& mc = model->cfg;
    if (n < 0 || cfg->k_min < 1 || cfg->k_min > mc.K || cfg->slots < mc.K || cfg->window_us < 0 || cfg->max_len > mc.max_pos ||
        cfg->pad_id < 0 || cfg->pad_id >= mc.vocab || (cfg->k_start != 0 && (cfg->k_start < cfg->k_min || cfg->k_start > mc.K)))
        return SP_ESHAPE;
    for (int64_t i = 0; i < n; ++i)
        if (id_offsets[i + 1] <= id_offsets[i] || (i && arrival_us[i] < arrival_us[i - 1])) return SP_ESHAPE;
    sp_lab* buf = nullptr;
    sp_ctl* ctl = nullptr;
    int rc = sp_lab_create(cfg->bin_width, cfg->max_len, cfg->max_elem, cfg->capacity, &buf);
    if (rc == SP_OK) rc = sp_ctl_create(mc.K, cfg->slots, cfg->k_min, cfg->window_us, cfg->k_start, &ctl);
    if (rc != SP_OK) { sp_lab_free(buf); sp_ctl_free(ctl); return rc; }

    Shared S;
    S.model = model; S.cfg = cfg; S.token_ids = token_ids; S.id_offsets = id_offsets; S.done_us = done_us; S.logits = logits;
    S.classes = mc.classes;
    const int nworkers = cfg->slots / cfg->k_min;
    const int32_t max_tokens = cfg->max_elem * cfg->max_len;
    S.ws_bytes = sp_workspace_bytes(&mc, max_tokens, cfg->max_elem);
    S.cu_room = (cfg->max_elem + 1 + 63) / 64 * 64;      // keeps the ids 256-byte aligned
    std::unique_ptr<Worker[]> wstore(new (std::nothrow) Worker[(size_t)nworkers]);
    if (!wstore) { sp_lab_free(buf); sp_ctl_free(ctl); return SP_ENOMEM; }
    struct WorkerRange {
        Worker *b, *e;
        Worker* begin() const { return b; }
        Worker* end() const { return e; }
        Worker& operator[](size_t i) const { return b[i]; }
    } workers{wstore.get(), wstore.get() + nworkers};
    bool ok = hipGetDevice(&S.device) == hipSuccess && S.ws_bytes > 0;
    for (int g = 0; g < nworkers && ok; ++g) {
        Worker& w = workers[(size_t)g];
        w.index = g;
        ok = hipStreamCreateWithFlags(&w.stream, hipStreamNonBlocking) == hipSuccess &&
             hipHostMalloc((void**)&w.h_cu, sizeof(int32_t) * (size_t)(S.cu_room + max_tokens), hipHostMallocMapped) == hipSuccess &&
             hipHostMalloc((void**)&w.h_logits, sizeof(float) * (size_t)cfg->max_elem * mc.classes, hipHostMallocMapped) == hipSuccess &&
             hipHostGetDevicePointer((void**)&w.h_cu_dev, w.h_cu, 0) == hipSuccess && w.h_cu_dev &&
             hipHostGetDevicePointer((void**)&w.h_logits_dev, w.h_logits, 0) == hipSuccess && w.h_logits_dev &&
             hipMalloc((void**)&w.d_cu, sizeof(int32_t) * (size_t)(S.cu_room + max_tokens)) == hipSuccess &&
             hipMalloc(&w.d_ws, S.ws_bytes) == hipSuccess;
        if (ok) { w.h_ids = w.h_cu + S.cu_room; w.d_ids = w.d_cu + S.cu_room; }
        if (ok) {
            try { w.job.ids.resize((size_t)cfg->max_elem); w.job.lens.resize((size_t)cfg->max_elem); }
            catch (const std::bad_alloc&) { ok = false; }
        }
    }
    if (!ok) {
        for (auto& w : workers) release(w);
        sp_lab_free(buf); sp_ctl_free(ctl);
        return SP_EHIP;
    }
    S.t0 = std::chrono::steady_clock::now();
    std::vector<int> fin, idle;
    std::vector<int64_t> eid;
    std::vector<int32_t> elen;
    try {
        fin.reserve((size_t)nworkers);
        idle.reserve((size_t)nworkers);
        S.cq.reserve((size_t)nworkers);
        eid.resize((size_t)cfg->max_elem);
        elen.resize((size_t)cfg->max_elem);
        for (auto& w : workers) w.th = std::thread(worker_main, &S, &w);
    } catch (...) {                                     // no memory or no thread: stop what was started
        for (auto& w : workers) {
            { std::lock_guard<std::mutex> lk(w.mu); w.stop = true; w.flag.store(true, std::memory_order_release); }
            w.cv.notify_one();
            if (w.th.joinable()) w.th.join();
            release(w);
        }
        sp_lab_free(buf); sp_ctl_free(ctl);
        return SP_ENOMEM;
    }

    for (int g = nworkers - 1; g >= 0; --g) idle.push_back(g);
    int busy = 0;
    int64_t ne = 0, nref = 0, last_progress = 0;
    auto groups = [&] { const int g = sp_ctl_groups(ctl); return g < nworkers ? g : nworkers; };
    auto hand_over = [&](int32_t count, int32_t bin_len, const int64_t* ids, const int32_t* lens) {
        Worker& w = workers[(size_t)idle.back()];
        idle.pop_back();
        const int64_t t = now_us(S);
        const int32_t k = sp_ctl_k(ctl);
        if (busy == 0) last_progress = t;
        for (int32_t i = 0; i < count; ++i) { dispatch_us[ids[i]] = t; k_used[ids[i]] = k; element[ids[i]] = ne; }
        {
            std::lock_guard<std::mutex> lk(w.mu);
            w.job.count = count; w.job.bin_len = bin_len; w.job.k = k;
            for (int32_t i = 0; i < count; ++i) { w.job.ids[(size_t)i] = ids[i]; w.job.lens[(size_t)i] = lens[i]; }
            w.has_job = true;
            w.flag.store(true, std::memory_order_release);
        }
        w.cv.notify_one();
        elem_size[ne++] = count;
        ++busy;
    };
    auto drain = [&] {
        while (sp_lab_elements(buf) > 0 && busy < groups()) {
            int32_t bin, bl, cnt;
            sp_lab_pop(buf, &bin, &bl, eid.data(), elen.data(), &cnt);
            hand_over(cnt, bl, eid.data(), elen.data());
        }
    };

    int64_t i = 0;
    while ((i < n || busy > 0) && S.error.load() == 0) {
        // completions first
        if (S.cq_count.load() > 0) {
            {
                std::lock_guard<std::mutex> lk(S.cq_mu);
                fin.assign(S.cq.begin(), S.cq.end());   // at most one entry per worker: within the reserved room
                S.cq.clear();
                S.cq_count.store(0);
            }
            for (int g : fin) { idle.push_back(g); --busy; }
            last_progress = now_us(S);
            drain();
            sp_ctl_on_tick(ctl, now_us(S), sp_lab_elements(buf), busy);
        }
        // arrivals that are due
        int64_t t = now_us(S);
        while (i < n && arrival_us[i] <= t) {
            int64_t len64 = id_offsets[i + 1] - id_offsets[i];
            const int32_t len = (int32_t)(len64 > cfg->max_len ? cfg->max_len : len64);
            if (sp_lab_elements(buf) == 0 && busy < groups()) {
                hand_over(1, sp_lab_bin_len(buf, sp_lab_bin_of(buf, len)), &i, &len);
                sp_ctl_on_tick(ctl, t, 0, busy);
            } else {
                int32_t joined = 0;
                if (sp_lab_push(buf, i, len, &joined) == SP_OK) {
                    if (sp_ctl_on_buffered(ctl, sp_lab_elements(buf)) == 1) drain();
                } else {
                    dispatch_us[i] = done_us[i] = -1; k_used[i] = 0; element[i] = -1;
                    ++nref;
                }
            }
            ++i;
            t = now_us(S);
        }
        // wait for the next arrival or a completion
        const int64_t t_next = i < n ? arrival_us[i] : t + 1000;
        while (S.cq_count.load() == 0) {
            const int64_t rem = t_next - now_us(S);
            if (rem <= 0) break;
            if (rem > 300) {
                std::unique_lock<std::mutex> lk(S.cq_mu);
                S.cq_cv.wait_for(lk, std::chrono::microseconds(rem - 150), [&] { return !S.cq.empty(); });
            } else {
                std::this_thread::yield();
            }
        }
        if (busy > 0 && S.cq_count.load() == 0 && now_us(S) - last_progress > 10'000'000)
            S.error.store(SP_EHIP);      // no group has finished for 10 s
    }
    // stop the workers (a worker that is still inside a forward finishes it first)
    for (auto& w : workers) {
        { std::lock_guard<std::mutex> lk(w.mu); w.stop = true; w.flag.store(true, std::memory_order_release); }
        w.cv.notify_one();
    }
    for (auto& w : workers) w.th.join();
    for (auto& w : workers) release(w);
    *n_elements = ne; *refused = nref; *k_final = sp_ctl_k(ctl);
    sp_lab_free(buf);
    sp_ctl_free(ctl);
    return S.error.load();
}
