// The worker's executors (paper section 5.2, "Actions" and "Results"): one thread per action type
// that takes its actions in order of their `earliest` time stamps, waits until `earliest`, rejects
// what it reaches after `latest`, runs the rest on a stream of its own and reports status and
// timing.  INFER passes through three executors: the input copy runs on receipt, EXEC inherits the
// action's window, the output copy follows EXEC at once.  Host code only; every GPU operation is
// one of the library's own calls.
#include "../../include/clockwork_exec.h"

#include <hip/hip_runtime.h>
#include <pthread.h>
#include <time.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <deque>
#include <map>
#include <mutex>
#include <thread>
#include <vector>

namespace {

uint64_t now_ns() {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

struct Item {
    cw_action a;
    int32_t slot = -1;
    uint64_t begin_ns = 0, device_ns = 0;
    uint64_t seq = 0;  // arrival order, for equal `earliest`
};

// Actions waiting for one executor, kept in `earliest` order (arrival order among equals).
struct Queue {
    std::mutex mu;
    std::condition_variable cv;
    std::deque<Item> items;
    void push(const Item &it, bool by_time) {
        {
            std::lock_guard<std::mutex> g(mu);
            auto pos = items.end();
            if (by_time)
                pos = std::upper_bound(items.begin(), items.end(), it, [](const Item &x, const Item &y) {
                    return x.a.earliest_ns != y.a.earliest_ns ? x.a.earliest_ns < y.a.earliest_ns : x.seq < y.seq;
                });
            items.insert(pos, it);
        }
        cv.notify_all();
    }
};

enum { EX_LOAD = 0, EX_UNLOAD, EX_INPUT, EX_EXEC, EX_OUTPUT, N_EXEC };

struct Samples {  // the last 10 durations of one (type, model, batch)
    uint64_t v[10] = {0};
    uint32_t n = 0;
};

}  // namespace

struct cw_worker {
    cw_ctx *ctx = nullptr;
    int device = -1;
    std::mutex ctx_mu;  // the context's calls are not thread-safe: one at a time (each only enqueues)
    Queue q[N_EXEC];
    std::thread th[N_EXEC];
    hipStream_t stream[N_EXEC] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    hipEvent_t load_ev[2] = {nullptr, nullptr};
    std::atomic<bool> stop{false};
    std::mutex res_mu;
    std::condition_variable res_cv;
    std::deque<cw_result> results;
    std::mutex prof_mu;
    std::map<std::tuple<int32_t, int32_t, int32_t>, Samples> prof;
    uint64_t seq = 0;
    std::mutex seq_mu;
    uint64_t submitted = 0, finished = 0;
};

namespace {

void post(cw_worker *w, const Item &it, int32_t status, uint64_t end_ns) {
    cw_result r{};
    r.id = it.a.id;
    r.type = it.a.type;
    r.status = status;
    r.begin_ns = it.begin_ns;
    r.end_ns = end_ns;
    r.device_ns = it.device_ns;
    if (status == CW_OK) {
        std::lock_guard<std::mutex> g(w->prof_mu);
        Samples &s = w->prof[std::make_tuple(it.a.type, it.a.model_id, it.a.type == CW_ACTION_INFER ? it.a.batch : 0)];
        s.v[s.n % 10] = it.device_ns ? it.device_ns : end_ns - it.begin_ns;
        ++s.n;
    }
    {
        std::lock_guard<std::mutex> g(w->res_mu);
        w->results.push_back(r);
        ++w->finished;
    }
    w->res_cv.notify_all();
}

// Waits for the next action of executor `ex`; for the executors with a window also until the
// action's `earliest`.  An action that arrives meanwhile with an earlier `earliest` goes first.
// Returns false when the worker stops.
bool take(cw_worker *w, int ex, bool windowed, Item *out) {
    Queue &q = w->q[ex];
    std::unique_lock<std::mutex> lk(q.mu);
    for (;;) {
        if (w->stop) return false;
        if (q.items.empty()) {
            q.cv.wait(lk);
            continue;
        }
        const uint64_t t = now_ns(), e = q.items.front().a.earliest_ns;
        if (windowed && t < e) {
            // sleep to within 50 us of `earliest`, then poll: the start should not be late
            if (e - t > 50000) q.cv.wait_for(lk, std::chrono::nanoseconds(e - t - 50000));
            else { lk.unlock(); lk.lock(); }
            continue;
        }
        *out = q.items.front();
        q.items.pop_front();
        return true;
    }
}

int32_t sync_stream(cw_worker *w, int ex) {
    if (w->device < 0) return CW_OK;
    return hipStreamSynchronize(w->stream[ex]) == hipSuccess ? CW_OK : CW_ERR_HIP;
}

// LOAD waits for milliseconds and nothing waits for it to the microsecond: it sleeps between
// polls.  (A thread blocked in hipStreamSynchronize for the length of a LOAD was measured to make
// the EXEC executor's launches, issued meanwhile, late by tens of microseconds.)
int32_t nap_stream(cw_worker *w, int ex) {
    if (w->device < 0) return CW_OK;
    for (;;) {
        const hipError_t e = hipStreamQuery(w->stream[ex]);
        if (e == hipSuccess) return CW_OK;
        if (e != hipErrorNotReady) return CW_ERR_HIP;
        std::this_thread::sleep_for(std::chrono::microseconds(100));
    }
}

// The EXEC executor polls instead of sleeping in the driver: it owns its core, and the wake-up
// of a blocking wait (tens of microseconds) would be idle GPU time between two EXECs.
int32_t spin_stream(cw_worker *w, int ex) {
    if (w->device < 0) return CW_OK;
    for (;;) {
        const hipError_t e = hipStreamQuery(w->stream[ex]);
        if (e == hipSuccess) return CW_OK;
        if (e != hipErrorNotReady) return CW_ERR_HIP;
    }
}

void run_load(cw_worker *w) {
    if (w->device >= 0) (void)hipSetDevice(w->device);
    Item it;
    while (take(w, EX_LOAD, true, &it)) {
        it.begin_ns = now_ns();
        if (it.begin_ns > it.a.latest_ns) { post(w, it, CW_ERR_TOO_LATE, it.begin_ns); continue; }
        // The context is held only while the copies and pack kernels are enqueued and while the
        // recorded graphs are installed; the recording itself (milliseconds of host work) runs
        // beside the other executors, and the action's result is posted when all of it is done.
        int32_t rc;
        cw_load_pending *pending = nullptr;
        {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            if (w->device >= 0) (void)hipEventRecord(w->load_ev[0], w->stream[EX_LOAD]);
            rc = cw_load_weights_begin(w->ctx, it.a.model_id, it.a.host_in, it.a.host_in_bytes, w->stream[EX_LOAD], &pending);
            if (w->device >= 0) (void)hipEventRecord(w->load_ev[1], w->stream[EX_LOAD]);
        }
        if (rc == CW_OK) {
            (void)cw_load_weights_record(w->ctx, pending);
            {
                std::lock_guard<std::mutex> g(w->ctx_mu);
                (void)cw_load_weights_end(w->ctx, pending);   // without graphs EXEC issues plain launches
            }
            cw_load_weights_release(pending);
            rc = nap_stream(w, EX_LOAD);
        }
        if (rc == CW_OK && w->device >= 0) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, w->load_ev[0], w->load_ev[1]) == hipSuccess) it.device_ns = (uint64_t)((double)ms * 1e6 + 0.5);
        }
        post(w, it, rc, now_ns());
    }
}

void run_unload(cw_worker *w) {
    Item it;
    while (take(w, EX_UNLOAD, true, &it)) {
        it.begin_ns = now_ns();
        if (it.begin_ns > it.a.latest_ns) { post(w, it, CW_ERR_TOO_LATE, it.begin_ns); continue; }
        int32_t rc;
        {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            rc = cw_unload_weights(w->ctx, it.a.model_id);
        }
        post(w, it, rc, now_ns());
    }
}

void run_input(cw_worker *w) {
    if (w->device >= 0) (void)hipSetDevice(w->device);
    Item it;
    while (take(w, EX_INPUT, false, &it)) {
        int32_t rc;
        {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            rc = cw_input(w->ctx, it.a.model_id, it.a.batch, static_cast<const float *>(it.a.host_in), &it.slot, w->stream[EX_INPUT]);
        }
        if (rc != CW_OK) {
            it.begin_ns = now_ns();
            post(w, it, rc, it.begin_ns);
            continue;
        }
        w->q[EX_EXEC].push(it, true);  // EXEC waits for the copy through the slot's event, not here
    }
}

void run_exec(cw_worker *w) {
    if (w->device >= 0) (void)hipSetDevice(w->device);
    Item it;
    while (take(w, EX_EXEC, true, &it)) {
        it.begin_ns = now_ns();
        int32_t rc = CW_OK;
        if (it.begin_ns > it.a.latest_ns) rc = CW_ERR_TOO_LATE;
        if (rc == CW_OK) {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            rc = cw_exec(w->ctx, it.a.model_id, it.a.batch, it.slot, w->stream[EX_EXEC]);
        }
        if (rc == CW_OK) rc = spin_stream(w, EX_EXEC);  // one EXEC at a time
        if (rc == CW_OK) {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            rc = cw_exec_duration_ns(w->ctx, it.slot, &it.device_ns);
        }
        if (rc != CW_OK) {
            {
                std::lock_guard<std::mutex> g(w->ctx_mu);
                (void)cw_release(w->ctx, it.slot);
            }
            post(w, it, rc, now_ns());
            continue;
        }
        w->q[EX_OUTPUT].push(it, false);
    }
}

void run_output(cw_worker *w) {
    if (w->device >= 0) (void)hipSetDevice(w->device);
    Item it;
    while (take(w, EX_OUTPUT, false, &it)) {
        int32_t rc;
        {
            std::lock_guard<std::mutex> g(w->ctx_mu);
            rc = cw_output(w->ctx, it.slot, it.a.host_probs, it.a.host_logits, w->stream[EX_OUTPUT]);
        }
        if (rc == CW_OK) rc = sync_stream(w, EX_OUTPUT);
        post(w, it, rc, now_ns());
    }
}

void pin(std::thread &t, int core) {
    if (core >= 0) {
        cpu_set_t set;
        CPU_ZERO(&set);
        CPU_SET(core, &set);
        (void)pthread_setaffinity_np(t.native_handle(), sizeof set, &set);
    }
    sched_param sp{};
    sp.sched_priority = 1;
    (void)pthread_setschedparam(t.native_handle(), SCHED_FIFO, &sp);  // needs privileges; best effort
}

}  // namespace

extern "C" {

uint64_t cw_worker_now_ns(void) { return now_ns(); }

int32_t cw_worker_create(cw_ctx *ctx, const int32_t *cores, cw_worker **out) {
    if (!ctx || !out) return CW_ERR_INVALID;
    *out = nullptr;
    cw_worker *w = new cw_worker;
    w->ctx = ctx;
    w->device = cw_context_device(ctx);
    if (w->device >= 0) {
        int prev = 0;
        (void)hipGetDevice(&prev);
        bool ok = hipSetDevice(w->device) == hipSuccess;
        for (int i = 0; i < N_EXEC && ok; ++i)
            if (i != EX_UNLOAD) ok = hipStreamCreate(&w->stream[i]) == hipSuccess;  // default priority
        for (int i = 0; i < 2 && ok; ++i) ok = hipEventCreate(&w->load_ev[i]) == hipSuccess;
        (void)hipSetDevice(prev);
        if (!ok) {
            cw_worker_destroy(w);
            return CW_ERR_HIP;
        }
    }
    void (*fn[N_EXEC])(cw_worker *) = {run_load, run_unload, run_input, run_exec, run_output};
    for (int i = 0; i < N_EXEC; ++i) {
        w->th[i] = std::thread(fn[i], w);
        pin(w->th[i], cores ? cores[i] : -1);
    }
    *out = w;
    return CW_OK;
}

int32_t cw_worker_submit(cw_worker *w, const cw_action *a) {
    if (!w || !a) return CW_ERR_INVALID;
    if (a->type != CW_ACTION_LOAD && a->type != CW_ACTION_UNLOAD && a->type != CW_ACTION_INFER) return CW_ERR_INVALID;
    if (a->latest_ns < a->earliest_ns) return CW_ERR_INVALID;
    if (a->type == CW_ACTION_INFER && (!a->host_in || !a->host_probs)) return CW_ERR_INVALID;
    if (a->type == CW_ACTION_LOAD && !a->host_in) return CW_ERR_INVALID;
    Item it;
    it.a = *a;
    {
        std::lock_guard<std::mutex> g(w->seq_mu);
        it.seq = w->seq++;
    }
    {
        std::lock_guard<std::mutex> g(w->res_mu);
        ++w->submitted;
    }
    const int ex = a->type == CW_ACTION_LOAD ? EX_LOAD : a->type == CW_ACTION_UNLOAD ? EX_UNLOAD : EX_INPUT;
    w->q[ex].push(it, ex != EX_INPUT);
    return CW_OK;
}

int32_t cw_worker_next_result(cw_worker *w, cw_result *out, uint64_t timeout_ns) {
    if (!w || !out) return CW_ERR_INVALID;
    std::unique_lock<std::mutex> lk(w->res_mu);
    if (!w->res_cv.wait_for(lk, std::chrono::nanoseconds(timeout_ns), [&] { return !w->results.empty(); })) return CW_ERR_TIMEOUT;
    *out = w->results.front();
    w->results.pop_front();
    return CW_OK;
}

int32_t cw_worker_profile(cw_worker *w, int32_t type, int32_t model_id, int32_t batch, uint32_t *n, uint64_t *mean_ns, uint64_t *max_ns) {
    if (!w || !n || !mean_ns || !max_ns) return CW_ERR_INVALID;
    std::lock_guard<std::mutex> g(w->prof_mu);
    auto itp = w->prof.find(std::make_tuple(type, model_id, type == CW_ACTION_INFER ? batch : 0));
    *n = 0; *mean_ns = 0; *max_ns = 0;
    if (itp == w->prof.end()) return CW_OK;
    const uint32_t k = std::min<uint32_t>(itp->second.n, 10);
    uint64_t sum = 0;
    for (uint32_t i = 0; i < k; ++i) { sum += itp->second.v[i]; *max_ns = std::max(*max_ns, itp->second.v[i]); }
    *n = k;
    *mean_ns = k ? sum / k : 0;
    return CW_OK;
}

int32_t cw_worker_destroy(cw_worker *w) {
    if (!w) return CW_ERR_INVALID;
    for (int i = 0; i < N_EXEC; ++i) {
        {
            std::lock_guard<std::mutex> g(w->q[i].mu);
            w->stop = true;
        }
        w->q[i].cv.notify_all();
    }
    for (int i = 0; i < N_EXEC; ++i)
        if (w->th[i].joinable()) w->th[i].join();
    // actions never started: their INFER slots go back, nothing else to undo
    for (int i = 0; i < N_EXEC; ++i)
        for (Item &it : w->q[i].items)
            if (it.slot >= 0) (void)cw_release(w->ctx, it.slot);
    if (w->device >= 0) {
        (void)hipSetDevice(w->device);
        for (int i = 0; i < N_EXEC; ++i)
            if (w->stream[i]) { (void)hipStreamSynchronize(w->stream[i]); (void)hipStreamDestroy(w->stream[i]); }
        for (int i = 0; i < 2; ++i)
            if (w->load_ev[i]) (void)hipEventDestroy(w->load_ev[i]);
    }
    delete w;
    return CW_OK;
}

}  // extern "C"
