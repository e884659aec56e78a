// Dynamic batching in front of the preprocessing handles (PREBA section 4.3): the release rule
// (prep_policy_*) and a small server that runs it with real consumers (prep_server_*).
#include <chrono>
#include <condition_variable>
#include <deque>
#include <limits>
#include <mutex>
#include <new>
#include <string.h>
#include <thread>
#include <vector>

#include <hip/hip_runtime.h>

#include "../../include/prep.h"

// ---- the rule ---------------------------------------------------------------------------------
struct prep_policy {
    int32_t batch_max;
    int64_t time_queue_ns;
    struct Waiting { uint64_t id; int64_t t; };
    std::deque<Waiting> queue;  // oldest first
};

namespace {

int64_t deadline_of(const prep_policy &p)
{
    if (p.queue.empty()) return std::numeric_limits<int64_t>::max();
    // the limit of the oldest request, or the arrival that filled a batch if that came first
    int64_t due = p.queue.front().t + p.time_queue_ns;
    if (p.queue.size() >= (size_t)p.batch_max) due = std::min(due, p.queue[(size_t)p.batch_max - 1].t);
    return due;
}

// Timed wait on a condition variable.  The steady clock is the right one; a build for a
// sanitizer whose runtime does not know the steady-clock wait of the C library defines
// PREP_WAIT_ON_SYSTEM_CLOCK and waits on the system clock instead.
template <typename Lock>
void wait_ns(std::condition_variable &cv, Lock &lock, int64_t ns)
{
#ifdef PREP_WAIT_ON_SYSTEM_CLOCK
    cv.wait_until(lock, std::chrono::system_clock::now() + std::chrono::nanoseconds(ns));
#else
    cv.wait_for(lock, std::chrono::nanoseconds(ns));
#endif
}

int64_t now_ns()
{
    return std::chrono::duration_cast<std::chrono::nanoseconds>(
               std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace

extern "C" {

int prep_policy_create(prep_policy **out, int32_t batch_max, int64_t time_queue_ns)
{
    if (!out) return PREP_E_INVALID_ARG;
    *out = nullptr;
    if (batch_max < 1 || time_queue_ns < 0) return PREP_E_INVALID_ARG;
    prep_policy *p = new (std::nothrow) prep_policy;
    if (!p) return PREP_E_NOMEM;
    p->batch_max = batch_max;
    p->time_queue_ns = time_queue_ns;
    *out = p;
    return PREP_OK;
}

void prep_policy_destroy(prep_policy *p) { delete p; }

int prep_policy_arrive(prep_policy *p, uint64_t id, int64_t t_ns)
{
    if (!p || (!p->queue.empty() && t_ns < p->queue.back().t)) return PREP_E_INVALID_ARG;
    p->queue.push_back({id, t_ns});
    return PREP_OK;
}

int64_t prep_policy_deadline(const prep_policy *p)
{
    return p ? deadline_of(*p) : std::numeric_limits<int64_t>::max();
}

int32_t prep_policy_take(prep_policy *p, int64_t now, uint64_t *ids, int32_t cap)
{
    if (!p || !ids || cap < p->batch_max) return PREP_E_INVALID_ARG;
    if (deadline_of(*p) > now) return 0;
    int32_t n = 0;
    while (n < p->batch_max && !p->queue.empty()) {
        ids[n++] = p->queue.front().id;
        p->queue.pop_front();
    }
    return n;
}

int32_t prep_policy_pending(const prep_policy *p) { return p ? (int32_t)p->queue.size() : 0; }

}  // extern "C"

// ---- the server -------------------------------------------------------------------------------
namespace {

constexpr int kOutputSlots = 3;  // output buffers per consumer; one is reused when its results are released

struct Request {
    uint64_t tag = 0;
    int64_t arrival = 0;
    uint32_t len = 0;
    std::vector<uint8_t> bytes;  // capacity max_request_bytes, reserved at start
};

struct Consumer {
    prep_handle *handle = nullptr;
    hipStream_t stream = nullptr;
    void *d_out[kOutputSlots] = {nullptr, nullptr, nullptr};
    int32_t unreleased[kOutputSlots] = {0, 0, 0};  // results of the slot's batch still with the caller
    int slot = 0;
    std::vector<uint8_t> bits;       // the batch's files back to back
    std::vector<uint64_t> offsets;
    std::vector<uint64_t> ids;
    std::vector<int32_t> status;
    std::thread thread;
};

}  // namespace

struct prep_server {
    prep_server_config cfg;
    size_t slab_bytes = 0;
    std::mutex m;
    std::condition_variable work, results_ready;
    prep_policy *policy = nullptr;
    std::vector<Request> requests;   // pool; a request's id in the policy is its index here
    std::vector<uint32_t> free_requests;
    struct Finished { prep_server_result result; uint32_t request; };
    std::deque<Finished> results;
    std::condition_variable slot_free;
    std::vector<Consumer> consumers;
    bool stopping = false;
    int failed = PREP_OK;            // first batch-level failure of a consumer
};

namespace {

void consume(prep_server *s, int ci)
{
    Consumer &c = s->consumers[(size_t)ci];
    (void)hipSetDevice(s->cfg.handle.device);
    std::unique_lock<std::mutex> lock(s->m);
    for (;;) {
        // wait until the rule releases a batch (or the server stops)
        int32_t n = 0;
        while (!s->stopping) {
            n = prep_policy_take(s->policy, now_ns(), c.ids.data(), (int32_t)c.ids.size());
            if (n != 0) break;
            const int64_t due = prep_policy_deadline(s->policy);
            if (due == std::numeric_limits<int64_t>::max())
                s->work.wait(lock);
            else
                wait_ns(s->work, lock, std::max<int64_t>(due - now_ns(), 0));
        }
        if (s->stopping || n < 0) return;
        const int64_t start = now_ns();
        // the batch's files, back to back (the requests stay reserved until the results are out)
        uint64_t at = 0;
        for (int32_t i = 0; i < n; i++) {
            const Request &r = s->requests[(size_t)c.ids[(size_t)i]];
            c.offsets[(size_t)i] = at;
            at += r.len;
        }
        c.offsets[(size_t)n] = at;
        // the output buffer whose turn it is; the caller may still hold tensors of the batch
        // that used it last
        const int slot = c.slot;
        c.slot = (c.slot + 1) % kOutputSlots;
        while (c.unreleased[slot] != 0 && !s->stopping) s->slot_free.wait(lock);
        if (s->stopping) return;
        lock.unlock();
        for (int32_t i = 0; i < n; i++) {
            const Request &r = s->requests[(size_t)c.ids[(size_t)i]];
            memcpy(c.bits.data() + c.offsets[(size_t)i], r.bytes.data(), r.len);
        }
        void *out = c.d_out[slot];
        int rc = prep_decode_resize_batch(c.handle, c.bits.data(), c.offsets.data(), n, &s->cfg.params, out,
                                          c.stream);
        if (rc == PREP_OK) rc = prep_get_status(c.handle, c.status.data(), n);  // waits for the stream
        const int64_t done = now_ns();
        lock.lock();
        if (rc != PREP_OK && s->failed == PREP_OK) s->failed = rc;
        for (int32_t i = 0; i < n; i++) {
            const uint32_t id = (uint32_t)c.ids[(size_t)i];
            const Request &r = s->requests[id];
            prep_server_result res;
            memset(&res, 0, sizeof res);
            res.tag = r.tag;
            res.status = rc != PREP_OK ? rc : c.status[(size_t)i];
            res.batch_size = n;
            res.consumer = ci;
            res.slot = slot;
            res.arrival_ns = r.arrival;
            res.start_ns = start;
            res.done_ns = done;
            res.tensor = static_cast<const uint8_t *>(out) + (size_t)i * s->slab_bytes;
            s->results.push_back({res, id});  // the request's place is given back when the result is read
            c.unreleased[slot]++;
        }
        s->results_ready.notify_all();
    }
}

}  // namespace

extern "C" {

int prep_server_create(prep_server **out, const prep_server_config *cfg)
{
    if (!out) return PREP_E_INVALID_ARG;
    *out = nullptr;
    if (!cfg || cfg->n_consumers < 1 || cfg->n_consumers > 64 || cfg->batch_max < 1 || cfg->batch_max > 65535 ||
        cfg->time_queue_us < 0 || cfg->max_request_bytes < 1 || cfg->queue_capacity < cfg->batch_max ||
        cfg->params.crop_h < 1 || cfg->params.crop_w < 1 ||
        (cfg->params.out_dtype != PREP_F32 && cfg->params.out_dtype != PREP_F16 &&
         cfg->params.out_dtype != PREP_U8_NHWC))
        return PREP_E_INVALID_ARG;
    prep_server *s = new (std::nothrow) prep_server;
    if (!s) return PREP_E_NOMEM;
    s->cfg = *cfg;
    s->cfg.handle.max_batch = cfg->batch_max;
    const uint64_t batch_bytes = (uint64_t)cfg->batch_max * (uint64_t)cfg->max_request_bytes;
    if (s->cfg.handle.max_bitstream_bytes < batch_bytes) s->cfg.handle.max_bitstream_bytes = batch_bytes;
    s->slab_bytes = (size_t)3 * cfg->params.crop_h * cfg->params.crop_w *
                    (cfg->params.out_dtype == PREP_F32 ? 4 : cfg->params.out_dtype == PREP_F16 ? 2 : 1);
    int rc = prep_policy_create(&s->policy, cfg->batch_max, cfg->time_queue_us * 1000);
    // requests in flight: those waiting, those being served and those whose result nobody has
    // read yet (when these fill the pool, submissions are refused until results are read)
    const size_t pool = (size_t)cfg->queue_capacity + 2 * (size_t)cfg->n_consumers * cfg->batch_max;
    if (rc == PREP_OK) {
        s->requests.resize(pool);
        for (size_t i = 0; i < pool; i++) {
            s->requests[i].bytes.resize((size_t)cfg->max_request_bytes);
            s->free_requests.push_back((uint32_t)(pool - 1 - i));
        }
        s->consumers.resize((size_t)cfg->n_consumers);
    }
    for (int i = 0; rc == PREP_OK && i < cfg->n_consumers; i++) {
        Consumer &c = s->consumers[(size_t)i];
        rc = prep_create(&c.handle, &s->cfg.handle);
        if (rc != PREP_OK) break;
        if (hipSetDevice(cfg->handle.device) != hipSuccess ||
            hipStreamCreateWithFlags(&c.stream, hipStreamNonBlocking) != hipSuccess) {
            rc = PREP_E_HIP;
            break;
        }
        for (int k = 0; k < kOutputSlots; k++)
            if (hipMalloc(&c.d_out[k], s->slab_bytes * (size_t)cfg->batch_max) != hipSuccess) rc = PREP_E_NOMEM;
        c.bits.resize((size_t)batch_bytes);
        c.offsets.resize((size_t)cfg->batch_max + 1);
        c.ids.resize((size_t)cfg->batch_max);
        c.status.resize((size_t)cfg->batch_max);
    }
    if (rc != PREP_OK) {
        prep_server_destroy(s);
        return rc;
    }
    for (int i = 0; i < cfg->n_consumers; i++) s->consumers[(size_t)i].thread = std::thread(consume, s, i);
    *out = s;
    return PREP_OK;
}

int prep_server_destroy(prep_server *s)
{
    if (!s) return PREP_E_INVALID_ARG;
    {
        std::lock_guard<std::mutex> lock(s->m);
        s->stopping = true;
    }
    s->work.notify_all();
    s->results_ready.notify_all();
    s->slot_free.notify_all();
    for (Consumer &c : s->consumers) {
        if (c.thread.joinable()) c.thread.join();
        if (c.handle) prep_destroy(c.handle);
        for (int k = 0; k < kOutputSlots; k++)
            if (c.d_out[k]) (void)hipFree(c.d_out[k]);
        if (c.stream) (void)hipStreamDestroy(c.stream);
    }
    prep_policy_destroy(s->policy);
    delete s;
    return PREP_OK;
}

int prep_server_submit(prep_server *s, const uint8_t *jpeg, uint64_t len, uint64_t tag)
{
    if (!s || !jpeg || len == 0) return PREP_E_INVALID_ARG;
    if (len > (uint64_t)s->cfg.max_request_bytes) return PREP_E_TOO_LARGE;
    uint32_t id;
    {
        std::lock_guard<std::mutex> lock(s->m);
        if (s->stopping) return PREP_E_INVALID_ARG;
        if (s->failed != PREP_OK) return s->failed;
        if (prep_policy_pending(s->policy) >= s->cfg.queue_capacity || s->free_requests.empty())
            return PREP_E_TOO_LARGE;
        id = s->free_requests.back();
        s->free_requests.pop_back();
    }
    // the copy is made outside the lock: the request is not visible to the consumers yet
    Request &r = s->requests[id];
    memcpy(r.bytes.data(), jpeg, (size_t)len);
    r.len = (uint32_t)len;
    r.tag = tag;
    {
        std::lock_guard<std::mutex> lock(s->m);
        r.arrival = now_ns();
        prep_policy_arrive(s->policy, id, r.arrival);
    }
    // a consumer that sleeps until the old deadline must look again: the batch may be full now
    s->work.notify_one();
    return PREP_OK;
}

int prep_server_copy_tensor(prep_server *s, const prep_server_result *r, void *host_out)
{
    if (!s || !r || !r->tensor || !host_out) return PREP_E_INVALID_ARG;
    if (hipSetDevice(s->cfg.handle.device) != hipSuccess ||
        hipMemcpy(host_out, r->tensor, s->slab_bytes, hipMemcpyDeviceToHost) != hipSuccess)
        return PREP_E_HIP;
    return PREP_OK;
}

int prep_server_next(prep_server *s, prep_server_result *out, int64_t timeout_us)
{
    if (!s || !out || timeout_us < 0) return PREP_E_INVALID_ARG;
    std::unique_lock<std::mutex> lock(s->m);
    const int64_t until = now_ns() + timeout_us * 1000;
    while (s->results.empty() && !s->stopping) {
        const int64_t left = until - now_ns();
        if (left <= 0) return 0;
        wait_ns(s->results_ready, lock, left);
    }
    if (s->results.empty()) return 0;
    *out = s->results.front().result;
    s->free_requests.push_back(s->results.front().request);
    s->results.pop_front();
    return 1;
}

int32_t prep_server_next_many(prep_server *s, prep_server_result *out, int32_t cap, int64_t timeout_us)
{
    if (!s || !out || cap < 1 || timeout_us < 0) return PREP_E_INVALID_ARG;
    std::unique_lock<std::mutex> lock(s->m);
    const int64_t until = now_ns() + timeout_us * 1000;
    while (s->results.empty() && !s->stopping) {
        const int64_t left = until - now_ns();
        if (left <= 0) return 0;
        wait_ns(s->results_ready, lock, left);
    }
    int32_t n = 0;
    while (n < cap && !s->results.empty()) {
        out[n++] = s->results.front().result;
        s->free_requests.push_back(s->results.front().request);
        s->results.pop_front();
    }
    return n;
}

int prep_server_release_many(prep_server *s, const prep_server_result *r, int32_t n)
{
    if (!s || !r || n < 0) return PREP_E_INVALID_ARG;
    int rc = PREP_OK;
    {
        std::lock_guard<std::mutex> lock(s->m);
        for (int32_t i = 0; i < n; i++) {
            if (r[i].consumer < 0 || r[i].consumer >= (int32_t)s->consumers.size() || r[i].slot < 0 ||
                r[i].slot >= kOutputSlots || s->consumers[(size_t)r[i].consumer].unreleased[r[i].slot] <= 0) {
                rc = PREP_E_INVALID_ARG;
                continue;
            }
            s->consumers[(size_t)r[i].consumer].unreleased[r[i].slot]--;
        }
    }
    s->slot_free.notify_all();
    return rc;
}

int prep_server_release(prep_server *s, const prep_server_result *r)
{
    return prep_server_release_many(s, r, r ? 1 : -1);
}

}  // extern "C"
