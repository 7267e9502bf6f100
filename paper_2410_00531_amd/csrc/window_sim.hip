// Host model of the device side of the sliding window (Sec. 3.3): queues that
// execute in order, events, asynchronous copies, and "kernels" that read a
// range of memory.  Nothing runs when it is queued; the model executes the
// queued operations later, always choosing at random (seeded) among the queues
// whose next operation may run.  Every order the real device could choose --
// subject to queue order and event waits only -- is therefore possible, and a
// window that lets a copy overtake a reader, or a reader overtake its copy,
// shows up as a wrong hash in some of the orders.  Beside the order the model
// keeps time: every queue has a clock, a copy takes bytes / rate, a kernel the
// cost its caller states, a wait moves the clock to the recording's time --
// the times depend on the dependencies only, not on the order drawn.  No
// device is touched: "device memory" is ordinary host memory of the caller.
#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"
#include "window_engine.hpp"

using tpi::fail;

namespace {

enum OpKind { kCopy, kRecord, kWait, kRead };

struct Op {
    OpKind kind;
    void *dst = nullptr;
    const void *src = nullptr;
    size_t bytes = 0;
    uint64_t rec = 0;          // kRecord: id of this recording; kWait: the recording waited for
    uint64_t *out = nullptr;   // kRead: receives the hash
    double cost = 0.0;         // kRead: duration in model milliseconds
    double *start = nullptr;   // kRead: receives the time it started, may be null
};

struct SimEvent {
    uint64_t last_rec = 0;     // id of the latest recording queued for this event (0: never recorded)
};

struct SimQueue {
    std::deque<Op> ops;
    double clock = 0.0;        // model time at which the queue's next operation can start
};

uint64_t fnv1a(const void *p, size_t n)
{
    const unsigned char *b = static_cast<const unsigned char *>(p);
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
    return h;
}

}  // namespace

struct tpi_sim final : tpi::WindowEngine {
    std::mutex mu;
    std::vector<SimQueue *> queues;          // [0] is the copy queue
    std::vector<double> rec_time;            // per recording id: model time when it ran, < 0 while pending
    std::vector<SimEvent *> events;
    uint64_t rng;
    double bytes_per_ms = 1e6;               // rate of the copy queue
    uint64_t executed = 0;
    char text[160] = "";

    explicit tpi_sim(uint64_t seed) : rng(seed * 0x9E3779B97F4A7C15ull + 0x632BE59BD9B4E019ull)
    {
        queues.push_back(new SimQueue);
        rec_time.push_back(0.0);             // id 0: "never recorded", counts as done
    }
    ~tpi_sim() override
    {
        for (auto q : queues) delete q;
        for (auto e : events) delete e;
    }
    uint64_t next_random()
    {
        rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
        return rng;
    }
    bool runnable(const SimQueue *q) const
    {
        if (q->ops.empty()) return false;
        const Op &o = q->ops.front();
        return o.kind != kWait || rec_time[o.rec] >= 0.0;
    }
    void execute(SimQueue *q)
    {
        Op o = q->ops.front();
        q->ops.pop_front();
        switch (o.kind) {
        case kCopy: std::memcpy(o.dst, o.src, o.bytes); q->clock += (double)o.bytes / bytes_per_ms; break;
        case kRecord: rec_time[o.rec] = q->clock; break;
        case kWait: if (rec_time[o.rec] > q->clock) q->clock = rec_time[o.rec]; break;
        case kRead:
            if (o.out) *o.out = fnv1a(o.src, o.bytes);
            if (o.start) *o.start = q->clock;
            q->clock += o.cost;
            break;
        }
        executed += 1;
    }
    // Runs operations until done() holds; false when it does not hold and nothing more can run.  mu is held.
    template <class Pred>
    bool run_until(Pred done)
    {
        std::vector<SimQueue *> ready;
        while (!done()) {
            ready.clear();
            for (auto q : queues)
                if (runnable(q)) ready.push_back(q);
            if (ready.empty()) return false;
            execute(ready[next_random() % ready.size()]);
        }
        return true;
    }
    int stuck(const char *what)
    {
        snprintf(text, sizeof(text), "the modelled device cannot make progress (%s)", what);
        return 1;
    }
    uint64_t queue_record(SimQueue *q, SimEvent *e)
    {
        const uint64_t id = rec_time.size();
        rec_time.push_back(-1.0);
        Op o; o.kind = kRecord; o.rec = id;
        q->ops.push_back(o);
        e->last_rec = id;
        return id;
    }
    void queue_wait(SimQueue *q, SimEvent *e)
    {
        if (!e->last_rec) return;                // an event never recorded holds nobody back
        Op o; o.kind = kWait; o.rec = e->last_rec;
        q->ops.push_back(o);
    }
    SimQueue *stream_of(void *handle)
    {
        if (!handle) {                            // the null stream: one queue of its own
            if (queues.size() < 2) queues.push_back(new SimQueue);
            return queues[1];
        }
        for (auto q : queues)
            if (q == handle) return q;
        return nullptr;
    }

    // ---- WindowEngine ----
    void *event_create(bool) override
    {
        std::lock_guard<std::mutex> lk(mu);
        events.push_back(new SimEvent);
        return events.back();
    }
    void event_destroy(void *) override {}        // owned by the model until it is destroyed
    int copy_wait(void *ev) override
    {
        std::lock_guard<std::mutex> lk(mu);
        queue_wait(queues[0], static_cast<SimEvent *>(ev));
        return 0;
    }
    int copy_h2d(void *dst, const void *src, size_t bytes) override
    {
        std::lock_guard<std::mutex> lk(mu);
        Op o; o.kind = kCopy; o.dst = dst; o.src = src; o.bytes = bytes;
        queues[0]->ops.push_back(o);
        return 0;
    }
    int copy_record(void *ev) override
    {
        std::lock_guard<std::mutex> lk(mu);
        queue_record(queues[0], static_cast<SimEvent *>(ev));
        return 0;
    }
    int copy_sync() override
    {
        std::lock_guard<std::mutex> lk(mu);
        return run_until([&] { return queues[0]->ops.empty(); }) ? 0 : stuck("copy queue");
    }
    int stream_wait(void *stream, void *ev) override
    {
        std::lock_guard<std::mutex> lk(mu);
        SimQueue *q = stream_of(stream);
        if (!q) { snprintf(text, sizeof(text), "not a stream of this model"); return 1; }
        queue_wait(q, static_cast<SimEvent *>(ev));
        return 0;
    }
    int stream_record(void *stream, void *ev) override
    {
        std::lock_guard<std::mutex> lk(mu);
        SimQueue *q = stream_of(stream);
        if (!q) { snprintf(text, sizeof(text), "not a stream of this model"); return 1; }
        queue_record(q, static_cast<SimEvent *>(ev));
        return 0;
    }
    int event_sync(void *ev) override
    {
        std::lock_guard<std::mutex> lk(mu);
        const uint64_t id = static_cast<SimEvent *>(ev)->last_rec;
        return run_until([&] { return rec_time[id] >= 0.0; }) ? 0 : stuck("event");
    }
    int elapsed_ms(void *from, void *to, float *ms) override
    {
        std::lock_guard<std::mutex> lk(mu);
        const uint64_t a = static_cast<SimEvent *>(from)->last_rec, b = static_cast<SimEvent *>(to)->last_rec;
        if (rec_time[a] < 0.0 || rec_time[b] < 0.0) { snprintf(text, sizeof(text), "event not reached yet"); return 1; }
        *ms = (float)(rec_time[b] - rec_time[a]);
        return 0;
    }
    void *pinned_alloc(size_t bytes) override { return ::operator new(bytes, std::nothrow); }
    void pinned_free(void *p) override { ::operator delete(p); }
    int calibrate(void *, int *tried) override { *tried = 1; return 0; }   // the model's queues never share anything
    int bind_thread() override { return 0; }
    const char *error_text() override { return text; }
};

tpi::WindowEngine *tpi_sim_engine(tpi_sim *sim) { return sim; }

extern "C" {

int tpi_sim_create(tpi_sim **out, uint64_t seed)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = new (std::nothrow) tpi_sim(seed);
    if (!*out) return fail(TPI_ERUNTIME, "out of host memory");
    return TPI_OK;
}

void *tpi_sim_stream(tpi_sim *sim)
{
    if (!sim) return nullptr;
    std::lock_guard<std::mutex> lk(sim->mu);
    if (sim->queues.size() < 2) sim->queues.push_back(new SimQueue);   // [1] stays the null stream's queue
    sim->queues.push_back(new SimQueue);
    return sim->queues.back();
}

int tpi_sim_read(tpi_sim *sim, void *stream, const void *ptr, size_t bytes, double cost_ms, uint64_t *host_hash,
                 double *host_start_ms)
{
    if (!sim) return fail(TPI_EINVAL, "sim is null");
    if ((bytes && (!ptr || !host_hash)) || !(cost_ms >= 0.0)) return fail(TPI_EINVAL, "null range or negative cost");
    std::lock_guard<std::mutex> lk(sim->mu);
    SimQueue *q = sim->stream_of(stream);
    if (!q || q == sim->queues[0]) return fail(TPI_EINVAL, "not a compute stream of this model");
    Op o; o.kind = kRead; o.src = ptr; o.bytes = bytes; o.out = bytes ? host_hash : nullptr; o.cost = cost_ms;
    o.start = host_start_ms;
    q->ops.push_back(o);
    return TPI_OK;
}

int tpi_sim_set_copy_rate(tpi_sim *sim, double bytes_per_ms)
{
    if (!sim || !(bytes_per_ms > 0.0)) return fail(TPI_EINVAL, "null model or rate <= 0");
    std::lock_guard<std::mutex> lk(sim->mu);
    sim->bytes_per_ms = bytes_per_ms;
    return TPI_OK;
}

int tpi_sim_stream_time(tpi_sim *sim, void *stream, double *host_ms)
{
    if (!sim || !host_ms) return fail(TPI_EINVAL, "null argument");
    std::lock_guard<std::mutex> lk(sim->mu);
    SimQueue *q = sim->stream_of(stream);
    if (!q) return fail(TPI_EINVAL, "not a stream of this model");
    *host_ms = q->clock;
    return TPI_OK;
}

int tpi_sim_run(tpi_sim *sim)
{
    if (!sim) return fail(TPI_EINVAL, "sim is null");
    std::lock_guard<std::mutex> lk(sim->mu);
    auto all_empty = [&] {
        for (auto q : sim->queues)
            if (!q->ops.empty()) return false;
        return true;
    };
    if (!sim->run_until(all_empty)) return fail(TPI_ESTATE, "operations are left that wait for an event nobody will record");
    return TPI_OK;
}

uint64_t tpi_sim_hash(const void *ptr, size_t bytes) { return ptr ? fnv1a(ptr, bytes) : 0; }

int tpi_sim_destroy(tpi_sim *sim)
{
    if (!sim) return fail(TPI_EINVAL, "sim is null");
    delete sim;
    return TPI_OK;
}

}  // extern "C"
