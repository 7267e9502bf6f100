// Sliding window of weight blocks: host runtime over one copy queue and
// per-slot events (the scheduler of Sec. 3.3 with asynchronous copies as the
// loader).  The state machine below reaches the device only through
// WindowEngine (window_engine.hpp): the HIP runtime in production, a host
// model of streams and events where the ordering itself is under test.
//
// A block is a contiguous run of bytes in pinned host memory: a whole layer
// shard, or -- at the paper's granularity -- one attention block or one FFN
// block.  Blocks of a slot class share a ring of equally sized HBM slots; a
// retained block (the FFN blocks the scheduler keeps, Prop. 6) has a device
// home of its own, is copied once and never evicted.
#include <hip/hip_runtime.h>

#include <fcntl.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <cstdio>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"
#include "window_engine.hpp"

namespace {

enum SlotState { kEmpty = 0, kPrefetched, kAcquired, kReleased };

struct Slot {
    int block = -1;
    SlotState state = kEmpty;
    void *ready = nullptr;        // recorded on the copy queue after the slot's copy
    void *freed = nullptr;        // recorded on the compute stream at release
};

struct Ring {
    char *base = nullptr;
    size_t slot_bytes = 0;
    int n_slots = 0;
    uint64_t n_prefetch = 0;      // the k-th prefetch of the class uses slot k % n_slots (ring order)
    std::vector<Slot> slots;

    int find(int block, SlotState st) const
    {
        // oldest first: start at the slot the ring will reuse next
        for (int i = 0; i < n_slots; ++i) {
            int s = (int)((n_prefetch + i) % n_slots);
            if (slots[s].state == st && slots[s].block == block) return s;
        }
        return -1;
    }
};

struct Block {
    const void *host = nullptr;   // pinned host memory, or null with the file tier
    int fd = -1;                  // file tier: open file and offset of the block
    uint64_t file_offset = 0;
    size_t bytes = 0;
    int cls = 0;
    char *resident = nullptr;     // non-null: retained block
    bool loaded = false;          // retained: its one copy has been queued
    int acquired = 0;             // retained: acquire / release pairing
    void *ready = nullptr;        // retained: recorded after the copy
};

}  // namespace

// One request to the loader thread: read block -> staging buffer -> dst.
struct LoadRequest {
    int block = -1;
    void *dst = nullptr;
    void *after = nullptr;        // the copy must wait for this event (previous tenant released), may be null
    void *ready = nullptr;        // recorded on the copy queue after the copy
    uint64_t seq = 0;
};

struct tpi_window {
    std::vector<Block> blocks;
    std::vector<Ring> rings;
    tpi::WindowEngine *eng = nullptr;
    bool owns_engine = false;
    void *first_begin = nullptr, *last_done = nullptr;       // timing span of the copies
    bool any_copy = false;
    uint64_t bytes_copied = 0;

    // file tier
    bool file_tier = false;
    std::vector<int> fds;                    // distinct files, closed at destroy
    std::vector<void *> staging;             // pinned buffers, owned by the window
    std::vector<void *> staging_done;        // the staging buffer's last copy has left it
    std::vector<char> staging_used;
    size_t staging_bytes = 0;
    int n_readers = 1;                       // threads that share the read of one block
    std::thread loader;
    std::mutex mu;
    std::condition_variable cv_req, cv_done;
    std::deque<LoadRequest> queue;
    uint64_t n_requested = 0, n_issued = 0;  // requests handed to / finished by the loader
    std::vector<uint64_t> issued_seq;        // per block: sequence number of its latest request
    bool stop = false;
    bool loader_failed = false;
    std::string loader_error;
    double read_seconds = 0.0;               // time the loader spent in pread
};

using tpi::fail;

// ---------------------------------------------------------------------------
// The HIP runtime as the window's engine
// ---------------------------------------------------------------------------
namespace tpi {
namespace {

struct HipEngine final : WindowEngine {
    hipStream_t copy = nullptr;
    int device = 0;
    char text[160] = "";

    int note(hipError_t e, const char *what)
    {
        if (e == hipSuccess) return 0;
        snprintf(text, sizeof(text), "%s: %s", what, hipGetErrorString(e));
        return 1;
    }
    ~HipEngine() override
    {
        if (copy) (void)hipStreamDestroy(copy);
    }
    void *event_create(bool timing) override
    {
        hipEvent_t e = nullptr;
        if (note(timing ? hipEventCreate(&e) : hipEventCreateWithFlags(&e, hipEventDisableTiming), "hipEventCreate")) return nullptr;
        return e;
    }
    void event_destroy(void *ev) override { (void)hipEventDestroy((hipEvent_t)ev); }
    int copy_wait(void *ev) override { return note(hipStreamWaitEvent(copy, (hipEvent_t)ev, 0), "hipStreamWaitEvent"); }
    int copy_h2d(void *dst, const void *src, size_t bytes) override
    {
        return note(hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, copy), "hipMemcpyAsync");
    }
    int copy_record(void *ev) override { return note(hipEventRecord((hipEvent_t)ev, copy), "hipEventRecord"); }
    int copy_sync() override { return note(hipStreamSynchronize(copy), "hipStreamSynchronize"); }
    int stream_wait(void *stream, void *ev) override
    {
        return note(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)ev, 0), "hipStreamWaitEvent");
    }
    int stream_record(void *stream, void *ev) override { return note(hipEventRecord((hipEvent_t)ev, (hipStream_t)stream), "hipEventRecord"); }
    int event_sync(void *ev) override { return note(hipEventSynchronize((hipEvent_t)ev), "hipEventSynchronize"); }
    int elapsed_ms(void *from, void *to, float *ms) override
    {
        return note(hipEventElapsedTime(ms, (hipEvent_t)from, (hipEvent_t)to), "hipEventElapsedTime");
    }
    void *pinned_alloc(size_t bytes) override
    {
        void *p = nullptr;
        if (note(hipHostMalloc(&p, bytes, hipHostMallocDefault), "hipHostMalloc")) return nullptr;
        return p;
    }
    void pinned_free(void *p) override { (void)hipHostFree(p); }
    // A process has few hardware queues (four here) and its streams share them.  When the copy stream shares one
    // with the compute stream, the marker that follows a copy holds back the kernels queued behind it and the
    // copies no longer overlap with compute.  Probe: a 16 MiB copy on the copy stream, then a 4-byte fill on the
    // compute stream; on queues of their own the fill is done long before the copy.  If not, a further stream is
    // created (the earlier ones stay alive meanwhile, so that it lands on another queue) and probed, up to 8.
    int calibrate(void *stream, int *tried) override
    {
        constexpr size_t kBytes = (size_t)16 << 20;
        constexpr int kMaxTries = 8;
        void *host = nullptr, *dev = nullptr;
        hipEvent_t c0 = nullptr, c1 = nullptr, t1 = nullptr;
        hipStream_t rejected[kMaxTries] = {};
        int n_rejected = 0, rc = 0;
        *tried = 0;
        if (note(hipHostMalloc(&host, kBytes, hipHostMallocDefault), "hipHostMalloc")) return 1;
        rc = note(hipMalloc(&dev, kBytes + 256), "hipMalloc");
        if (!rc) rc = note(hipEventCreate(&c0), "hipEventCreate");
        if (!rc) rc = note(hipEventCreate(&c1), "hipEventCreate");
        if (!rc) rc = note(hipEventCreate(&t1), "hipEventCreate");
        hipStream_t cs = (hipStream_t)stream;
        while (!rc) {
            *tried += 1;
            float copy_ms = 0.f, fill_ms = 0.f;
            rc = note(hipStreamSynchronize(cs), "hipStreamSynchronize");
            if (!rc) rc = note(hipStreamSynchronize(copy), "hipStreamSynchronize");
            for (int warm = 0; !rc && warm < 2; ++warm) {          // the second pass is the measurement
                rc = note(hipEventRecord(c0, copy), "hipEventRecord");
                if (!rc) rc = note(hipMemcpyAsync(dev, host, kBytes, hipMemcpyHostToDevice, copy), "hipMemcpyAsync");
                if (!rc) rc = note(hipEventRecord(c1, copy), "hipEventRecord");
                if (!rc) rc = note(hipMemsetAsync(static_cast<char *>(dev) + kBytes, 0, 4, cs), "hipMemsetAsync");
                if (!rc) rc = note(hipEventRecord(t1, cs), "hipEventRecord");
                if (!rc) rc = note(hipEventSynchronize(c1), "hipEventSynchronize");
                if (!rc) rc = note(hipEventSynchronize(t1), "hipEventSynchronize");
            }
            if (!rc) rc = note(hipEventElapsedTime(&copy_ms, c0, c1), "hipEventElapsedTime");
            if (!rc) rc = note(hipEventElapsedTime(&fill_ms, c0, t1), "hipEventElapsedTime");
            if (rc) break;
            if (fill_ms < 0.5f * copy_ms || *tried >= kMaxTries) break;     // independent (or out of tries: keep the last)
            rejected[n_rejected++] = copy;
            hipStream_t fresh = nullptr;
            rc = note(hipStreamCreateWithFlags(&fresh, hipStreamNonBlocking), "hipStreamCreateWithFlags");
            if (rc) { copy = rejected[--n_rejected]; break; }
            copy = fresh;
        }
        for (int i = 0; i < n_rejected; ++i) (void)hipStreamDestroy(rejected[i]);
        if (c0) (void)hipEventDestroy(c0);
        if (c1) (void)hipEventDestroy(c1);
        if (t1) (void)hipEventDestroy(t1);
        if (dev) (void)hipFree(dev);
        if (host) (void)hipHostFree(host);
        return rc;
    }
    int bind_thread() override { return note(hipSetDevice(device), "hipSetDevice"); }
    const char *error_text() override { return text; }
};

}  // namespace

WindowEngine *make_hip_engine()
{
    HipEngine *g = new (std::nothrow) HipEngine;
    if (!g) {
        fail(TPI_ERUNTIME, "out of host memory");
        return nullptr;
    }
    hipError_t e = hipGetDevice(&g->device);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&g->copy, hipStreamNonBlocking);
    if (e != hipSuccess) {
        fail(TPI_ERUNTIME, "window setup: %s", hipGetErrorString(e));
        delete g;
        return nullptr;
    }
    return g;
}

}  // namespace tpi

#define TPI_ENG(w, call)                                                                           \
    do {                                                                                           \
        if ((w)->eng->call) return fail(TPI_ERUNTIME, "%s: %s", #call, (w)->eng->error_text());    \
    } while (0)

namespace {

void destroy_objects(tpi_window *w)
{
    tpi::WindowEngine *g = w->eng;
    for (int fd : w->fds)
        if (fd >= 0) ::close(fd);
    if (!g) return;
    for (auto e : w->staging_done)
        if (e) g->event_destroy(e);
    for (auto p : w->staging)
        if (p) g->pinned_free(p);
    for (auto &r : w->rings)
        for (auto &s : r.slots) {
            if (s.ready) g->event_destroy(s.ready);
            if (s.freed) g->event_destroy(s.freed);
        }
    for (auto &b : w->blocks)
        if (b.ready) g->event_destroy(b.ready);
    if (w->first_begin) g->event_destroy(w->first_begin);
    if (w->last_done) g->event_destroy(w->last_done);
    if (w->owns_engine) delete g;
    w->eng = nullptr;
}

// `after`: event the copy has to wait for (the slot's previous tenant released), or null.
int queue_copy(tpi_window *w, int block, void *dst, void *after, void *ready)
{
    const Block &b = w->blocks[block];
    if (w->file_tier) {
        // hand the request to the loader thread; acquire() waits until it has been carried out
        std::lock_guard<std::mutex> lk(w->mu);
        if (w->loader_failed) return fail(TPI_ERUNTIME, "loader thread: %s", w->loader_error.c_str());
        LoadRequest rq;
        rq.block = block; rq.dst = dst; rq.after = after; rq.ready = ready; rq.seq = ++w->n_requested;
        w->issued_seq[block] = rq.seq;
        w->queue.push_back(rq);
        w->bytes_copied += b.bytes;
        w->cv_req.notify_one();
        return TPI_OK;
    }
    if (after) TPI_ENG(w, copy_wait(after));
    if (!w->any_copy) TPI_ENG(w, copy_record(w->first_begin));
    TPI_ENG(w, copy_h2d(dst, b.host, b.bytes));
    TPI_ENG(w, copy_record(ready));
    TPI_ENG(w, copy_record(w->last_done));
    w->any_copy = true;
    w->bytes_copied += b.bytes;
    return TPI_OK;
}

// File tier: block until the loader has carried out the latest request for `block` (its copy is queued and
// its ready event recorded), so that the caller may make a stream wait for that event.
int wait_issued(tpi_window *w, int block)
{
    if (!w->file_tier) return TPI_OK;
    std::unique_lock<std::mutex> lk(w->mu);
    const uint64_t seq = w->issued_seq[block];
    w->cv_done.wait(lk, [&] { return w->n_issued >= seq || w->loader_failed; });
    if (w->loader_failed) return fail(TPI_ERUNTIME, "loader thread: %s", w->loader_error.c_str());
    return TPI_OK;
}

void loader_fail(tpi_window *w, const std::string &msg)
{
    std::lock_guard<std::mutex> lk(w->mu);
    w->loader_failed = true;
    w->loader_error = msg;
    w->cv_done.notify_all();
}

// The scheduler's daemon thread: requests are carried out strictly in order.
void loader_main(tpi_window *w)
{
    tpi::WindowEngine *g = w->eng;
    if (g->bind_thread()) { loader_fail(w, std::string("loader thread: ") + g->error_text()); return; }
    uint64_t k = 0;
    for (;;) {
        LoadRequest rq;
        {
            std::unique_lock<std::mutex> lk(w->mu);
            w->cv_req.wait(lk, [&] { return w->stop || !w->queue.empty(); });
            if (w->queue.empty()) return;          // stop requested and nothing left to do
            rq = w->queue.front();
            w->queue.pop_front();
        }
        const Block &b = w->blocks[rq.block];
        const int si = (int)(k % w->staging.size());
        k += 1;
        int e = 0;
        if (w->staging_used[si]) e = g->event_sync(w->staging_done[si]);   // its previous copy has left it
        if (e) { loader_fail(w, std::string("waiting for a staging buffer: ") + g->error_text()); return; }
        // read the block from its file: n_readers threads, a contiguous part each (this thread takes the first)
        timespec t0, t1;
        clock_gettime(CLOCK_MONOTONIC, &t0);
        char *dst = static_cast<char *>(w->staging[si]);
        const int parts = (b.bytes >= ((size_t)1 << 20)) ? w->n_readers : 1;
        const size_t per = ((b.bytes + parts - 1) / parts + 4095) & ~(size_t)4095;
        std::vector<std::string> errs(parts);
        auto read_part = [&](int p) {
            size_t lo = std::min(b.bytes, (size_t)p * per), hi = std::min(b.bytes, lo + per);
            while (lo < hi) {
                ssize_t r = ::pread(b.fd, dst + lo, hi - lo, (off_t)(b.file_offset + lo));
                if (r < 0 && errno == EINTR) continue;
                if (r <= 0) {
                    errs[p] = r == 0 ? "block " + std::to_string(rq.block) + ": file ends inside the block"
                                     : "block " + std::to_string(rq.block) + ": pread: " + std::strerror(errno);
                    return;
                }
                lo += (size_t)r;
            }
        };
        {
            std::vector<std::thread> helpers;
            for (int p = 1; p < parts; ++p) helpers.emplace_back(read_part, p);
            read_part(0);
            for (auto &t : helpers) t.join();
        }
        for (const auto &msg : errs)
            if (!msg.empty()) { loader_fail(w, msg); return; }
        clock_gettime(CLOCK_MONOTONIC, &t1);
        if (rq.after) e = g->copy_wait(rq.after);
        if (!e && !w->any_copy) e = g->copy_record(w->first_begin);
        if (!e) e = g->copy_h2d(rq.dst, w->staging[si], b.bytes);
        if (!e) e = g->copy_record(rq.ready);
        if (!e) e = g->copy_record(w->staging_done[si]);
        if (!e) e = g->copy_record(w->last_done);
        if (e) { loader_fail(w, std::string("copy of a block: ") + g->error_text()); return; }
        w->staging_used[si] = 1;
        {
            std::lock_guard<std::mutex> lk(w->mu);
            w->any_copy = true;
            w->n_issued = rq.seq;
            w->read_seconds += (double)(t1.tv_sec - t0.tv_sec) + 1e-9 * (double)(t1.tv_nsec - t0.tv_nsec);
            w->cv_done.notify_all();
        }
    }
}

// stops the loader (after it has carried out everything queued) and joins it
void stop_loader(tpi_window *w)
{
    if (!w->file_tier || !w->loader.joinable()) return;
    {
        std::lock_guard<std::mutex> lk(w->mu);
        w->stop = true;
        w->cv_req.notify_all();
    }
    w->loader.join();
}

}  // namespace

extern "C" {

static int create_common(tpi_window **out, int32_t n_blocks, const tpi_window_block *blocks, int32_t n_classes,
                         const tpi_window_slots *classes, bool need_host, tpi::WindowEngine *borrowed)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    if (n_blocks < 1 || n_classes < 1) return fail(TPI_EINVAL, "n_blocks %d / n_classes %d < 1", n_blocks, n_classes);
    if (!blocks || !classes) return fail(TPI_EINVAL, "null argument");
    for (int c = 0; c < n_classes; ++c)
        if (classes[c].n_slots < 1 || classes[c].slot_bytes == 0 || !classes[c].base)
            return fail(TPI_EINVAL, "slot class %d: null or empty slots", c);
    for (int i = 0; i < n_blocks; ++i) {
        const tpi_window_block &b = blocks[i];
        if ((need_host && !b.host) || b.bytes == 0) return fail(TPI_EINVAL, "block %d: null or empty host memory", i);
        if (b.retained) {
            if (!b.resident) return fail(TPI_EINVAL, "block %d is retained but has no resident device memory", i);
        } else {
            if (b.slot_class < 0 || b.slot_class >= n_classes)
                return fail(TPI_EINVAL, "block %d: slot class %d outside [0, %d)", i, b.slot_class, n_classes);
            if (b.bytes > classes[b.slot_class].slot_bytes)
                return fail(TPI_EINVAL, "block %d: %zu bytes do not fit a slot of class %d (%zu bytes)", i, b.bytes,
                            b.slot_class, classes[b.slot_class].slot_bytes);
        }
    }
    tpi_window *w = new (std::nothrow) tpi_window;
    if (!w) return fail(TPI_ERUNTIME, "out of host memory");
    if (borrowed) {
        w->eng = borrowed;
    } else {
        w->eng = tpi::make_hip_engine();          // sets the error text itself
        w->owns_engine = true;
        if (!w->eng) {
            delete w;
            return TPI_ERUNTIME;
        }
    }
    tpi::WindowEngine *g = w->eng;
    w->blocks.resize(n_blocks);
    w->rings.resize(n_classes);
    bool ok = true;
    for (int c = 0; c < n_classes; ++c) {
        Ring &r = w->rings[c];
        r.base = static_cast<char *>(classes[c].base);
        r.slot_bytes = classes[c].slot_bytes;
        r.n_slots = classes[c].n_slots;
        r.slots.resize(r.n_slots);
        for (int i = 0; ok && i < r.n_slots; ++i) {
            ok = (r.slots[i].ready = g->event_create(false)) != nullptr;
            if (ok) ok = (r.slots[i].freed = g->event_create(false)) != nullptr;
        }
    }
    for (int i = 0; i < n_blocks; ++i) {
        Block &b = w->blocks[i];
        b.host = blocks[i].host;
        b.bytes = blocks[i].bytes;
        b.cls = blocks[i].slot_class;
        b.resident = blocks[i].retained ? static_cast<char *>(blocks[i].resident) : nullptr;
        if (b.resident && ok) ok = (b.ready = g->event_create(false)) != nullptr;
    }
    if (ok) ok = (w->first_begin = g->event_create(true)) != nullptr;
    if (ok) ok = (w->last_done = g->event_create(true)) != nullptr;
    if (!ok) {
        int rc = fail(TPI_ERUNTIME, "window setup: %s", g->error_text());
        destroy_objects(w);
        delete w;
        return rc;
    }
    *out = w;
    return TPI_OK;
}

int tpi_window_create_blocks(tpi_window **out, int32_t n_blocks, const tpi_window_block *blocks, int32_t n_classes,
                             const tpi_window_slots *classes)
{
    return create_common(out, n_blocks, blocks, n_classes, classes, true, nullptr);
}

int tpi_window_create_blocks_sim(tpi_window **out, tpi_sim *sim, int32_t n_blocks, const tpi_window_block *blocks,
                                 int32_t n_classes, const tpi_window_slots *classes)
{
    if (!sim) return fail(TPI_EINVAL, "sim is null");
    return create_common(out, n_blocks, blocks, n_classes, classes, true, tpi_sim_engine(sim));
}

static int create_files_common(tpi_window **out, int32_t n_blocks, const tpi_window_file_block *blocks, int32_t n_classes,
                               const tpi_window_slots *classes, int32_t n_staging, int32_t n_readers,
                               tpi::WindowEngine *borrowed)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    if (n_blocks < 1 || !blocks) return fail(TPI_EINVAL, "null or empty block list");
    if (n_staging < 1) return fail(TPI_EINVAL, "n_staging %d < 1", n_staging);
    if (n_readers < 1 || n_readers > 64) return fail(TPI_EINVAL, "n_readers %d outside [1, 64]", n_readers);
    std::vector<tpi_window_block> plain(n_blocks);
    size_t largest = 0;
    for (int i = 0; i < n_blocks; ++i) {
        if (!blocks[i].path) return fail(TPI_EINVAL, "block %d: path is null", i);
        plain[i] = tpi_window_block{nullptr, blocks[i].bytes, blocks[i].slot_class, blocks[i].retained, blocks[i].resident};
        if (blocks[i].bytes > largest) largest = blocks[i].bytes;
    }
    // open every distinct file once (before anything is created on the device)
    std::vector<std::string> paths;
    std::vector<int> fds, fd_of(n_blocks, -1);
    auto close_all = [&] {
        for (int fd : fds) ::close(fd);
    };
    for (int i = 0; i < n_blocks; ++i) {
        int at = -1;
        for (size_t k = 0; k < paths.size(); ++k)
            if (paths[k] == blocks[i].path) at = (int)k;
        if (at < 0) {
            int fd = ::open(blocks[i].path, O_RDONLY | O_CLOEXEC);
            if (fd < 0) {
                int rc = fail(TPI_EINVAL, "block %d: cannot open %s: %s", i, blocks[i].path, std::strerror(errno));
                close_all();
                return rc;
            }
            paths.push_back(blocks[i].path);
            fds.push_back(fd);
            at = (int)paths.size() - 1;
        }
        fd_of[i] = fds[at];
    }
    tpi_window *w = nullptr;
    int rc = create_common(&w, n_blocks, plain.data(), n_classes, classes, false, borrowed);
    if (rc != TPI_OK) {
        close_all();
        return rc;
    }
    w->fds = fds;                                   // the window closes them from here on
    for (int i = 0; i < n_blocks; ++i) {
        w->blocks[i].fd = fd_of[i];
        w->blocks[i].file_offset = blocks[i].offset;
    }
    auto bail = [&](int code) {
        destroy_objects(w);
        delete w;
        return code;
    };
    w->staging_bytes = largest;
    w->n_readers = n_readers;
    w->staging.assign(n_staging, nullptr);
    w->staging_done.assign(n_staging, nullptr);
    w->staging_used.assign(n_staging, 0);
    w->issued_seq.assign(n_blocks, 0);
    for (int k = 0; k < n_staging; ++k) {
        w->staging[k] = w->eng->pinned_alloc(largest);
        if (w->staging[k]) w->staging_done[k] = w->eng->event_create(false);
        if (!w->staging[k] || !w->staging_done[k])
            return bail(fail(TPI_ERUNTIME, "staging buffers: %s", w->eng->error_text()));
    }
    w->file_tier = true;
    try {
        w->loader = std::thread(loader_main, w);
    } catch (...) {
        w->file_tier = false;
        return bail(fail(TPI_ERUNTIME, "cannot start the loader thread"));
    }
    *out = w;
    return TPI_OK;
}

int tpi_window_create_files(tpi_window **out, int32_t n_blocks, const tpi_window_file_block *blocks, int32_t n_classes,
                            const tpi_window_slots *classes, int32_t n_staging, int32_t n_readers)
{
    return create_files_common(out, n_blocks, blocks, n_classes, classes, n_staging, n_readers, nullptr);
}

int tpi_window_create_files_sim(tpi_window **out, tpi_sim *sim, int32_t n_blocks, const tpi_window_file_block *blocks,
                                int32_t n_classes, const tpi_window_slots *classes, int32_t n_staging, int32_t n_readers)
{
    if (!sim) return fail(TPI_EINVAL, "sim is null");
    return create_files_common(out, n_blocks, blocks, n_classes, classes, n_staging, n_readers, tpi_sim_engine(sim));
}

int tpi_window_read_stats(tpi_window *w, double *read_ms)
{
    if (!w || !read_ms) return fail(TPI_EINVAL, "null argument");
    std::lock_guard<std::mutex> lk(w->mu);
    *read_ms = w->read_seconds * 1e3;
    return TPI_OK;
}

int tpi_window_create(tpi_window **out, int32_t n_layers, int32_t window_layers, size_t layer_bytes,
                      const void *const *host_layer_blobs, void *device_slots)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    if (n_layers < 1 || window_layers < 1) return fail(TPI_EINVAL, "n_layers %d / window_layers %d < 1", n_layers, window_layers);
    if (layer_bytes == 0 || !host_layer_blobs || !device_slots) return fail(TPI_EINVAL, "null or empty buffers");
    std::vector<tpi_window_block> blocks(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        if (!host_layer_blobs[l]) return fail(TPI_EINVAL, "host blob %d is null", l);
        blocks[l] = tpi_window_block{host_layer_blobs[l], layer_bytes, 0, 0, nullptr};
    }
    tpi_window_slots cls{device_slots, layer_bytes, window_layers};
    return tpi_window_create_blocks(out, n_layers, blocks.data(), 1, &cls);
}

int tpi_window_prefetch(tpi_window *w, int32_t layer)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    const int n = (int)w->blocks.size();
    if (layer < 0 || layer >= n) return fail(TPI_EINVAL, "block %d outside [0, %d)", layer, n);
    Block &b = w->blocks[layer];
    if (b.resident) {
        // retained: the first prefetch brings it in for good, later ones find it there
        if (b.loaded) return TPI_OK;
        int rc = queue_copy(w, layer, b.resident, nullptr, b.ready);
        if (rc != TPI_OK) return rc;
        b.loaded = true;
        return TPI_OK;
    }
    Ring &r = w->rings[b.cls];
    const int si = (int)(r.n_prefetch % r.n_slots);
    Slot &s = r.slots[si];
    if (s.state == kPrefetched || s.state == kAcquired)
        return fail(TPI_ESTATE, "prefetch of block %d: the window is full, slot %d of class %d still holds block %d (%s)",
                    layer, si, b.cls, s.block, s.state == kAcquired ? "acquired, not released" : "prefetched, not yet used");
    // the previous tenant's readers must have finished before the copy lands
    int rc = queue_copy(w, layer, r.base + (size_t)si * r.slot_bytes, s.state == kReleased ? s.freed : nullptr, s.ready);
    if (rc != TPI_OK) return rc;
    r.n_prefetch += 1;
    s.block = layer;
    s.state = kPrefetched;
    return TPI_OK;
}

int tpi_window_acquire(tpi_window *w, int32_t layer, void *compute_stream, const void **dev_blob)
{
    if (!w || !dev_blob) return fail(TPI_EINVAL, "null argument");
    const int n = (int)w->blocks.size();
    if (layer < 0 || layer >= n) return fail(TPI_EINVAL, "block %d outside [0, %d)", layer, n);
    Block &b = w->blocks[layer];
    if (b.resident) {
        if (!b.loaded) return fail(TPI_ESTATE, "acquire of retained block %d: it was never prefetched", layer);
        if (int rc = wait_issued(w, layer)) return rc;
        TPI_ENG(w, stream_wait(compute_stream, b.ready));
        b.acquired += 1;
        *dev_blob = b.resident;
        return TPI_OK;
    }
    Ring &r = w->rings[b.cls];
    const int si = r.find(layer, kPrefetched);
    if (si < 0) return fail(TPI_ESTATE, "acquire of block %d: no prefetched copy of it is in the window", layer);
    Slot &s = r.slots[si];
    if (int rc = wait_issued(w, layer)) return rc;
    TPI_ENG(w, stream_wait(compute_stream, s.ready));
    s.state = kAcquired;
    *dev_blob = r.base + (size_t)si * r.slot_bytes;
    return TPI_OK;
}

int tpi_window_release(tpi_window *w, int32_t layer, void *compute_stream)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    const int n = (int)w->blocks.size();
    if (layer < 0 || layer >= n) return fail(TPI_EINVAL, "block %d outside [0, %d)", layer, n);
    Block &b = w->blocks[layer];
    if (b.resident) {
        if (b.acquired < 1) return fail(TPI_ESTATE, "release of block %d: it was not acquired", layer);
        b.acquired -= 1;
        return TPI_OK;
    }
    Ring &r = w->rings[b.cls];
    const int si = r.find(layer, kAcquired);
    if (si < 0) return fail(TPI_ESTATE, "release of block %d: it was not acquired", layer);
    Slot &s = r.slots[si];
    TPI_ENG(w, stream_record(compute_stream, s.freed));
    s.state = kReleased;
    return TPI_OK;
}

int tpi_window_calibrate(tpi_window *w, void *compute_stream, int32_t *tried)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    if (w->any_copy || w->bytes_copied) return fail(TPI_ESTATE, "calibrate belongs before the first prefetch");
    int n = 0;
    if (w->eng->calibrate(compute_stream, &n)) return fail(TPI_ERUNTIME, "calibrate: %s", w->eng->error_text());
    if (tried) *tried = n;
    return TPI_OK;
}

int tpi_window_copy_stats(tpi_window *w, double *copy_ms, uint64_t *bytes)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    if (w->file_tier) {
        std::unique_lock<std::mutex> lk(w->mu);
        // the time span needs everything requested so far to have been handed to the copy stream
        if (copy_ms) w->cv_done.wait(lk, [&] { return w->n_issued >= w->n_requested || w->loader_failed; });
        if (w->loader_failed) return fail(TPI_ERUNTIME, "loader thread: %s", w->loader_error.c_str());
        if (bytes) *bytes = w->bytes_copied;
    } else if (bytes) {
        *bytes = w->bytes_copied;
    }
    if (copy_ms) {
        *copy_ms = 0.0;
        if (w->any_copy) {
            TPI_ENG(w, copy_sync());
            float ms = 0.f;
            TPI_ENG(w, elapsed_ms(w->first_begin, w->last_done, &ms));
            *copy_ms = ms;
        }
    }
    return TPI_OK;
}

int tpi_window_destroy(tpi_window *w)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    stop_loader(w);
    int rc = TPI_OK;
    if (w->eng->copy_sync()) rc = fail(TPI_ERUNTIME, "waiting for the copies: %s", w->eng->error_text());
    destroy_objects(w);
    delete w;
    return rc;
}

}  // extern "C"
