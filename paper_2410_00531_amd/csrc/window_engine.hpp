// What the sliding window (Sec. 3.3) needs from the device runtime: one copy
// queue, events, and the two ways a compute stream meets an event.  The slot
// state machine in window.hip talks to this interface only, so it runs
// unchanged on the HIP runtime (HipEngine) and on a host-side model of streams
// and events (tpi_sim, window_sim.hip) that executes the queued operations in
// a seeded random order and so exposes any read of a slot before its copy, or
// any copy over a slot that is still being read.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace tpi {

struct WindowEngine {
    virtual ~WindowEngine() {}
    // events; `timing`: elapsed_ms may be asked of it.  Null on failure.
    virtual void *event_create(bool timing) = 0;
    virtual void event_destroy(void *ev) = 0;
    // the copy queue: strictly in order
    virtual int copy_wait(void *ev) = 0;                                     // later copies wait for ev
    virtual int copy_h2d(void *dst, const void *src, size_t bytes) = 0;      // asynchronous
    virtual int copy_record(void *ev) = 0;
    virtual int copy_sync() = 0;                                             // host waits for the queue
    // a compute stream of the caller
    virtual int stream_wait(void *stream, void *ev) = 0;                     // acquire
    virtual int stream_record(void *stream, void *ev) = 0;                   // release
    // host side
    virtual int event_sync(void *ev) = 0;
    virtual int elapsed_ms(void *from, void *to, float *ms) = 0;
    virtual void *pinned_alloc(size_t bytes) = 0;                            // staging buffers of the file tier
    virtual void pinned_free(void *p) = 0;
    // Makes sure that work on the copy queue does not hold back work queued on `stream` afterwards (see
    // tpi_window_calibrate); *tried receives the number of copy queues tried.  Nothing may be queued on the copy queue.
    virtual int calibrate(void *stream, int *tried) = 0;
    virtual int bind_thread() = 0;          // called once by the loader thread before it uses the engine
    virtual const char *error_text() = 0;   // of the last call that returned nonzero
};

// The HIP runtime: a non-blocking stream of default priority for the copies.  Null (and tpi_last_error
// set) when the stream cannot be created.
WindowEngine *make_hip_engine();

}  // namespace tpi

// Host model of streams and events (declared in tpi.h as an opaque type).  The window borrows it.
struct tpi_sim;
tpi::WindowEngine *tpi_sim_engine(tpi_sim *sim);
