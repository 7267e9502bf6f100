// Sliding window of layer shards: host runtime over one copy stream and
// per-slot events (the scheduler of Sec. 3.3 with hipMemcpyAsync as the loader).
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"

namespace {

enum SlotState { kEmpty = 0, kPrefetched, kAcquired, kReleased };

struct Slot {
    int layer = -1;
    SlotState state = kEmpty;
    hipEvent_t ready = nullptr;   // recorded on the copy stream after the slot's copy
    hipEvent_t freed = nullptr;   // recorded on the compute stream at release
};

}  // namespace

struct tpi_window {
    int n_layers = 0, n_slots = 0;
    size_t layer_bytes = 0;
    std::vector<const void *> blobs;
    char *slots_base = nullptr;
    hipStream_t copy = nullptr;
    std::vector<Slot> slots;
    hipEvent_t first_begin = nullptr, last_done = nullptr;   // timing span of the copies
    bool any_copy = false;
    uint64_t bytes_copied = 0;
    uint64_t n_prefetch = 0;      // the k-th prefetch uses slot k % n_slots (ring order)

    int find(int layer, SlotState st) const
    {
        // oldest first: start at the slot the ring will reuse next
        for (int i = 0; i < n_slots; ++i) {
            int s = (int)((n_prefetch + i) % n_slots);
            if (slots[s].state == st && slots[s].layer == layer) return s;
        }
        return -1;
    }
};

using tpi::fail;

#define TPI_HIP(call)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(TPI_ERUNTIME, "%s: %s", #call, hipGetErrorString(e_));   \
    } while (0)

extern "C" {

int tpi_window_create(tpi_window **out, int32_t n_layers, int32_t window_layers, size_t layer_bytes,
                      const void *const *host_layer_blobs, void *device_slots)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    if (n_layers < 1 || window_layers < 1) return fail(TPI_EINVAL, "n_layers %d / window_layers %d < 1", n_layers, window_layers);
    if (layer_bytes == 0 || !host_layer_blobs || !device_slots) return fail(TPI_EINVAL, "null or empty buffers");
    for (int l = 0; l < n_layers; ++l)
        if (!host_layer_blobs[l]) return fail(TPI_EINVAL, "host blob %d is null", l);
    tpi_window *w = new (std::nothrow) tpi_window;
    if (!w) return fail(TPI_ERUNTIME, "out of host memory");
    w->n_layers = n_layers;
    w->n_slots = window_layers;
    w->layer_bytes = layer_bytes;
    w->blobs.assign(host_layer_blobs, host_layer_blobs + n_layers);
    w->slots_base = static_cast<char *>(device_slots);
    w->slots.resize(window_layers);
    hipError_t e = hipStreamCreateWithFlags(&w->copy, hipStreamNonBlocking);
    for (int i = 0; e == hipSuccess && i < window_layers; ++i) {
        e = hipEventCreateWithFlags(&w->slots[i].ready, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&w->slots[i].freed, hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreate(&w->first_begin);
    if (e == hipSuccess) e = hipEventCreate(&w->last_done);
    if (e != hipSuccess) {
        int rc = fail(TPI_ERUNTIME, "window setup: %s", hipGetErrorString(e));
        for (auto &s : w->slots) {
            if (s.ready) (void)hipEventDestroy(s.ready);
            if (s.freed) (void)hipEventDestroy(s.freed);
        }
        if (w->first_begin) (void)hipEventDestroy(w->first_begin);
        if (w->last_done) (void)hipEventDestroy(w->last_done);
        if (w->copy) (void)hipStreamDestroy(w->copy);
        delete w;
        return rc;
    }
    *out = w;
    return TPI_OK;
}

int tpi_window_prefetch(tpi_window *w, int32_t layer)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    if (layer < 0 || layer >= w->n_layers) return fail(TPI_EINVAL, "layer %d outside [0, %d)", layer, w->n_layers);
    const int si = (int)(w->n_prefetch % w->n_slots);
    Slot &s = w->slots[si];
    if (s.state == kPrefetched || s.state == kAcquired)
        return fail(TPI_ESTATE, "prefetch of layer %d: the window is full, slot %d still holds layer %d (%s)", layer, si,
                    s.layer, s.state == kAcquired ? "acquired, not released" : "prefetched, not yet used");
    // the previous tenant's readers must have finished before the copy lands
    if (s.state == kReleased) TPI_HIP(hipStreamWaitEvent(w->copy, s.freed, 0));
    if (!w->any_copy) TPI_HIP(hipEventRecord(w->first_begin, w->copy));
    TPI_HIP(hipMemcpyAsync(w->slots_base + (size_t)si * w->layer_bytes, w->blobs[layer], w->layer_bytes,
                           hipMemcpyHostToDevice, w->copy));
    TPI_HIP(hipEventRecord(s.ready, w->copy));
    TPI_HIP(hipEventRecord(w->last_done, w->copy));
    w->any_copy = true;
    w->bytes_copied += w->layer_bytes;
    w->n_prefetch += 1;
    s.layer = layer;
    s.state = kPrefetched;
    return TPI_OK;
}

int tpi_window_acquire(tpi_window *w, int32_t layer, void *compute_stream, const void **dev_blob)
{
    if (!w || !dev_blob) return fail(TPI_EINVAL, "null argument");
    if (layer < 0 || layer >= w->n_layers) return fail(TPI_EINVAL, "layer %d outside [0, %d)", layer, w->n_layers);
    const int si = w->find(layer, kPrefetched);
    if (si < 0) return fail(TPI_ESTATE, "acquire of layer %d: no prefetched copy of it is in the window", layer);
    Slot &s = w->slots[si];
    TPI_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, s.ready, 0));
    s.state = kAcquired;
    *dev_blob = w->slots_base + (size_t)si * w->layer_bytes;
    return TPI_OK;
}

int tpi_window_release(tpi_window *w, int32_t layer, void *compute_stream)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    if (layer < 0 || layer >= w->n_layers) return fail(TPI_EINVAL, "layer %d outside [0, %d)", layer, w->n_layers);
    const int si = w->find(layer, kAcquired);
    if (si < 0) return fail(TPI_ESTATE, "release of layer %d: it was not acquired", layer);
    Slot &s = w->slots[si];
    TPI_HIP(hipEventRecord(s.freed, (hipStream_t)compute_stream));
    s.state = kReleased;
    return TPI_OK;
}

int tpi_window_copy_stats(tpi_window *w, double *copy_ms, uint64_t *bytes)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    if (bytes) *bytes = w->bytes_copied;
    if (copy_ms) {
        *copy_ms = 0.0;
        if (w->any_copy) {
            TPI_HIP(hipStreamSynchronize(w->copy));
            float ms = 0.f;
            TPI_HIP(hipEventElapsedTime(&ms, w->first_begin, w->last_done));
            *copy_ms = ms;
        }
    }
    return TPI_OK;
}

int tpi_window_destroy(tpi_window *w)
{
    if (!w) return fail(TPI_EINVAL, "window is null");
    hipError_t e = hipStreamSynchronize(w->copy);
    for (auto &s : w->slots) {
        (void)hipEventDestroy(s.ready);
        (void)hipEventDestroy(s.freed);
    }
    (void)hipEventDestroy(w->first_begin);
    (void)hipEventDestroy(w->last_done);
    (void)hipStreamDestroy(w->copy);
    delete w;
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "hipStreamSynchronize: %s", hipGetErrorString(e));
    return TPI_OK;
}

}  // extern "C"
