// Sliding window of weight blocks: host runtime over one copy stream and
// per-slot events (the scheduler of Sec. 3.3 with hipMemcpyAsync as the loader).
//
// A block is a contiguous run of bytes in pinned host memory: a whole layer
// shard, or -- at the paper's granularity -- one attention block or one FFN
// block.  Blocks of a slot class share a ring of equally sized HBM slots; a
// retained block (the FFN blocks the scheduler keeps, Prop. 6) has a device
// home of its own, is copied once and never evicted.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"

namespace {

enum SlotState { kEmpty = 0, kPrefetched, kAcquired, kReleased };

struct Slot {
    int block = -1;
    SlotState state = kEmpty;
    hipEvent_t ready = nullptr;   // recorded on the copy stream after the slot's copy
    hipEvent_t freed = nullptr;   // recorded on the compute stream at release
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
    const void *host = nullptr;
    size_t bytes = 0;
    int cls = 0;
    char *resident = nullptr;     // non-null: retained block
    bool loaded = false;          // retained: its one copy has been queued
    int acquired = 0;             // retained: acquire / release pairing
    hipEvent_t ready = nullptr;   // retained: recorded after the copy
};

}  // namespace

struct tpi_window {
    std::vector<Block> blocks;
    std::vector<Ring> rings;
    hipStream_t copy = nullptr;
    hipEvent_t first_begin = nullptr, last_done = nullptr;   // timing span of the copies
    bool any_copy = false;
    uint64_t bytes_copied = 0;
};

using tpi::fail;

#define TPI_HIP(call)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(TPI_ERUNTIME, "%s: %s", #call, hipGetErrorString(e_));   \
    } while (0)

namespace {

void destroy_objects(tpi_window *w)
{
    for (auto &r : w->rings)
        for (auto &s : r.slots) {
            if (s.ready) (void)hipEventDestroy(s.ready);
            if (s.freed) (void)hipEventDestroy(s.freed);
        }
    for (auto &b : w->blocks)
        if (b.ready) (void)hipEventDestroy(b.ready);
    if (w->first_begin) (void)hipEventDestroy(w->first_begin);
    if (w->last_done) (void)hipEventDestroy(w->last_done);
    if (w->copy) (void)hipStreamDestroy(w->copy);
}

int queue_copy(tpi_window *w, void *dst, const Block &b, hipEvent_t ready)
{
    if (!w->any_copy) TPI_HIP(hipEventRecord(w->first_begin, w->copy));
    TPI_HIP(hipMemcpyAsync(dst, b.host, b.bytes, hipMemcpyHostToDevice, w->copy));
    TPI_HIP(hipEventRecord(ready, w->copy));
    TPI_HIP(hipEventRecord(w->last_done, w->copy));
    w->any_copy = true;
    w->bytes_copied += b.bytes;
    return TPI_OK;
}

}  // namespace

extern "C" {

int tpi_window_create_blocks(tpi_window **out, int32_t n_blocks, const tpi_window_block *blocks, int32_t n_classes,
                             const tpi_window_slots *classes)
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
        if (!b.host || b.bytes == 0) return fail(TPI_EINVAL, "block %d: null or empty host memory", i);
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
    w->blocks.resize(n_blocks);
    w->rings.resize(n_classes);
    hipError_t e = hipStreamCreateWithFlags(&w->copy, hipStreamNonBlocking);
    for (int c = 0; c < n_classes; ++c) {
        Ring &r = w->rings[c];
        r.base = static_cast<char *>(classes[c].base);
        r.slot_bytes = classes[c].slot_bytes;
        r.n_slots = classes[c].n_slots;
        r.slots.resize(r.n_slots);
        for (int i = 0; e == hipSuccess && i < r.n_slots; ++i) {
            e = hipEventCreateWithFlags(&r.slots[i].ready, hipEventDisableTiming);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&r.slots[i].freed, hipEventDisableTiming);
        }
    }
    for (int i = 0; i < n_blocks; ++i) {
        Block &b = w->blocks[i];
        b.host = blocks[i].host;
        b.bytes = blocks[i].bytes;
        b.cls = blocks[i].slot_class;
        b.resident = blocks[i].retained ? static_cast<char *>(blocks[i].resident) : nullptr;
        if (b.resident && e == hipSuccess) e = hipEventCreateWithFlags(&b.ready, hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreate(&w->first_begin);
    if (e == hipSuccess) e = hipEventCreate(&w->last_done);
    if (e != hipSuccess) {
        int rc = fail(TPI_ERUNTIME, "window setup: %s", hipGetErrorString(e));
        destroy_objects(w);
        delete w;
        return rc;
    }
    *out = w;
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
        int rc = queue_copy(w, b.resident, b, b.ready);
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
    if (s.state == kReleased) TPI_HIP(hipStreamWaitEvent(w->copy, s.freed, 0));
    int rc = queue_copy(w, r.base + (size_t)si * r.slot_bytes, b, s.ready);
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
        TPI_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, b.ready, 0));
        b.acquired += 1;
        *dev_blob = b.resident;
        return TPI_OK;
    }
    Ring &r = w->rings[b.cls];
    const int si = r.find(layer, kPrefetched);
    if (si < 0) return fail(TPI_ESTATE, "acquire of block %d: no prefetched copy of it is in the window", layer);
    Slot &s = r.slots[si];
    TPI_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, s.ready, 0));
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
    destroy_objects(w);
    delete w;
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "hipStreamSynchronize: %s", hipGetErrorString(e));
    return TPI_OK;
}

}  // extern "C"
