// Measurement aid, not part of the method: what a hand-over between two dependent streaming stages costs on this
// chip, in the three ways a decode layer's stages (Alg. 2 loop body) could be chained.
//
// 256 workgroups of 8 streaming waves and one control wave read a buffer once, each wave its own contiguous
// region through a ring of 16 registers (16 KiB in flight per wave, 33 MB on the chip).  The stream is cut into
// segments; a segment stands for a stage (its bytes for the stage's weights) and may only be consumed once the
// previous segment's results are known:
//   mode 0  no hand-over: the segments follow each other freely (the streaming rate itself)
//   mode 1  hand-over inside the workgroup: the 8 waves report through LDS, the control wave releases them
//   mode 2  hand-over across the chip inside one kernel: every workgroup's control wave writes the workgroup's
//           result through to memory, joins a two-level counter tree (8 groups, a root), waits for its group's
//           flag, reads all 256 results (ordinary loads of lines no compute unit has touched before) and
//           releases its waves; the rings keep loading the next segment's data meanwhile
//   mode 3  hand-over by kernel boundary: one launch per segment on one stream
// In every mode the results are checked (the sum over all workgroups that each workgroup read back), so the
// hand-over is a real one.  All waits are bounded; a wait that gives up is reported, and the kernel still ends.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"

using tpi::fail;

namespace {

typedef unsigned long long u64;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_ptr;

constexpr int kWorkers = 8, kGroups = 8, kDepth = 16, kWgs = 256;
constexpr int kPad = 256;                  // 32-bit words between counters (1 KiB)
constexpr u64 kSpinLimitTicks = 2000000;   // 20 ms of the 100 MHz clock

__device__ __forceinline__ unsigned ld_dev(const unsigned *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(unsigned *p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned add_dev(unsigned *p, unsigned v) { return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

__global__ void k_probe_fill(unsigned *p, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        unsigned x = (unsigned)i * 2654435761u;
        x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
        p[i] = (x & 0x007fffffu) | 0x3f000000u;    // floats in [0.5, 1): the chip's clock depends on the data
    }
}

// expected word of (segment k, workgroup g): wrap-around sum of the segment's 32-bit words over the 8 waves
__global__ __launch_bounds__(64) void k_probe_ref(const uint4 *buf, size_t chunks_per_wave, int seg, unsigned *out)
{
    const int k = blockIdx.y, g = blockIdx.x;
    unsigned s = 0;
    for (int w = 0; w < kWorkers; ++w) {
        const uint4 *p = buf + ((size_t)(g * kWorkers + w) * chunks_per_wave + (size_t)k * seg) * 64 + threadIdx.x;
        for (int c = 0; c < seg; ++c) { uint4 v = p[(size_t)c * 64]; s += v.x + v.y + v.z + v.w; }
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) out[(size_t)k * kWgs + g] = s;
}

struct ProbeArgs {
    const uint4 *buf;
    size_t chunks_per_wave;   // 1 KiB chunks of a wave's whole region (stride between waves)
    size_t first_chunk;       // mode 3: the launch covers chunks first_chunk .. first_chunk + seg - 1 of every wave
    int seg, nseg;            // chunks per segment, segments this launch walks
    int k0;                   // index of the launch's first segment (row of `out`)
    unsigned *out;            // [segments][kWgs] results, a fresh row per segment
    unsigned *grp, *root, *go;
    unsigned bar_base;        // barriers completed by earlier launches
    unsigned *err;            // [2]: code, segment
    unsigned *check;          // [kWgs] segments whose total was right
    const unsigned *expect;   // [segments] expected totals
    u64 *stamps;              // [segments][kWgs][4]: results in, group answered, results of all read, next segment's first batch
    int mode;
};

__global__ __launch_bounds__((kWorkers + 1) * 64) void k_probe_stream(ProbeArgs a)
{
    __shared__ unsigned s_res[kWorkers];
    __shared__ unsigned s_done, s_ready, s_dead;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wg = blockIdx.x;
    if (threadIdx.x == 0) { s_done = 0; s_ready = 0; s_dead = 0; }
    __syncthreads();
    if (wave == kWorkers) {
        // ---------------- control wave ----------------
        if (a.mode == 0) return;
        const int g = wg % kGroups, gsize = (kWgs - g + kGroups - 1) / kGroups;
        unsigned good = 0;
        bool dead = false;
        for (int k = 0; k < a.nseg; ++k) {
            const u64 t0 = wall_clock64();
            while (!dead && __hip_atomic_load(&s_done, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (unsigned)(k + 1) * kWorkers) {
                __builtin_amdgcn_s_sleep(1);
                if (wall_clock64() - t0 > kSpinLimitTicks) {
                    dead = true;
                    if (lane == 0) { a.err[0] = 1; a.err[1] = k; __hip_atomic_store(&s_dead, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
                }
            }
            u64 *stp = a.stamps ? a.stamps + ((size_t)(a.k0 + k) * kWgs + wg) * 4 : nullptr;
            if (stp && lane == 0) stp[0] = wall_clock64();
            unsigned word = 0;
            for (int w = 0; w < kWorkers; ++w) word += s_res[w];
            if (a.mode == 1) {
                if (lane == 0) __hip_atomic_store(&s_ready, (unsigned)(k + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                continue;
            }
            if (lane == 0) st_dev(a.out + (size_t)(a.k0 + k) * kWgs + wg, word);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (a.mode == 3) continue;                        // the kernel boundary is the hand-over
            const unsigned b = a.bar_base + k + 1;            // barrier number over the life of the counters
            if (lane == 0 && !dead) {
                unsigned old = add_dev(a.grp + g * kPad, 1u);
                if (stp) stp[1] = wall_clock64();
                if (old == (unsigned)gsize * b - 1u) {
                    add_dev(a.root, 1u);
                    const u64 t1 = wall_clock64();
                    while (ld_dev(a.root) < (unsigned)kGroups * b)
                        if (wall_clock64() - t1 > kSpinLimitTicks) { a.err[0] = 2; a.err[1] = k; break; }
                    st_dev(a.go + g * kPad, b);
                }
            }
            {
                const u64 t1 = wall_clock64();
                while (!dead && ld_dev(a.go + g * kPad) < b) {
                    __builtin_amdgcn_s_sleep(1);
                    if (wall_clock64() - t1 > kSpinLimitTicks) {
                        dead = true;
                        if (lane == 0) { a.err[0] = 3; a.err[1] = k; __hip_atomic_store(&s_dead, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
                    }
                }
            }
            unsigned tot = 0;
            for (int i = lane; i < kWgs; i += 64) tot += a.out[(size_t)(a.k0 + k) * kWgs + i];
            for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o, 64);
            if (stp && lane == 0) stp[2] = wall_clock64();
            if (tot == a.expect[a.k0 + k]) good += 1;
            if (lane == 0) __hip_atomic_store(&s_ready, (unsigned)(k + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (lane == 0 && a.mode == 2) a.check[wg] = good;
        return;
    }
    // ---------------- streaming waves ----------------
    const size_t gw = (size_t)wg * kWorkers + wave;
    const uint4 *p = a.buf + (gw * a.chunks_per_wave + a.first_chunk) * 64 + lane;
    const size_t n = (size_t)a.seg * a.nseg;
    v4u r[kDepth];
#pragma unroll
    for (int s = 0; s < kDepth; ++s) r[s] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p + (size_t)(s < (int)n ? s : n - 1) * 64));
    unsigned acc = 0;
    int seg_left = a.seg, k = 0;
    // a batch of kDepth chunks at a time: wait for the input (first batch of a segment), consume the batch, report a
    // finished segment, and only then request the next batch
    for (size_t c = 0; c < n; c += kDepth) {
        const bool seg_first = seg_left == a.seg;
        if (seg_first && k > 0 && a.mode != 0) {
            const u64 t0 = wall_clock64();
            while (__hip_atomic_load(&s_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < (unsigned)k &&
                   !__hip_atomic_load(&s_dead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) {
                __builtin_amdgcn_s_sleep(1);
                if (wall_clock64() - t0 > 2 * kSpinLimitTicks) { if (lane == 0) { a.err[0] = 4; a.err[1] = k; } break; }
            }
        }
#pragma unroll
        for (int s = 0; s < kDepth; ++s) {
            v4u v = r[s];
            acc += v.x + v.y + v.z + v.w;
        }
        if (a.stamps && wave == 0 && lane == 0 && seg_first && k > 0 && acc != 0x12345u)
            a.stamps[((size_t)(a.k0 + k - 1) * kWgs + wg) * 4 + 3] = wall_clock64();
        seg_left -= kDepth;
        if (seg_left == 0) {
            for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
            // LDS operations of one wave are carried out in order: no fence (a release would also wait for the
            // ring's loads in flight)
            if (lane == 0)
                asm volatile("ds_write_b32 %0, %1\n s_waitcnt lgkmcnt(0)\n ds_add_u32 %2, %3\n s_waitcnt lgkmcnt(0)"
                             :: "v"((unsigned)(uintptr_t)(lds_ptr)&s_res[wave]), "v"(acc),
                                "v"((unsigned)(uintptr_t)(lds_ptr)&s_done), "v"(1u) : "memory");
            acc = 0; seg_left = a.seg; ++k;
        }
#pragma unroll
        for (int s = 0; s < kDepth; ++s) {
            size_t nc = c + s + kDepth;
            if (nc > n - 1) nc = n - 1;
            r[s] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p + nc * 64));
        }
    }
}

struct Buffers {
    uint4 *buf = nullptr;
    unsigned *out = nullptr, *ref = nullptr, *cnt = nullptr, *err = nullptr, *check = nullptr, *expect = nullptr;
    u64 *stamps = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Buffers()
    {
        for (void *p : {(void *)buf, (void *)out, (void *)ref, (void *)cnt, (void *)err, (void *)check, (void *)expect, (void *)stamps})
            if (p) (void)hipFree(p);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace

#define PROBE_HIP(call)                                                                            \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(TPI_ERUNTIME, "%s: %s", #call, hipGetErrorString(e_));   \
    } while (0)

extern "C" int tpi_probe_handover(uint64_t total_bytes, int32_t segment_kib_per_wave, int32_t mode, int32_t reps,
                                  tpi_probe_result *host_out, void *stream)
{
    if (!host_out) return fail(TPI_EINVAL, "host_out is null");
    if (mode < 0 || mode > 3) return fail(TPI_EINVAL, "mode %d outside [0, 3]", mode);
    if (reps < 1 || reps > 100) return fail(TPI_EINVAL, "reps %d outside [1, 100]", reps);
    const size_t n_waves = (size_t)kWgs * kWorkers;
    if (segment_kib_per_wave < kDepth || segment_kib_per_wave % kDepth)
        return fail(TPI_EINVAL, "segment_kib_per_wave %d must be a positive multiple of %d", segment_kib_per_wave, kDepth);
    const size_t cpw = total_bytes / 1024 / n_waves;
    if (cpw < (size_t)segment_kib_per_wave || cpw % segment_kib_per_wave || total_bytes != cpw * 1024 * n_waves)
        return fail(TPI_EINVAL, "total_bytes must be a multiple of %zu (2048 waves x the segment)", n_waves * 1024 * (size_t)segment_kib_per_wave);
    const int seg = segment_kib_per_wave, nseg = (int)(cpw / seg);
    if (nseg > 4096) return fail(TPI_EINVAL, "%d segments: at most 4096", nseg);
    hipStream_t st = (hipStream_t)stream;
    Buffers B;
    PROBE_HIP(hipMalloc(&B.buf, total_bytes));
    PROBE_HIP(hipMalloc(&B.out, (size_t)nseg * kWgs * 4));
    PROBE_HIP(hipMalloc(&B.ref, (size_t)nseg * kWgs * 4));
    PROBE_HIP(hipMalloc(&B.cnt, 3 * kGroups * kPad * 4));
    PROBE_HIP(hipMalloc(&B.err, 8));
    PROBE_HIP(hipMalloc(&B.check, kWgs * 4));
    PROBE_HIP(hipMalloc(&B.expect, (size_t)nseg * 4));
    PROBE_HIP(hipMalloc(&B.stamps, (size_t)nseg * kWgs * 4 * 8));
    PROBE_HIP(hipEventCreate(&B.e0));
    PROBE_HIP(hipEventCreate(&B.e1));
    PROBE_HIP(hipMemsetAsync(B.cnt, 0, 3 * kGroups * kPad * 4, st));
    PROBE_HIP(hipMemsetAsync(B.err, 0, 8, st));
    hipLaunchKernelGGL(k_probe_fill, dim3(4096), dim3(256), 0, st, (unsigned *)B.buf, total_bytes / 4);
    hipLaunchKernelGGL(k_probe_ref, dim3(kWgs, nseg), dim3(64), 0, st, B.buf, cpw, seg, B.ref);
    std::vector<unsigned> ref((size_t)nseg * kWgs), expect(nseg, 0);
    PROBE_HIP(hipMemcpyAsync(ref.data(), B.ref, ref.size() * 4, hipMemcpyDeviceToHost, st));
    PROBE_HIP(hipStreamSynchronize(st));
    for (int k = 0; k < nseg; ++k)
        for (int g = 0; g < kWgs; ++g) expect[k] += ref[(size_t)k * kWgs + g];
    PROBE_HIP(hipMemcpyAsync(B.expect, expect.data(), (size_t)nseg * 4, hipMemcpyHostToDevice, st));

    tpi_probe_result res{};
    res.segments = nseg;
    res.segment_mb = (double)seg * 1024.0 * n_waves / 1e6;
    double best_ms = 1e30;
    unsigned bar_base = 0;
    std::vector<u64> stamps((size_t)nseg * kWgs * 4);
    for (int rep = 0; rep < reps; ++rep) {
        PROBE_HIP(hipMemsetAsync(B.out, 0, (size_t)nseg * kWgs * 4, st));
        PROBE_HIP(hipMemsetAsync(B.check, 0, kWgs * 4, st));
        PROBE_HIP(hipMemsetAsync(B.stamps, 0, stamps.size() * 8, st));
        ProbeArgs a{};
        a.buf = B.buf; a.chunks_per_wave = cpw; a.seg = seg; a.out = B.out;
        a.grp = B.cnt; a.root = B.cnt + kGroups * kPad; a.go = B.cnt + 2 * kGroups * kPad;
        a.bar_base = bar_base; a.err = B.err; a.check = B.check; a.expect = B.expect;
        a.stamps = mode == 2 ? B.stamps : nullptr; a.mode = mode;
        PROBE_HIP(hipEventRecord(B.e0, st));
        if (mode == 3) {
            for (int k = 0; k < nseg; ++k) {
                a.first_chunk = (size_t)k * seg; a.nseg = 1; a.k0 = k;
                hipLaunchKernelGGL(k_probe_stream, dim3(kWgs), dim3((kWorkers + 1) * 64), 0, st, a);
            }
        } else {
            a.first_chunk = 0; a.nseg = nseg; a.k0 = 0;
            hipLaunchKernelGGL(k_probe_stream, dim3(kWgs), dim3((kWorkers + 1) * 64), 0, st, a);
        }
        PROBE_HIP(hipGetLastError());
        PROBE_HIP(hipEventRecord(B.e1, st));
        PROBE_HIP(hipEventSynchronize(B.e1));
        if (mode == 2) bar_base += nseg;
        float ms = 0.f;
        PROBE_HIP(hipEventElapsedTime(&ms, B.e0, B.e1));
        unsigned err[2] = {0, 0};
        PROBE_HIP(hipMemcpy(err, B.err, 8, hipMemcpyDeviceToHost));
        if (err[0]) {
            res.gave_up = (int)err[0];
            *host_out = res;
            return fail(TPI_ERUNTIME, "a bounded wait of the probe gave up (kind %u, segment %u)", err[0], err[1]);
        }
        // the results: mode 2 checked them on the device (every workgroup, every segment); mode 3 is checked here
        int ok = 1;
        if (mode == 2) {
            std::vector<unsigned> chk(kWgs);
            PROBE_HIP(hipMemcpy(chk.data(), B.check, kWgs * 4, hipMemcpyDeviceToHost));
            for (unsigned v : chk) ok = ok && v == (unsigned)nseg;
        } else if (mode == 3) {
            std::vector<unsigned> out((size_t)nseg * kWgs);
            PROBE_HIP(hipMemcpy(out.data(), B.out, out.size() * 4, hipMemcpyDeviceToHost));
            ok = out == ref;
        }
        res.results_ok = (rep == 0 || res.results_ok) && ok;
        if (ms < best_ms) {
            best_ms = ms;
            if (mode == 2) {
                PROBE_HIP(hipMemcpy(stamps.data(), B.stamps, stamps.size() * 8, hipMemcpyDeviceToHost));
                // per segment: spread = last minus first "results in"; chain = mean "next segment's first batch
                // consumed" minus the last "results in"
                double spread = 0, chain = 0; int cnt = 0;
                for (int k = 1; k + 1 < nseg; ++k) {
                    u64 lo = ~0ull, hi = 0; double next = 0;
                    for (int g = 0; g < kWgs; ++g) {
                        const u64 *s = &stamps[((size_t)k * kWgs + g) * 4];
                        if (s[0] < lo) lo = s[0];
                        if (s[0] > hi) hi = s[0];
                        next += (double)s[3];
                    }
                    spread += (double)(hi - lo) * 0.01;
                    chain += (next / kWgs - (double)hi) * 0.01;
                    ++cnt;
                }
                res.spread_us = cnt ? spread / cnt : 0.0;
                res.chain_us = cnt ? chain / cnt : 0.0;
            }
        }
    }
    res.us_total = best_ms * 1e3;
    res.tb_per_s = (double)total_bytes / (best_ms * 1e-3) / 1e12;
    res.us_per_segment = best_ms * 1e3 / nseg;
    *host_out = res;
    return TPI_OK;
}
