// Device-side building blocks shared by the decode kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tpi {

constexpr int kWave = 64;
constexpr int kBlock = 256;              // threads per workgroup of every streaming kernel
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kChunk = kBlock * 4;       // floats one workgroup covers with one float4 per thread

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Streaming 16-byte load of weights that are read exactly once: the
// non-temporal hint keeps them from displacing the activation vectors in L2.
__device__ __forceinline__ float4 load_stream4(const float *p)
{
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ float dot4(float4 a, float4 b, float acc)
{
    acc = fmaf(a.x, b.x, acc);
    acc = fmaf(a.y, b.y, acc);
    acc = fmaf(a.z, b.z, acc);
    acc = fmaf(a.w, b.w, acc);
    return acc;
}

// Sum over the workgroup of one value per thread; every thread gets the
// result.  red: kWavesPerBlock floats of LDS.  Contains two barriers.
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) s += red[w];
    __syncthreads();
    return s;
}

// The slice of an input vector that one thread multiplies with: element group
// (c * 256 + tid) of every 1024-float chunk c.  The same slice meets every
// weight row, so it stays in registers for the whole stage (no LDS staging).
template <int KCH>
__device__ __forceinline__ void load_x_slice(const float *x, int K, float4 (&xr)[KCH])
{
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
        int k = c * kChunk + threadIdx.x * 4;
        xr[c] = (k < K) ? *reinterpret_cast<const float4 *>(x + k) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// Streams the weight rows of a sequence of units through registers, two
// batches deep: while batch s is multiplied, batch s+1 (possibly the next
// unit's first) is already in flight, so the memory pipe does not drain at a
// unit's reduction.  A unit is ROWS rows of length K (K % 4 == 0, rows
// 16-byte aligned); a batch is UB chunks of 1024 floats of each row.
//
//   RowFn(unit, const float *(&rows)[ROWS])  sets the unit's row pointers
//   EpiFn(unit, float (&y)[ROWS])            consumes the unit's ROWS sums
//                                            (every thread holds all of them)
// Units first, first + stride, ... < n_units are processed.  prefetch() may be
// called before the input slice exists; run() needs it.  red: ROWS * 4 floats.
template <int ROWS, int KCH, int UB>
struct RowStreamer {
    static constexpr int NB = (KCH + UB - 1) / UB;   // batches per unit
    float4 wa[UB][ROWS], wb[UB][ROWS];
    int unit, stride, n_units, K;

    template <class RowFn>
    __device__ __forceinline__ void issue(float4 (&w)[UB][ROWS], int u, int b, RowFn &rowfn)
    {
        const float *rows[ROWS];
        rowfn(u, rows);
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            int k = (b * UB + i) * kChunk + threadIdx.x * 4;
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                w[i][r] = (k < K) ? load_stream4(rows[r] + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }

    __device__ __forceinline__ void consume(const float4 (&w)[UB][ROWS], int b, const float4 (&xr)[KCH],
                                            float (&acc)[ROWS])
    {
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            // b is a run-time value: pick the slice with a compile-time index per batch
#pragma unroll
            for (int bb = 0; bb < NB; ++bb) {
                if (bb == b && bb * UB + i < KCH) {
#pragma unroll
                    for (int r = 0; r < ROWS; ++r) acc[r] = dot4(w[i][r], xr[bb * UB + i], acc[r]);
                }
            }
        }
    }

    template <class RowFn>
    __device__ __forceinline__ void prefetch(int first, int stride_, int n_units_, int K_, RowFn &rowfn)
    {
        unit = first; stride = stride_; n_units = n_units_; K = K_;
        if (unit < n_units) issue(wa, unit, 0, rowfn);
    }

    template <class EpiFn>
    __device__ __forceinline__ void finish_unit(int u, float (&acc)[ROWS], float *red, EpiFn &epi)
    {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) acc[r] = wave_sum(acc[r]);
        if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
            for (int r = 0; r < ROWS; ++r) red[r * kWavesPerBlock + threadIdx.x / kWave] = acc[r];
        }
        __syncthreads();
        float y[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) s += red[r * kWavesPerBlock + w];
            y[r] = s;
            acc[r] = 0.f;
        }
        __syncthreads();
        epi(u, y);
    }

    template <class RowFn, class EpiFn>
    __device__ __forceinline__ void run(const float4 (&xr)[KCH], float *red, RowFn &rowfn, EpiFn &epi)
    {
        float acc[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
        int u = unit, b = 0;
        if (u >= n_units) return;
        while (true) {
            // current step sits in wa
            int nu = u, nb = b + 1;
            if (nb == NB) { nb = 0; nu = u + stride; }
            bool more = nu < n_units;
            if (more) issue(wb, nu, nb, rowfn);
            consume(wa, b, xr, acc);
            if (b == NB - 1) finish_unit(u, acc, red, epi);
            if (!more) break;
            u = nu; b = nb;
            // current step sits in wb
            nu = u; nb = b + 1;
            if (nb == NB) { nb = 0; nu = u + stride; }
            more = nu < n_units;
            if (more) issue(wa, nu, nb, rowfn);
            consume(wb, b, xr, acc);
            if (b == NB - 1) finish_unit(u, acc, red, epi);
            if (!more) break;
            u = nu; b = nb;
        }
    }

    // The same walk for units whose input vectors differ: XFn(unit, float4 (&x)[KCH]) loads the unit's slice.
    // The next unit's slice is requested right behind that unit's first weight batch, a whole unit before it
    // is multiplied.
    template <class XFn, class RowFn, class EpiFn>
    __device__ __forceinline__ void run_x(XFn &xfn, float *red, RowFn &rowfn, EpiFn &epi)
    {
        float acc[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
        int u = unit, b = 0;
        if (u >= n_units) return;
        float4 xc[KCH], xn[KCH];
        xfn(u, xc);
#pragma unroll
        for (int c = 0; c < KCH; ++c) xn[c] = xc[c];
        while (true) {
            // current step sits in wa
            int nu = u, nb = b + 1;
            if (nb == NB) { nb = 0; nu = u + stride; }
            bool more = nu < n_units;
            if (more) {
                issue(wb, nu, nb, rowfn);
                if (nb == 0) xfn(nu, xn);
            }
            consume(wa, b, xc, acc);
            if (b == NB - 1) {
                finish_unit(u, acc, red, epi);
#pragma unroll
                for (int c = 0; c < KCH; ++c) xc[c] = xn[c];
            }
            if (!more) break;
            u = nu; b = nb;
            // current step sits in wb
            nu = u; nb = b + 1;
            if (nb == NB) { nb = 0; nu = u + stride; }
            more = nu < n_units;
            if (more) {
                issue(wa, nu, nb, rowfn);
                if (nb == 0) xfn(nu, xn);
            }
            consume(wb, b, xc, acc);
            if (b == NB - 1) {
                finish_unit(u, acc, red, epi);
#pragma unroll
                for (int c = 0; c < KCH; ++c) xc[c] = xn[c];
            }
            if (!more) break;
            u = nu; b = nb;
        }
    }
};

}  // namespace tpi
