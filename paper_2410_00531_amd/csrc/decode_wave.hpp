// Wave-autonomous GEMV stages for the whole-token persistent kernel.
//
// The persistent kernel runs one wave per SIMD (it must stay co-resident), so
// nothing hides a wave's stalls but its own loads in flight.  Each wave
// therefore streams whole weight rows on its own -- the stage's input vector
// sits in LDS (written once per workgroup), reductions go by DPP and readlane,
// no workgroup barrier inside a stage -- and keeps two batches of 16 float4
// per lane in flight, 128 KB per compute unit.  prefetch() issues the first two batches of a
// stage; it is called BEFORE the grid barrier that precedes the stage, because
// weights never depend on activations: the barrier's latency and the previous
// stage's tail are covered by the next stage's weight traffic.
#pragma once
#include "decode_args.hpp"
#include "decode_stages.hpp"

namespace tpi {

constexpr int kWChunk = kWave * 4;       // floats one wave covers with one float4 per lane

// sum over the wave, result uniform
__device__ __forceinline__ float wave_sum_dpp(float x)
{
    x = row16_sum(x);
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

// The stage's input vector goes to LDS once per workgroup (all 256 threads), where the four
// waves read it while they stream rows on their own.  Both contain a workgroup barrier.
__device__ __forceinline__ void stage_x_plain(const float *x, int n, float *xs)
{
    for (int k = threadIdx.x * 4; k < n; k += kBlock * 4)
        *reinterpret_cast<float4 *>(xs + k) = *reinterpret_cast<const float4 *>(x + k);
    __syncthreads();
}

// xs <- x * g; returns 1/sqrt(mean(x^2) + eps).  red: 4 floats of LDS.
__device__ __forceinline__ float stage_x_norm(const float *x, const float *g, int h, float eps, float *xs, float *red)
{
    float ss = 0.f;
    for (int k = threadIdx.x * 4; k < h; k += kBlock * 4) {
        float4 v = *reinterpret_cast<const float4 *>(x + k);
        float4 w = *reinterpret_cast<const float4 *>(g + k);
        ss = dot4(v, v, ss);
        *reinterpret_cast<float4 *>(xs + k) = make_float4(v.x * w.x, v.y * w.y, v.z * w.z, v.w * w.w);
    }
    ss = block_sum(ss, red);          // two barriers: xs is visible afterwards
    return 1.0f / sqrtf(ss / (float)h + eps);
}

// A unit is ROWS rows of length K; a batch is CB chunks (of 256 floats) of each row, ROWS * CB
// float4 per lane; two batches are in flight.  Units first, first + stride, ... < n_units.
template <int ROWS, int CB>
struct WaveStreamer {
    float4 wa[CB][ROWS], wb[CB][ROWS];
    int first, stride, n_steps, K, nb;   // nb: batches per unit

    template <class RowFn>
    __device__ __forceinline__ void issue(float4 (&w)[CB][ROWS], int s, RowFn &rowfn)
    {
        const int lane = threadIdx.x & (kWave - 1);
        const int uu = s / nb, b = s - uu * nb;
        const float *rows[ROWS];
        rowfn(first + uu * stride, rows);
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            int k = (b * CB + i) * kWChunk + lane * 4;
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                w[i][r] = (k < K) ? load_stream4(rows[r] + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }

    __device__ __forceinline__ void consume(const float4 (&w)[CB][ROWS], int b, const float *xs, float (&acc)[ROWS])
    {
        const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            int k = (b * CB + i) * kWChunk + lane * 4;
            if (k < K) {
                float4 x4 = *reinterpret_cast<const float4 *>(xs + k);
#pragma unroll
                for (int r = 0; r < ROWS; ++r) acc[r] = dot4(w[i][r], x4, acc[r]);
            }
        }
    }

    __device__ __forceinline__ void clear(float4 (&w)[CB][ROWS])
    {
#pragma unroll
        for (int i = 0; i < CB; ++i)
#pragma unroll
            for (int r = 0; r < ROWS; ++r) w[i][r] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // first_ / stride_ count waves
    template <class RowFn>
    __device__ __forceinline__ void prefetch(int first_, int stride_, int n_units, int K_, RowFn &rowfn)
    {
        first = first_; stride = stride_; K = K_;
        nb = (K + CB * kWChunk - 1) / (CB * kWChunk);
        int mine = (first < n_units) ? (n_units - first + stride - 1) / stride : 0;
        n_steps = mine * nb;
        // both buffers are always defined here, so no stale value is carried into the stage
        if (n_steps > 0) issue(wa, 0, rowfn); else clear(wa);
        if (n_steps > 1) issue(wb, 1, rowfn); else clear(wb);
    }

    template <class EpiFn>
    __device__ __forceinline__ void step_done(int s, float (&acc)[ROWS], EpiFn &epi)
    {
        const int uu = s / nb;
        if (s - uu * nb != nb - 1) return;
        float y[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            y[r] = wave_sum_dpp(acc[r]);
            acc[r] = 0.f;
        }
        epi(first + uu * stride, y);
    }

    template <class RowFn, class EpiFn>
    __device__ __forceinline__ void run(const float *xs, RowFn &rowfn, EpiFn &epi)
    {
        float acc[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
        for (int s = 0; s < n_steps; s += 2) {
            consume(wa, s % nb, xs, acc);
            if (s + 2 < n_steps) issue(wa, s + 2, rowfn);
            step_done(s, acc, epi);
            if (s + 1 < n_steps) {
                consume(wb, (s + 1) % nb, xs, acc);
                if (s + 3 < n_steps) issue(wb, s + 3, rowfn);
                step_done(s + 1, acc, epi);
            }
        }
    }
};

// Row functors (plain structs: they live across a grid barrier between prefetch and run).
template <int PAIRS>
struct QkvRows {
    const float *w; int d, h, half, npairs;
    __device__ __forceinline__ void operator()(int u, const float *(&rows)[2 * PAIRS]) const
    {
#pragma unroll
        for (int i = 0; i < PAIRS; ++i) {
            int p = min(u * PAIRS + i, npairs - 1);
            int hd = p / half, e = p - hd * half;
            rows[2 * i] = w + ((size_t)hd * d + e) * h;
            rows[2 * i + 1] = rows[2 * i] + (size_t)half * h;
        }
    }
};

template <int ROWS>
struct PlainRows {
    const float *w; int n_rows, K;
    __device__ __forceinline__ void operator()(int u, const float *(&rows)[ROWS]) const
    {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) rows[r] = w + (size_t)min(u * ROWS + r, n_rows - 1) * K;
    }
};

template <int COLS>
struct GateUpRows {
    const float *wg, *wu; int sl, h;
    __device__ __forceinline__ void operator()(int u, const float *(&rows)[2 * COLS]) const
    {
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            size_t j = (size_t)min(u * COLS + c, sl - 1);
            rows[2 * c] = wg + j * h;
            rows[2 * c + 1] = wu + j * h;
        }
    }
};

}  // namespace tpi
