// Device-side building blocks shared by the decode kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tpi {

constexpr int kWave = 64;
constexpr int kBlock = 256;              // threads per workgroup of every streaming kernel
constexpr int kWavesPerBlock = kBlock / kWave;

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

// y[r] = sum_k rows[r][k] * xs[k] for ROWS rows of length K (K % 4 == 0, rows
// 16-byte aligned), the 256 threads of the workgroup striding over k.  xs is
// in LDS.  pre holds the loads of the first batch, issued by the caller
// before xs was ready (weights do not depend on activations).  On return
// every thread holds all ROWS sums.  red: ROWS * kWavesPerBlock floats of LDS.
template <int ROWS, int U>
struct GemvTile {
    float4 w[U][ROWS];

    __device__ __forceinline__ void issue(const float *const (&rows)[ROWS], int K, int k0)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int k = k0 + (u * kBlock + threadIdx.x) * 4;
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                w[u][r] = (k < K) ? load_stream4(rows[r] + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }

    __device__ __forceinline__ void consume(const float *xs, int K, int k0, float (&acc)[ROWS])
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int k = k0 + (u * kBlock + threadIdx.x) * 4;
            if (k < K) {
                float4 x = *reinterpret_cast<const float4 *>(xs + k);
#pragma unroll
                for (int r = 0; r < ROWS; ++r) acc[r] = dot4(w[u][r], x, acc[r]);
            }
        }
    }
};

template <int ROWS, int U>
__device__ __forceinline__ void gemv_rows(const float *const (&rows)[ROWS], int K, const float *xs,
                                          GemvTile<ROWS, U> &tile, float *red, float (&y)[ROWS])
{
    constexpr int kStep = U * kBlock * 4;
    float acc[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = 0.f;
    for (int k0 = 0;;) {
        tile.consume(xs, K, k0, acc);
        k0 += kStep;
        if (k0 >= K) break;
        tile.issue(rows, K, k0);
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = wave_sum(acc[r]);
    if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) red[r * kWavesPerBlock + threadIdx.x / kWave] = acc[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) s += red[r * kWavesPerBlock + w];
        y[r] = s;
    }
    __syncthreads();
}

}  // namespace tpi
