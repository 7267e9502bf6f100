// Star all-reduce sum on one GPU: the master's aggregation step, in rank order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "prof.hpp"
#include "star_reduce.hpp"

namespace tpi {

// out[i] = (((p0[i] + p1[i]) + ...) + p_{n-1}[i]) + residual[i]; plain fp32
// additions in exactly this order (contraction off: there is nothing to fuse,
// and nothing may be reassociated).
__device__ __forceinline__ unsigned short to_bf16(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

#pragma clang fp contract(off)
__global__ __launch_bounds__(256) void k_star_reduce(ReduceArgs a)
{
    const int64_t n4 = a.vec_ok ? a.len / 4 : 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 acc = reinterpret_cast<const float4 *>(a.p[0])[i];
        for (int r = 1; r < a.n; ++r) {
            float4 v = reinterpret_cast<const float4 *>(a.p[r])[i];
            acc.x = acc.x + v.x; acc.y = acc.y + v.y; acc.z = acc.z + v.z; acc.w = acc.w + v.w;
        }
        if (a.residual) {
            float4 v = reinterpret_cast<const float4 *>(a.residual)[i];
            acc.x = acc.x + v.x; acc.y = acc.y + v.y; acc.z = acc.z + v.z; acc.w = acc.w + v.w;
        }
        reinterpret_cast<float4 *>(a.out)[i] = acc;
        if (a.out_bf16) {
            ushort4 b = make_ushort4(to_bf16(acc.x), to_bf16(acc.y), to_bf16(acc.z), to_bf16(acc.w));
            reinterpret_cast<ushort4 *>(a.out_bf16)[i] = b;
        }
    }
    // ragged tail (len % 4 elements), or everything when a pointer is not 16-byte aligned
    for (int64_t t = n4 * 4 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < a.len; t += stride) {
        float acc = a.p[0][t];
        for (int r = 1; r < a.n; ++r) acc = acc + a.p[r][t];
        if (a.residual) acc = acc + a.residual[t];
        a.out[t] = acc;
        if (a.out_bf16) a.out_bf16[t] = to_bf16(acc);
    }
}

hipError_t launch_star_reduce(const ReduceArgs &a, hipStream_t st)
{
    if (a.len == 0) return hipSuccess;
    int64_t work = a.vec_ok ? (a.len + 3) / 4 : a.len;
    int64_t blocks = (work + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    ProfScope ps(kStageReduce, st);
    hipLaunchKernelGGL(k_star_reduce, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace tpi
