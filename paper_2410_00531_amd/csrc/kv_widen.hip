// The KV cache is one object across prefill and decode (Sec. 3.1; Alg. 1 stores (K, V) for every token it has
// seen).  The prefill entry points fill a bf16 cache, the decode entry points read an fp32 one: this kernel carries
// the first n_slots slots of a layer's bf16 cache over into an fp32 cache (every bf16 value is an fp32 value, so
// the copy is exact).
#include <hip/hip_runtime.h>

#include "../../include/tpi.h"
#include "host_util.hpp"

using tpi::fail;

namespace {

__global__ __launch_bounds__(256) void k_kv_widen(const unsigned short *__restrict__ ks, const unsigned short *__restrict__ vs,
                                                  float *__restrict__ kd, float *__restrict__ vd, int n_slots, int d,
                                                  int src_seq, int dst_seq)
{
    // grid.y: KV head; one thread per pair of elements
    const int g = blockIdx.y;
    const size_t per_head = (size_t)n_slots * d / 2;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < per_head; i += (size_t)gridDim.x * blockDim.x) {
        const size_t e = 2 * i, slot = e / d, col = e - slot * d;
        const size_t so = ((size_t)g * src_seq + slot) * d + col, dof = ((size_t)g * dst_seq + slot) * d + col;
        const unsigned kk = *reinterpret_cast<const unsigned *>(ks + so), vv = *reinterpret_cast<const unsigned *>(vs + so);
        *reinterpret_cast<float2 *>(kd + dof) = make_float2(__uint_as_float(kk << 16), __uint_as_float(kk & 0xffff0000u));
        *reinterpret_cast<float2 *>(vd + dof) = make_float2(__uint_as_float(vv << 16), __uint_as_float(vv & 0xffff0000u));
    }
}

}  // namespace

extern "C" int tpi_kv_widen(int32_t n_kv_local, int32_t head_dim, int32_t n_slots, const tpi_kv_layer *host_src_bf16,
                            int32_t src_max_seq, const tpi_kv_layer *host_dst_f32, int32_t dst_max_seq, void *stream)
{
    if (!host_src_bf16 || !host_dst_f32 || !host_src_bf16->k || !host_src_bf16->v || !host_dst_f32->k || !host_dst_f32->v)
        return fail(TPI_EINVAL, "null argument");
    if (n_kv_local < 1 || head_dim < 2 || head_dim % 2 || src_max_seq < 1 || dst_max_seq < 1)
        return fail(TPI_EINVAL, "sizes must be positive and head_dim even");
    if (n_slots < 0 || n_slots > src_max_seq || n_slots > dst_max_seq)
        return fail(TPI_EINVAL, "n_slots %d outside the caches (%d and %d slots)", n_slots, src_max_seq, dst_max_seq);
    if (n_kv_local > 65535) return fail(TPI_EUNSUPPORTED, "n_kv_local %d: more heads than the grid can index", n_kv_local);
    auto al = [](const void *p, unsigned a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; };
    if (!al(host_src_bf16->k, 4) || !al(host_src_bf16->v, 4) || !al(host_dst_f32->k, 8) || !al(host_dst_f32->v, 8))
        return fail(TPI_EUNSUPPORTED, "cache pointers must be 4-byte (bf16) and 8-byte (fp32) aligned");
    if (n_slots == 0) return TPI_OK;
    const size_t per_head = (size_t)n_slots * head_dim / 2;
    const unsigned gx = (unsigned)((per_head + 255) / 256 > 4096 ? 4096 : (per_head + 255) / 256);
    hipLaunchKernelGGL(k_kv_widen, dim3(gx, n_kv_local), dim3(256), 0, (hipStream_t)stream,
                       (const unsigned short *)host_src_bf16->k, (const unsigned short *)host_src_bf16->v,
                       (float *)host_dst_f32->k, (float *)host_dst_f32->v, n_slots, head_dim, src_max_seq, dst_max_seq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}
