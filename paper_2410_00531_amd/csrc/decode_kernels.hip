// Batch-1 decode of one shard's decoder layer on gfx950 (fp32, HBM-bound).
//
// Five streaming stages, one kernel each; a grid dimension selects the
// emulated shard.
//   ATTN phase: k_qkv_rope   RMSNorm + column-parallel QKV GEMV + rotary + cache append
//               k_attn       GQA attention over the cache, split along the KV length,
//                            merged by the last split to finish
//   (cont.)     k_oproj      row-parallel output projection
//   FFN phase:  k_gate_up    RMSNorm + gate/up GEMV + SiLU gate
//               k_down       row-parallel down projection
// Every GEMV streams its weight rows once with 16-byte non-temporal loads, 256
// threads striding along the row.  A thread meets the same slice of the input
// vector in every row, so the slice lives in registers (no LDS staging), and
// the rows pass through a two-deep register pipeline (RowStreamer) whose first
// batch is issued before the input vector is touched: weights never depend on
// activations.
#include <algorithm>

#include "decode_args.hpp"
#include "decode_stages.hpp"
#include "prof.hpp"

namespace tpi {

// ---------------------------------------------------------------------------
// One kernel per stage (the per-phase entry points)
// ---------------------------------------------------------------------------
template <int PAIRS, int KCH, int UB>
__global__ __launch_bounds__(kBlock) void k_qkv_rope(DecodeArgs a)
{
    __shared__ float red[2 * PAIRS * kWavesPerBlock + kWavesPerBlock];
    __shared__ float rope[2 * kRopeHalf];
    stage_qkv<PAIRS, KCH, UB>(a, a.s[blockIdx.y], blockIdx.x, gridDim.x, red, rope);
}

template <int GT, int EPL>
__global__ __launch_bounds__(kBlock) void k_attn(DecodeArgs a)
{
    extern __shared__ float smem[];
    const int G = a.nq / a.nkv;
    const int n_ht = (G + GT - 1) / GT;
    const int g = blockIdx.y / n_ht, ht = blockIdx.y - g * n_ht;
    stage_attn<GT, EPL>(a, a.s[blockIdx.z], blockIdx.x, g, ht, smem);
}

// FOLD: 0 plain; 8 / 16: the star reduce folded in, with that many rank slots compiled in
template <int ROWS, int KCH, int UB, int FOLD>
__global__ __launch_bounds__(kBlock) void k_oproj(DecodeArgs a)
{
    __shared__ float red[ROWS * kWavesPerBlock];
    stage_oproj<ROWS, KCH, UB, (FOLD > 0), (FOLD > 0 ? FOLD : 8)>(a, a.s[blockIdx.y], blockIdx.x, gridDim.x, red, a.rf);
}

template <int COLS, int KCH, int UB>
__global__ __launch_bounds__(kBlock) void k_gate_up(DecodeArgs a)
{
    __shared__ float red[2 * COLS * kWavesPerBlock + kWavesPerBlock];
    stage_gate_up<COLS, KCH, UB>(a, a.s[blockIdx.y], blockIdx.x, gridDim.x, red);
}

template <int ROWS, int KCH, int UB, int FOLD>
__global__ __launch_bounds__(kBlock) void k_down(DecodeArgs a)
{
    __shared__ float red[ROWS * kWavesPerBlock];
    stage_down<ROWS, KCH, UB, (FOLD > 0), (FOLD > 0 ? FOLD : 8)>(a, a.s[blockIdx.y], blockIdx.x, gridDim.x, red, a.rf);
}

// all shards of a batched call, the star reduce folded in: workgroup = ROWS rows of the output, all ranks
template <int ROWS, int KCH, int UB, bool DOWN>
__global__ __launch_bounds__(kBlock) void k_rowpar_all(DecodeArgs a, int n_shards)
{
    __shared__ float red[ROWS * kWavesPerBlock];
    stage_rowpar_all<ROWS, KCH, UB, DOWN>(a, n_shards, blockIdx.x, red);
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// chunks of 1024 floats a row of length K spans, rounded up to a power of two (the template choices)
static inline int kch_of(int K)
{
    int c = cdiv(K, kChunk), p = 1;
    while (p < c) p *= 2;
    return p;
}

constexpr int kMaxWgPerShard = 1024;   // workgroups one shard's stage is dealt to (4 per CU)

// Workgroups for n_units units: at most kMaxWgPerShard, and every workgroup gets the same number
// of units (up to one), so the stage does not end with half the grid idle.
static inline int balanced_grid(int n_units)
{
    int per = cdiv(n_units, kMaxWgPerShard);
    return cdiv(n_units, per);
}

#define TPI_KCH_SWITCH(K, ...)                                      \
    switch (kch_of(K)) {                                            \
    case 1: { constexpr int KCH = 1, UB = 1, WIDE = 1; __VA_ARGS__; } break;  \
    case 2: { constexpr int KCH = 2, UB = 2, WIDE = 0; __VA_ARGS__; } break;  \
    case 4: { constexpr int KCH = 4, UB = 2, WIDE = 0; __VA_ARGS__; } break;  \
    case 8: { constexpr int KCH = 8, UB = 2, WIDE = 0; __VA_ARGS__; } break;  \
    case 16: { constexpr int KCH = 16, UB = 2, WIDE = 0; __VA_ARGS__; } break; \
    default: return hipErrorInvalidValue;                           \
    }

template <int GT>
static hipError_t launch_attn_gt(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    const int G = a.nq / a.nkv;
    const int n_ht = cdiv(G, GT);
    dim3 grid(a.n_splits, a.nkv * n_ht, n_shards);
    const int epl = a.d <= 64 ? 1 : (a.d <= 128 ? 2 : 4);
    size_t lds = sizeof(float) * ((size_t)kWavesPerBlock * GT * a.d + 2 * kWavesPerBlock * GT);
    switch (epl) {
    case 1: hipLaunchKernelGGL((k_attn<GT, 1>), grid, dim3(kBlock), lds, st, a); break;
    case 2: hipLaunchKernelGGL((k_attn<GT, 2>), grid, dim3(kBlock), lds, st, a); break;
    default: hipLaunchKernelGGL((k_attn<GT, 4>), grid, dim3(kBlock), lds, st, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_attn_phase(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    {
        const int npairs = (a.nq + 2 * a.nkv) * (a.d / 2);
        ProfScope ps(kStageQkv, st);
        // One rotary pair per unit keeps a single shard's grid large enough to balance over the chip; with
        // several shards per launch there are workgroups to spare, and two pairs per unit halve the
        // per-workgroup prologue (input slice, norm, rotary table).
        const bool fat = (long)npairs * n_shards >= 4096;
        TPI_KCH_SWITCH(a.h, {
            if (WIDE) {
                int gx = balanced_grid(cdiv(npairs, 4));
                hipLaunchKernelGGL((k_qkv_rope<4, KCH, UB>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            } else if (fat) {
                int gx = balanced_grid(cdiv(npairs, 2));
                hipLaunchKernelGGL((k_qkv_rope<2, KCH, UB>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            } else {
                int gx = balanced_grid(cdiv(npairs, 1));
                hipLaunchKernelGGL((k_qkv_rope<1, KCH, UB>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            }
        })
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope ps(kStageAttn, st);
        const int G = a.nq / a.nkv;
        hipError_t e = (G == 1)   ? launch_attn_gt<1>(a, n_shards, st)
                       : (G == 2) ? launch_attn_gt<2>(a, n_shards, st)
                       : (G <= 4) ? launch_attn_gt<4>(a, n_shards, st)
                                  : launch_attn_gt<8>(a, n_shards, st);
        if (e != hipSuccess) return e;
    }
    {
        ProfScope ps(kStageOproj, st);
        if (a.rf.all) {
            TPI_KCH_SWITCH(a.nq * a.d, {
                constexpr int ROWS = WIDE ? 8 : 4;
                hipLaunchKernelGGL((k_rowpar_all<ROWS, KCH, UB, false>), dim3(cdiv(a.h, ROWS)), dim3(kBlock), 0, st, a, n_shards);
            })
            return hipGetLastError();
        }
        TPI_KCH_SWITCH(a.nq * a.d, {
            constexpr int ROWS = WIDE ? 8 : 4;
            int gx = std::max(balanced_grid(cdiv(a.h, ROWS)), cdiv(a.h, kBlock));   // <= 256 rows per workgroup
            if (a.rf.n > 8) hipLaunchKernelGGL((k_oproj<ROWS, KCH, UB, 16>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            else if (a.rf.n > 0) hipLaunchKernelGGL((k_oproj<ROWS, KCH, UB, 8>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            else hipLaunchKernelGGL((k_oproj<ROWS, KCH, UB, 0>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
        })
        return hipGetLastError();
    }
}

hipError_t launch_ffn_phase(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    {
        ProfScope ps(kStageGateUp, st);
        TPI_KCH_SWITCH(a.h, {
            constexpr int COLS = WIDE ? 4 : 2;
            int gx = balanced_grid(cdiv(a.sl, COLS));
            hipLaunchKernelGGL((k_gate_up<COLS, KCH, UB>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
        })
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope ps(kStageDown, st);
        if (a.rf.all) {
            TPI_KCH_SWITCH(a.sl, {
                constexpr int ROWS = WIDE ? 8 : 4;
                hipLaunchKernelGGL((k_rowpar_all<ROWS, KCH, UB, true>), dim3(cdiv(a.h, ROWS)), dim3(kBlock), 0, st, a, n_shards);
            })
            return hipGetLastError();
        }
        TPI_KCH_SWITCH(a.sl, {
            constexpr int ROWS = WIDE ? 8 : 4;
            int gx = std::max(balanced_grid(cdiv(a.h, ROWS)), cdiv(a.h, kBlock));   // <= 256 rows per workgroup
            if (a.rf.n > 8) hipLaunchKernelGGL((k_down<ROWS, KCH, UB, 16>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            else if (a.rf.n > 0) hipLaunchKernelGGL((k_down<ROWS, KCH, UB, 8>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
            else hipLaunchKernelGGL((k_down<ROWS, KCH, UB, 0>), dim3(gx, n_shards), dim3(kBlock), 0, st, a);
        })
        return hipGetLastError();
    }
}

}  // namespace tpi
