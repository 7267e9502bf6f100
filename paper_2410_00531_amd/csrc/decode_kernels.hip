// Batch-1 decode of one shard's decoder layer on gfx950 (fp32, HBM-bound).
//
// Five streaming stages, one kernel each; the workgroup index along y selects
// the emulated shard.
//   ATTN phase: k_qkv_rope   RMSNorm + column-parallel QKV GEMV + rotary + cache append
//               k_attn_split GQA attention over the cache, split along the KV length
//               k_oproj      merge of the splits + row-parallel output projection
//   FFN phase:  k_gate_up    RMSNorm + gate/up GEMV + SiLU gate
//               k_down       row-parallel down projection
// Every GEMV streams its weight rows once with 16-byte non-temporal loads,
// 256 threads striding along the row, the activation vector staged in LDS.
// The first batch of weight loads is issued before the activation vector is
// touched: weights never depend on activations, so their latency overlaps the
// prologue (norm, merge) of the stage.
#include "decode_args.hpp"
#include "prof.hpp"
#include "tpi_device.hpp"

namespace tpi {

// ---------------------------------------------------------------------------
// Prologues that fill xs (LDS) with the stage's input vector
// ---------------------------------------------------------------------------

// xs[k] = x[k] * g[k]; returns 1/sqrt(mean(x^2) + eps).  The normalisation
// factor is applied to the row sums afterwards (it is a scalar).
__device__ __forceinline__ float stage_norm_input(const float *x, const float *g, int h, float eps,
                                                  float *xs, float *red)
{
    float ss = 0.f;
    for (int k = threadIdx.x * 4; k < h; k += kBlock * 4) {
        float4 v = *reinterpret_cast<const float4 *>(x + k);
        float4 w = *reinterpret_cast<const float4 *>(g + k);
        ss = dot4(v, v, ss);
        *reinterpret_cast<float4 *>(xs + k) = make_float4(v.x * w.x, v.y * w.y, v.z * w.z, v.w * w.w);
    }
    ss = block_sum(ss, red);
    return 1.0f / sqrtf(ss / (float)h + eps);
}

__device__ __forceinline__ void stage_copy_input(const float *x, int n, float *xs)
{
    for (int k = threadIdx.x * 4; k < n; k += kBlock * 4)
        *reinterpret_cast<float4 *>(xs + k) = *reinterpret_cast<const float4 *>(x + k);
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Stage 1: RMSNorm + QKV GEMV + rotary embedding + KV-cache append
// ---------------------------------------------------------------------------
// A workgroup owns PAIRS row pairs (i, i + d/2) of one head, so the rotation
// of a pair happens in registers.  V rows use the same pairing, unrotated.
template <int PAIRS, int U>
__global__ __launch_bounds__(kBlock) void k_qkv_rope(DecodeArgs a)
{
    extern __shared__ float smem[];
    float *xs = smem;
    float *red = smem + a.h;
    const ShardView &s = a.s[blockIdx.y];
    const int tid = threadIdx.x;
    const int half = a.d / 2;
    const int npairs = (a.nq + 2 * a.nkv) * half;
    constexpr int ROWS = 2 * PAIRS;

    const float *rows[ROWS];
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
        int p = min((int)blockIdx.x * PAIRS + i, npairs - 1);
        int hd = p / half, e = p - hd * half;
        rows[2 * i] = s.w_qkv + ((size_t)hd * a.d + e) * a.h;
        rows[2 * i + 1] = rows[2 * i] + (size_t)half * a.h;
    }
    GemvTile<ROWS, U> tile;
    tile.issue(rows, a.h, 0);

    // rotation of the pair this thread will finalise, in fp64 (angles reach
    // pos radians; fp32 would lose the low bits of the phase)
    float cs = 1.f, sn = 0.f;
    int my_hd = -1, my_e = 0;
    if (tid < PAIRS) {
        int p = blockIdx.x * PAIRS + tid;
        if (p < npairs) {
            my_hd = p / half;
            my_e = p - my_hd * half;
            if (my_hd < a.nq + a.nkv && a.pos != 0) {
                double theta = exp2(-(2.0 * (double)my_e / (double)a.d) * a.log2_base);
                double sd, cd;
                sincos((double)a.pos * theta, &sd, &cd);
                cs = (float)cd;
                sn = (float)sd;
            }
        }
    }

    const float rinv = stage_norm_input(a.h_in, s.attn_norm, a.h, a.eps, xs, red);
    float y[ROWS];
    gemv_rows<ROWS, U>(rows, a.h, xs, tile, red, y);

#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
        if (tid == i && my_hd >= 0) {
            float lo = y[2 * i] * rinv, hi = y[2 * i + 1] * rinv;
            float *dst;
            if (my_hd < a.nq) {
                dst = s.ws + a.ws_q + (size_t)my_hd * a.d;
            } else if (my_hd < a.nq + a.nkv) {
                dst = s.k + ((size_t)(my_hd - a.nq) * a.max_seq + a.pos) * a.d;
            } else {
                dst = s.v + ((size_t)(my_hd - a.nq - a.nkv) * a.max_seq + a.pos) * a.d;
            }
            dst[my_e] = lo * cs - hi * sn;
            dst[my_e + half] = hi * cs + lo * sn;
        }
    }
}

// ---------------------------------------------------------------------------
// Stage 2: attention of the local heads over cache slots 0..pos
// ---------------------------------------------------------------------------
// grid.x = split of the KV length, grid.y = (KV head, tile of its query heads),
// grid.z = shard.  All GT query heads of a group share each K/V row load.
// LPR lanes cover one cache row (4 floats per lane), so a wave loads 64/LPR
// rows at once; a tile is 64 slots, 16 per wave.  Each split leaves
// (max, sum, unnormalised output) for the merge in stage 3.
template <int GT, int LPR>
__global__ __launch_bounds__(kBlock) void k_attn_split(DecodeArgs a)
{
    constexpr int RPW = kWave / LPR;        // rows per wave-load
    constexpr int TILE = 64;
    constexpr int ROWS_PER_WAVE = TILE / kWavesPerBlock;   // 16
    constexpr int ITERS = ROWS_PER_WAVE / RPW;

    extern __shared__ float smem[];
    float *sc = smem;                       // [GT][TILE] scores, then probabilities
    float *alpha = sc + GT * TILE;          // [8] (GT used)
    float *m_run = alpha + 8;               // [8]
    float *l_run = m_run + 8;               // [8]
    float *wacc = l_run + 8;                // [waves][GT][LPR*4], 16-byte aligned

    const ShardView &s = a.s[blockIdx.z];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int sub = lane % LPR, rsel = lane / LPR;
    const int G = a.nq / a.nkv;
    const int n_ht = (G + GT - 1) / GT;
    const int g = blockIdx.y / n_ht, ht = blockIdx.y - g * n_ht;
    const int split = blockIdx.x;
    const int n_valid = a.pos + 1;
    const int t_begin = split * a.chunk_len;
    const int t_end = min(t_begin + a.chunk_len, n_valid);
    const bool col_ok = sub * 4 < a.d;
    const float scale = 1.0f / sqrtf((float)a.d);

    const float *Kg = s.k + (size_t)g * a.max_seq * a.d;
    const float *Vg = s.v + (size_t)g * a.max_seq * a.d;

    float4 q[GT];
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        int hj = min(ht * GT + j, G - 1);
        const float *qp = s.ws + a.ws_q + (size_t)(g * G + hj) * a.d;
        q[j] = col_ok ? *reinterpret_cast<const float4 *>(qp + sub * 4) : make_float4(0, 0, 0, 0);
        q[j].x *= scale; q[j].y *= scale; q[j].z *= scale; q[j].w *= scale;
    }
    float4 acc[GT];
#pragma unroll
    for (int j = 0; j < GT; ++j) acc[j] = make_float4(0, 0, 0, 0);
    if (tid < GT) { m_run[tid] = -INFINITY; l_run[tid] = 0.f; }
    __syncthreads();

    for (int t0 = t_begin; t0 < t_end; t0 += TILE) {
        float4 kk[ITERS], vv[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int t = t0 + wave * ROWS_PER_WAVE + it * RPW + rsel;
            bool ok = (t < t_end) && col_ok;
            kk[it] = ok ? *reinterpret_cast<const float4 *>(Kg + (size_t)t * a.d + sub * 4) : make_float4(0, 0, 0, 0);
            vv[it] = ok ? *reinterpret_cast<const float4 *>(Vg + (size_t)t * a.d + sub * 4) : make_float4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int tl = wave * ROWS_PER_WAVE + it * RPW + rsel;
            bool ok = (t0 + tl) < t_end;
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                float p = dot4(q[j], kk[it], 0.f);
#pragma unroll
                for (int o = LPR / 2; o > 0; o >>= 1) p += __shfl_xor(p, o, kWave);
                if (sub == 0) sc[j * TILE + tl] = ok ? p : -INFINITY;
            }
        }
        __syncthreads();
        // running softmax statistics, one wave per head, one lane per slot
        for (int j = wave; j < GT; j += kWavesPerBlock) {
            float sv = sc[j * TILE + lane];
            float mt = wave_max(sv);
            float m_old = m_run[j];
            float m_new = fmaxf(m_old, mt);
            float p = (sv == -INFINITY) ? 0.f : expf(sv - m_new);
            float ls = wave_sum(p);
            sc[j * TILE + lane] = p;
            if (lane == 0) {
                float al = (m_old == -INFINITY) ? 0.f : expf(m_old - m_new);
                alpha[j] = al;
                m_run[j] = m_new;
                l_run[j] = l_run[j] * al + ls;
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < GT; ++j) {
            float al = alpha[j];
            acc[j].x *= al; acc[j].y *= al; acc[j].z *= al; acc[j].w *= al;
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int tl = wave * ROWS_PER_WAVE + it * RPW + rsel;
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                float p = sc[j * TILE + tl];
                acc[j].x = fmaf(p, vv[it].x, acc[j].x);
                acc[j].y = fmaf(p, vv[it].y, acc[j].y);
                acc[j].z = fmaf(p, vv[it].z, acc[j].z);
                acc[j].w = fmaf(p, vv[it].w, acc[j].w);
            }
        }
        __syncthreads();
    }

    // rows of a wave, then the four waves
#pragma unroll
    for (int j = 0; j < GT; ++j) {
#pragma unroll
        for (int o = LPR; o < kWave; o <<= 1) {
            acc[j].x += __shfl_xor(acc[j].x, o, kWave);
            acc[j].y += __shfl_xor(acc[j].y, o, kWave);
            acc[j].z += __shfl_xor(acc[j].z, o, kWave);
            acc[j].w += __shfl_xor(acc[j].w, o, kWave);
        }
        if (rsel == 0)
            *reinterpret_cast<float4 *>(wacc + ((size_t)(wave * GT + j) * LPR + sub) * 4) = acc[j];
    }
    __syncthreads();
    const int d4 = a.d / 4;
    for (int idx = tid; idx < GT * d4; idx += kBlock) {
        int j = idx / d4, c = idx - j * d4;
        if (ht * GT + j >= G) continue;
        float4 r = make_float4(0, 0, 0, 0);
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            float4 v = *reinterpret_cast<const float4 *>(wacc + ((size_t)(w * GT + j) * LPR + c) * 4);
            r.x += v.x; r.y += v.y; r.z += v.z; r.w += v.w;
        }
        int head = g * G + ht * GT + j;
        float *dst = s.ws + a.ws_att_acc + ((size_t)head * kAttnMaxSplits + split) * a.d + c * 4;
        *reinterpret_cast<float4 *>(dst) = r;
    }
    if (tid < GT && ht * GT + tid < G) {
        int head = g * G + ht * GT + tid;
        s.ws[a.ws_att_m + head * kAttnMaxSplits + split] = m_run[tid];
        s.ws[a.ws_att_l + head * kAttnMaxSplits + split] = l_run[tid];
    }
}

// ---------------------------------------------------------------------------
// Stage 3: merge of the attention splits + row-parallel output projection
// ---------------------------------------------------------------------------
__device__ __forceinline__ void stage_attn_merge(const DecodeArgs &a, const ShardView &s, float *xs)
{
    const int dq = a.nq * a.d;
    for (int k = threadIdx.x * 4; k < dq; k += kBlock * 4) {
        int head = k / a.d, e = k - head * a.d;
        const float *mp = s.ws + a.ws_att_m + head * kAttnMaxSplits;
        const float *lp = s.ws + a.ws_att_l + head * kAttnMaxSplits;
        float M = -INFINITY;
        for (int c = 0; c < a.n_splits; ++c) M = fmaxf(M, mp[c]);
        float L = 0.f;
        float4 o = make_float4(0, 0, 0, 0);
        for (int c = 0; c < a.n_splits; ++c) {
            float w = expf(mp[c] - M);
            L = fmaf(w, lp[c], L);
            float4 v = *reinterpret_cast<const float4 *>(
                s.ws + a.ws_att_acc + ((size_t)head * kAttnMaxSplits + c) * a.d + e);
            o.x = fmaf(w, v.x, o.x); o.y = fmaf(w, v.y, o.y);
            o.z = fmaf(w, v.z, o.z); o.w = fmaf(w, v.w, o.w);
        }
        float inv = 1.0f / L;
        *reinterpret_cast<float4 *>(xs + k) = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    }
    __syncthreads();
}

template <int ROWS, int U>
__global__ __launch_bounds__(kBlock) void k_oproj(DecodeArgs a)
{
    extern __shared__ float smem[];
    const int dq = a.nq * a.d;
    float *xs = smem;
    float *red = smem + dq;
    const ShardView &s = a.s[blockIdx.y];
    const int r0 = blockIdx.x * ROWS;
    const float *rows[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) rows[r] = s.w_o + (size_t)min(r0 + r, a.h - 1) * dq;
    GemvTile<ROWS, U> tile;
    tile.issue(rows, dq, 0);
    stage_attn_merge(a, s, xs);
    float y[ROWS];
    gemv_rows<ROWS, U>(rows, dq, xs, tile, red, y);
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        if (threadIdx.x == r && r0 + r < a.h) s.partial_out[r0 + r] = y[r];
}

// ---------------------------------------------------------------------------
// Stage 4: RMSNorm + gate/up GEMV + SiLU gate
// ---------------------------------------------------------------------------
// A workgroup owns COLS FFN columns j: rows gate_j and up_j, so the product
// silu(gate_j) * up_j is formed in registers.
template <int COLS, int U>
__global__ __launch_bounds__(kBlock) void k_gate_up(DecodeArgs a)
{
    extern __shared__ float smem[];
    float *xs = smem;
    float *red = smem + a.h;
    const ShardView &s = a.s[blockIdx.y];
    constexpr int ROWS = 2 * COLS;
    const int j0 = blockIdx.x * COLS;
    const float *rows[ROWS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        size_t j = (size_t)min(j0 + c, a.sl - 1);
        rows[2 * c] = s.w_gate + j * a.h;
        rows[2 * c + 1] = s.w_up + j * a.h;
    }
    GemvTile<ROWS, U> tile;
    tile.issue(rows, a.h, 0);
    const float rinv = stage_norm_input(a.h_in, s.ffn_norm, a.h, a.eps, xs, red);
    float y[ROWS];
    gemv_rows<ROWS, U>(rows, a.h, xs, tile, red, y);
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        if (threadIdx.x == c && j0 + c < a.sl) {
            float gt = y[2 * c] * rinv, up = y[2 * c + 1] * rinv;
            s.ws[a.ws_act + j0 + c] = gt / (1.0f + expf(-gt)) * up;
        }
    }
}

// ---------------------------------------------------------------------------
// Stage 5: row-parallel down projection
// ---------------------------------------------------------------------------
template <int ROWS, int U>
__global__ __launch_bounds__(kBlock) void k_down(DecodeArgs a)
{
    extern __shared__ float smem[];
    float *xs = smem;
    float *red = smem + a.sl;
    const ShardView &s = a.s[blockIdx.y];
    const int r0 = blockIdx.x * ROWS;
    const float *rows[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) rows[r] = s.w_down + (size_t)min(r0 + r, a.h - 1) * a.sl;
    GemvTile<ROWS, U> tile;
    tile.issue(rows, a.sl, 0);
    stage_copy_input(s.ws + a.ws_act, a.sl, xs);
    float y[ROWS];
    gemv_rows<ROWS, U>(rows, a.sl, xs, tile, red, y);
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        if (threadIdx.x == r && r0 + r < a.h) s.partial_out[r0 + r] = y[r];
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------

static inline unsigned cdiv(unsigned a, unsigned b) { return (a + b - 1) / b; }

template <int GT>
static hipError_t launch_attn_gt(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    const int G = a.nq / a.nkv;
    const int n_ht = (G + GT - 1) / GT;
    dim3 grid(a.n_splits, a.nkv * n_ht, n_shards);
    int lpr = 8;
    while (lpr * 4 < a.d) lpr *= 2;
    size_t lds = sizeof(float) * ((size_t)GT * 64 + 24 + (size_t)kWavesPerBlock * GT * lpr * 4);
    switch (lpr) {
    case 8: hipLaunchKernelGGL((k_attn_split<GT, 8>), grid, dim3(kBlock), lds, st, a); break;
    case 16: hipLaunchKernelGGL((k_attn_split<GT, 16>), grid, dim3(kBlock), lds, st, a); break;
    case 32: hipLaunchKernelGGL((k_attn_split<GT, 32>), grid, dim3(kBlock), lds, st, a); break;
    case 64: hipLaunchKernelGGL((k_attn_split<GT, 64>), grid, dim3(kBlock), lds, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attn_phase(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    const int half = a.d / 2;
    const int npairs = (a.nq + 2 * a.nkv) * half;
    {
        constexpr int PAIRS = 2, U = 4;
        size_t lds = sizeof(float) * ((size_t)a.h + 2 * PAIRS * kWavesPerBlock + kWavesPerBlock);
        ProfScope ps(kStageQkv, st);
        hipLaunchKernelGGL((k_qkv_rope<PAIRS, U>), dim3(cdiv(npairs, PAIRS), n_shards), dim3(kBlock), lds, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        const int G = a.nq / a.nkv;
        ProfScope ps(kStageAttn, st);
        hipError_t e;
        if (G == 1) e = launch_attn_gt<1>(a, n_shards, st);
        else if (G == 2) e = launch_attn_gt<2>(a, n_shards, st);
        else if (G <= 4) e = launch_attn_gt<4>(a, n_shards, st);
        else e = launch_attn_gt<8>(a, n_shards, st);
        if (e != hipSuccess) return e;
    }
    {
        constexpr int ROWS = 8, U = 2;
        const int dq = a.nq * a.d;
        size_t lds = sizeof(float) * ((size_t)dq + ROWS * kWavesPerBlock);
        ProfScope ps(kStageOproj, st);
        hipLaunchKernelGGL((k_oproj<ROWS, U>), dim3(cdiv(a.h, ROWS), n_shards), dim3(kBlock), lds, st, a);
        return hipGetLastError();
    }
}

hipError_t launch_ffn_phase(const DecodeArgs &a, int n_shards, hipStream_t st)
{
    {
        constexpr int COLS = 2, U = 4;
        size_t lds = sizeof(float) * ((size_t)a.h + 2 * COLS * kWavesPerBlock + kWavesPerBlock);
        ProfScope ps(kStageGateUp, st);
        hipLaunchKernelGGL((k_gate_up<COLS, U>), dim3(cdiv(a.sl, COLS), n_shards), dim3(kBlock), lds, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        constexpr int ROWS = 8, U = 2;
        size_t lds = sizeof(float) * ((size_t)a.sl + ROWS * kWavesPerBlock);
        ProfScope ps(kStageDown, st);
        hipLaunchKernelGGL((k_down<ROWS, U>), dim3(cdiv(a.h, ROWS), n_shards), dim3(kBlock), lds, st, a);
        return hipGetLastError();
    }
}

}  // namespace tpi
