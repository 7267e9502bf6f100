// Stage bodies of the fp32 decode path, shared by the per-stage kernels and the
// whole-token persistent kernel.  (vwg, nvwg): this workgroup's index and the
// number of workgroups sharing the stage for one shard; units are dealt out
// cyclically.
#pragma once
#include "decode_args.hpp"
#include "tpi_device.hpp"

namespace tpi {

// RMSNorm folded into a GEMV: xr <- x * g (this thread's slice); returns
// 1/sqrt(mean(x^2) + eps), which scales the row sums afterwards.
template <int KCH>
__device__ __forceinline__ float norm_slice(const float *x, const float *g, int h, float eps, float4 (&xr)[KCH],
                                            float *red)
{
    float4 gr[KCH];
    load_x_slice<KCH>(x, h, xr);
    load_x_slice<KCH>(g, h, gr);
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
        ss = dot4(xr[c], xr[c], ss);
        xr[c] = make_float4(xr[c].x * gr[c].x, xr[c].y * gr[c].y, xr[c].z * gr[c].z, xr[c].w * gr[c].w);
    }
    ss = block_sum(ss, red);
    return 1.0f / sqrtf(ss / (float)h + eps);
}

// Every thread holds all ROWS sums of a unit; thread i takes element i (i < ROWS) without
// dynamic register indexing, so the epilogue of a unit runs on ROWS lanes side by side
// instead of ROWS divergent branches one after the other.
template <int ROWS>
__device__ __forceinline__ float pick_own(const float (&y)[ROWS], int i)
{
    // Each candidate is pinned in a register first.  Left to itself the compiler selects among the
    // ADDRESSES of y[r] instead, which turns y into an indexed array in LDS -- and the code that finds a
    // thread's slot of such an array reads the workgroup size from the dispatch packet, which sits in
    // host memory: microseconds per workgroup.
    float v = y[0];
    asm volatile("" : "+v"(v));
#pragma unroll
    for (int r = 1; r < ROWS; ++r) {
        float yr = y[r];
        asm volatile("" : "+v"(yr));
        v = (i == r) ? yr : v;
    }
    return v;
}

// Output of a row-parallel stage: the shard's partial sum, or -- with the star reduce folded
// in -- the reduced value: partials summed in rank order (this shard's own from the register,
// the peers' from memory), then the shortcut.  Plain fp32 additions, nothing to contract.
__device__ __forceinline__ void emit_row(const ShardView &s, const FusedReduce &rf, int row, float y)
{
    // all peers' values are requested before the first is used: each is a trip to memory
    float v[kMaxBatchShards];
#pragma unroll
    for (int i = 0; i < kMaxBatchShards; ++i) v[i] = (i < rf.n && i != rf.rank) ? rf.peer[i][row] : 0.f;
    const float res = rf.residual ? rf.residual[row] : 0.f;
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxBatchShards; ++i) {
        if (i < rf.n) {
            float t = (i == rf.rank) ? y : v[i];
            acc = (i == 0) ? t : acc + t;
        }
    }
    if (rf.residual) acc = acc + res;
    rf.out[row] = acc;
}

// The same in two halves, for the row-parallel stages: the peers' values and the shortcut of the row a
// thread will finish are requested early -- long before they are needed, so they cost no round trip at
// the end -- and summed once the shard's own value exists.  NP: the number of rank slots compiled in
// (8 or 16); with up to 8 ranks the table of peer pointers is one read of the kernel arguments.
template <int NP>
struct PeerRow {
    float v[NP];
    float res;
};

// Every load is unconditional -- slots without a peer read `dummy[row]` (any readable array of at least
// row + 1 floats) and are ignored later: a load under a branch makes the compiler wait for all earlier
// loads at the join, which would turn these requests into a chain of round trips.
template <int NP>
__device__ __forceinline__ void fetch_peers(const FusedReduce &rf, int row, const float *dummy, PeerRow<NP> &p)
{
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const float *src = (i < rf.n && i != rf.rank) ? rf.peer[i] : dummy;
        p.v[i] = src[row];
    }
    const float *rs = rf.residual ? rf.residual : dummy;
    p.res = rs[row];
}

template <int NP>
__device__ __forceinline__ void emit_row(const FusedReduce &rf, int row, float y, const PeerRow<NP> &p)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        if (i < rf.n) {
            float t = (i == rf.rank) ? y : p.v[i];
            acc = (i == 0) ? t : acc + t;
        }
    }
    if (rf.residual) acc = acc + p.res;
    rf.out[row] = acc;
}

// cos | sin of pos * theta_e for e < d/2 into LDS (rope[e], rope[kRopeHalf + e]); thread e
// computes entry e.  The angle reaches pos radians, so it is formed in fp64: fp32 would lose
// the low bits of the phase.  Callers put a workgroup barrier between this and the first use.
constexpr int kRopeHalf = 128;   // == TPI_MAX_HEAD_DIM / 2
__device__ __forceinline__ void fill_rope_table(const DecodeDims &a, float *rope)
{
    const int e = threadIdx.x;
    if (e < a.d / 2) {
        float cs = 1.f, sn = 0.f;
        if (a.pos != 0) {
            double theta = exp2(-(2.0 * (double)e / (double)a.d) * a.log2_base);
            double sd, cd;
            sincos((double)a.pos * theta, &sd, &cd);
            cs = (float)cd;
            sn = (float)sd;
        }
        rope[e] = cs;
        rope[kRopeHalf + e] = sn;
    }
}

// Stage 1: a unit is PAIRS rotary pairs (i, i + d/2) of one head, so a pair is
// rotated in registers.  V rows use the same pairing, unrotated.
template <int PAIRS, int KCH, int UB>
__device__ __forceinline__ void stage_qkv(const DecodeDims &a, const ShardView &s, int vwg, int nvwg, float *red,
                                          float *rope)
{
    // Every scalar argument the stage needs is requested here, in one batch: read where they are first used,
    // the loads from the argument block form a chain of round trips (shape, then branch, then pointer) ahead
    // of the first weight request.  The other stages begin the same way.
    asm volatile("" ::"s"(a.h), "s"(a.nq), "s"(a.nkv), "s"(a.d), "s"(a.max_seq), "s"(a.pos), "s"(a.eps), "s"(a.h_in),
                 "s"(s.w_qkv), "s"(s.attn_norm), "s"(s.ws), "s"(s.k), "s"(s.v), "s"(a.ws_q), "s"(a.ws_cnt));
    constexpr int ROWS = 2 * PAIRS;
    const int half = a.d / 2;
    const int npairs = (a.nq + 2 * a.nkv) * half;
    const int n_units = (npairs + PAIRS - 1) / PAIRS;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
#pragma unroll
        for (int i = 0; i < PAIRS; ++i) {
            int p = min(u * PAIRS + i, npairs - 1);
            int hd = p / half, e = p - hd * half;
            rows[2 * i] = s.w_qkv + ((size_t)hd * a.d + e) * a.h;
            rows[2 * i + 1] = rows[2 * i] + (size_t)half * a.h;
        }
    };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(vwg, nvwg, n_units, a.h, rowfn);
    if (vwg == 0)
        for (int g = threadIdx.x; g < a.nkv; g += kBlock) s.ws_u32()[a.ws_cnt + g] = 0u;   // attention tickets
    fill_rope_table(a, rope);                      // visible after the barriers inside norm_slice
    float4 xr[KCH];
    const float rinv = norm_slice<KCH>(a.h_in, s.attn_norm, a.h, a.eps, xr, red);
    auto epi = [&](int u, float (&y)[ROWS]) {
        const int i = threadIdx.x;                 // lane i finishes pair i of the unit
        float lo = y[0], hi = y[1];
#pragma unroll
        for (int q = 1; q < PAIRS; ++q) {
            lo = (i == q) ? y[2 * q] : lo;
            hi = (i == q) ? y[2 * q + 1] : hi;
        }
        const int p = u * PAIRS + i;
        if (i < PAIRS && p < npairs) {
            int hd = p / half, e = p - hd * half;
            lo *= rinv; hi *= rinv;
            float *dst;
            float cs = 1.f, sn = 0.f;
            if (hd < a.nq + a.nkv) { cs = rope[e]; sn = rope[kRopeHalf + e]; }
            if (hd < a.nq) dst = s.ws + a.ws_q + (size_t)hd * a.d;
            else if (hd < a.nq + a.nkv) dst = s.k + ((size_t)(hd - a.nq) * a.max_seq + a.pos) * a.d;
            else dst = s.v + ((size_t)(hd - a.nq - a.nkv) * a.max_seq + a.pos) * a.d;
            dst[e] = lo * cs - hi * sn;
            dst[e + half] = hi * cs + lo * sn;
        }
    };
    st.run(xr, red, rowfn, epi);
}

// Stage 3: a unit is ROWS rows of W_o; the input is the merged attention output.
template <int ROWS, int KCH, int UB, bool FOLD, int NP = kMaxBatchShards>
__device__ __forceinline__ void stage_oproj(const DecodeDims &a, const ShardView &s, int vwg, int nvwg, float *red,
                                            const FusedReduce &rf)
{
    asm volatile("" ::"s"(a.h), "s"(a.nq), "s"(a.d), "s"(s.w_o), "s"(s.ws), "s"(a.ws_o), "s"(s.partial_out));
    const int dq = a.nq * a.d;
    const int n_units = (a.h + ROWS - 1) / ROWS;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) rows[r] = s.w_o + (size_t)min(u * ROWS + r, a.h - 1) * dq;
    };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(vwg, nvwg, n_units, dq, rowfn);
    float4 xr[KCH];
    load_x_slice<KCH>(s.ws + a.ws_o, dq, xr);
    // With the reduce folded in, thread i finishes row i of this workgroup's rows (the launcher sizes the
    // grid so that a workgroup owns at most 256 rows).  Its peers' values are requested here, behind the
    // first weight batch in the in-order memory pipe (ahead of it they would hold the weights back) and
    // long before they are needed.
    constexpr bool fold = FOLD;      // compile-time: the plain stage carries none of the folding code
    int my_row = -1;
    PeerRow<NP> peers;
    if constexpr (fold) {
        if (vwg < n_units) {
            const int my_rows = ((n_units - vwg + nvwg - 1) / nvwg) * ROWS;
            const int i = threadIdx.x;
            const int row = (vwg + (i / ROWS) * nvwg) * ROWS + (i % ROWS);
            if (i < my_rows && row < a.h) {
                my_row = row;
                fetch_peers(rf, row, s.w_o, peers);
            }
        }
    }
    // A unit's sums wait in LDS and all rows of the workgroup are reduced together after the last unit.
    __shared__ float ysave[kBlock];
    auto epi = [&](int u, float (&y)[ROWS]) {
        if constexpr (fold) {
            const int r = threadIdx.x;
            const float mine = pick_own<ROWS>(y, r);
            if (r < ROWS) ysave[(((u - vwg) / nvwg) * ROWS + r) & (kBlock - 1)] = mine;
        } else {
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                if (threadIdx.x == r && u * ROWS + r < a.h) s.partial_out[u * ROWS + r] = y[r];
        }
    };
    st.run(xr, red, rowfn, epi);
    if constexpr (fold) if (vwg < n_units) {
        __syncthreads();
        if (my_row >= 0) emit_row(rf, my_row, ysave[threadIdx.x], peers);
    }
}

// Stage 4: a unit is COLS FFN columns j (rows gate_j and up_j), so
// silu(gate_j) * up_j is formed in registers.
template <int COLS, int KCH, int UB>
__device__ __forceinline__ void stage_gate_up(const DecodeDims &a, const ShardView &s, int vwg, int nvwg, float *red)
{
    asm volatile("" ::"s"(a.h), "s"(a.sl), "s"(a.eps), "s"(a.h_in), "s"(s.w_gate), "s"(s.w_up), "s"(s.ffn_norm), "s"(s.ws),
                 "s"(a.ws_act));
    constexpr int ROWS = 2 * COLS;
    const int n_units = (a.sl + COLS - 1) / COLS;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            size_t j = (size_t)min(u * COLS + c, a.sl - 1);
            rows[2 * c] = s.w_gate + j * a.h;
            rows[2 * c + 1] = s.w_up + j * a.h;
        }
    };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(vwg, nvwg, n_units, a.h, rowfn);
    float4 xr[KCH];
    const float rinv = norm_slice<KCH>(a.h_in, s.ffn_norm, a.h, a.eps, xr, red);
    auto epi = [&](int u, float (&y)[ROWS]) {
        const int c = threadIdx.x;                 // lane c finishes column c of the unit
        float gt = y[0], up = y[1];
#pragma unroll
        for (int q = 1; q < COLS; ++q) {
            gt = (c == q) ? y[2 * q] : gt;
            up = (c == q) ? y[2 * q + 1] : up;
        }
        const int j = u * COLS + c;
        if (c < COLS && j < a.sl) {
            gt *= rinv; up *= rinv;
            s.ws[a.ws_act + j] = gt / (1.0f + expf(-gt)) * up;
        }
    };
    st.run(xr, red, rowfn, epi);
}

// A row-parallel stage for ALL shards of a batched call with the star reduce folded in: the workgroup owns ROWS
// rows of the output and walks the shards in rank order (unit = shard), each with its own weight rows and its own
// input vector; a shard's ROWS sums are exactly the partial the one-shard stage stores (same threads, same order of
// additions), and they are added as the star reduce adds them: ((p0 + p1) + ... + p_{n-1}) + residual.  The
// partial vectors never go to memory.  DOWN: the down projection (input: the shard's activation), else the output
// projection (input: the shard's attention output).
template <int ROWS, int KCH, int UB, bool DOWN>
__device__ __forceinline__ void stage_rowpar_all(const DecodeArgs &a, int n_shards, int rg, float *red)
{
    asm volatile("" ::"s"(a.h), "s"(a.sl), "s"(a.nq), "s"(a.d), "s"(a.ws_act), "s"(a.ws_o), "s"(a.rf.residual), "s"(a.rf.out));
    const int K = DOWN ? a.sl : a.nq * a.d;
    const int xoff = DOWN ? a.ws_act : a.ws_o;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
        const float *W = DOWN ? a.s[u].w_down : a.s[u].w_o;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) rows[r] = W + (size_t)min(rg * ROWS + r, a.h - 1) * K;
    };
    auto xfn = [&](int u, float4 (&x)[KCH]) { load_x_slice<KCH>(a.s[u].ws + xoff, K, x); };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(0, 1, n_shards, K, rowfn);
    float tot[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) tot[r] = 0.f;
    auto epi = [&](int u, float (&y)[ROWS]) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) tot[r] = (u == 0) ? y[r] : tot[r] + y[r];
        if (u == n_shards - 1) {
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = rg * ROWS + r;
                if (threadIdx.x == r && row < a.h) a.rf.out[row] = tot[r] + a.rf.residual[row];
            }
        }
    };
    st.run_x(xfn, red, rowfn, epi);
}

// Stage 5: a unit is ROWS rows of W_down.
template <int ROWS, int KCH, int UB, bool FOLD, int NP = kMaxBatchShards>
__device__ __forceinline__ void stage_down(const DecodeDims &a, const ShardView &s, int vwg, int nvwg, float *red,
                                           const FusedReduce &rf)
{
    asm volatile("" ::"s"(a.h), "s"(a.sl), "s"(s.w_down), "s"(s.ws), "s"(a.ws_act), "s"(s.partial_out));
    const int n_units = (a.h + ROWS - 1) / ROWS;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) rows[r] = s.w_down + (size_t)min(u * ROWS + r, a.h - 1) * a.sl;
    };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(vwg, nvwg, n_units, a.sl, rowfn);
    float4 xr[KCH];
    load_x_slice<KCH>(s.ws + a.ws_act, a.sl, xr);
    // see stage_oproj
    constexpr bool fold = FOLD;
    int my_row = -1;
    PeerRow<NP> peers;
    if constexpr (fold) {
        if (vwg < n_units) {
            const int my_rows = ((n_units - vwg + nvwg - 1) / nvwg) * ROWS;
            const int i = threadIdx.x;
            const int row = (vwg + (i / ROWS) * nvwg) * ROWS + (i % ROWS);
            if (i < my_rows && row < a.h) {
                my_row = row;
                fetch_peers(rf, row, s.w_down, peers);
            }
        }
    }
    __shared__ float ysave[kBlock];
    auto epi = [&](int u, float (&y)[ROWS]) {
        if constexpr (fold) {
            const int r = threadIdx.x;
            const float mine = pick_own<ROWS>(y, r);
            if (r < ROWS) ysave[(((u - vwg) / nvwg) * ROWS + r) & (kBlock - 1)] = mine;
        } else {
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
                if (threadIdx.x == r && u * ROWS + r < a.h) s.partial_out[u * ROWS + r] = y[r];
        }
    };
    st.run(xr, red, rowfn, epi);
    if constexpr (fold) if (vwg < n_units) {
        __syncthreads();
        if (my_row >= 0) emit_row(rf, my_row, ysave[threadIdx.x], peers);
    }
}

// ---------------------------------------------------------------------------
// Stage 2: attention of the local heads over cache slots 0..pos
// ---------------------------------------------------------------------------
// One workgroup = one KV head x one tile of GT of its query heads x one split
// of the slots.  A tile is 64 slots, 16 per wave, and the four waves work
// independently until the end:
//   scores   a row of 16 lanes owns one slot (4 slots per pass, 4 passes);
//            each lane holds EPL float4 of the key and of every query, the
//            16 partial dot products meet in a DPP row reduction -- no LDS,
//            no cross-lane memory traffic;
//   softmax  wave-local running (max, sum) per head;
//   values   a lane owns EPL consecutive elements of the head dimension, the
//            wave's 16 V rows sit in registers, a slot's probability is
//            broadcast with readlane.
// The four wave partials meet in LDS; the split's (max, sum, unnormalised
// output) goes to the workspace and the workgroup that takes the last ticket
// of its KV head merges the splits into the normalised output.
template <int EPL> struct VecOf;
template <> struct VecOf<1> { typedef float T; };
template <> struct VecOf<2> { typedef float2 T; };
template <> struct VecOf<4> { typedef float4 T; };

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), CTRL, 0xF, 0xF, true));
}

// sum over each row of 16 lanes, result in all 16 lanes
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_mov<0xB1>(x);     // quad_perm [1,0,3,2]
    x += dpp_mov<0x4E>(x);     // quad_perm [2,3,0,1]
    x += dpp_mov<0x124>(x);    // row_ror 4
    x += dpp_mov<0x128>(x);    // row_ror 8
    return x;
}

// value of lane l (wave-uniform index) as a wave-uniform float
__device__ __forceinline__ float lane_value(float x, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

template <int GT, int EPL>
__device__ __forceinline__ void stage_attn(const DecodeDims &a, const ShardView &s, int split, int g, int ht,
                                           float *smem)
{
    constexpr int TILE = 64, KPW = TILE / kWavesPerBlock, PASSES = KPW / 4;   // 16 slots per wave, 4 per pass
    typedef typename VecOf<EPL>::T vec_t;
    const int d = a.d;
    float *wacc = smem;                            // [waves][GT][d]   wave partial outputs
    float *wm = smem + kWavesPerBlock * GT * d;    // [waves][GT]      wave maxima
    float *wl = wm + kWavesPerBlock * GT;          // [waves][GT]      wave sums
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int row = lane >> 4, eg = lane & 15;     // score phase: slot within the pass, slice of the head dimension
    const int G = a.nq / a.nkv;
    const int n_ht = (G + GT - 1) / GT;
    const int n_valid = a.pos + 1;
    const int t_begin = split * a.chunk_len;
    const int t_end = min(t_begin + a.chunk_len, n_valid);
    const float *Kg = s.k + (size_t)g * a.max_seq * d;
    const float *Vg = s.v + (size_t)g * a.max_seq * d;
    const float scale = 1.0f / sqrtf((float)d);
    const int d4 = d / 4;
    const bool e_ok = lane * EPL < d;              // value phase: this lane's elements exist

    // this lane's slice of every query of the tile (rotated q, scaled once here)
    float4 qv[GT][EPL];
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        int hj = min(ht * GT + j, G - 1);
        const float *qp = s.ws + a.ws_q + (size_t)(g * G + hj) * d;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            int e = (eg * EPL + c) * 4;
            float4 v = (e < d) ? *reinterpret_cast<const float4 *>(qp + e) : make_float4(0.f, 0.f, 0.f, 0.f);
            qv[j][c] = make_float4(v.x * scale, v.y * scale, v.z * scale, v.w * scale);
        }
    }
    float m_run[GT], l_run[GT];
    vec_t acc[GT];
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        m_run[j] = -INFINITY; l_run[j] = 0.f;
        float *ap = reinterpret_cast<float *>(&acc[j]);
#pragma unroll
        for (int i = 0; i < EPL; ++i) ap[i] = 0.f;
    }

    for (int t0 = t_begin; t0 < t_end; t0 += TILE) {
        const int tw = t0 + wave * KPW;            // first slot of this wave in the tile
        float4 kr[PASSES][EPL];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            int t = tw + i * 4 + row;
#pragma unroll
            for (int c = 0; c < EPL; ++c) {
                int e = (eg * EPL + c) * 4;
                kr[i][c] = (t < t_end && e < d) ? *reinterpret_cast<const float4 *>(Kg + (size_t)t * d + e)
                                                : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
        vec_t vr[KPW];
#pragma unroll
        for (int k = 0; k < KPW; ++k) {
            float *vp = reinterpret_cast<float *>(&vr[k]);
#pragma unroll
            for (int i = 0; i < EPL; ++i) vp[i] = 0.f;
            if (e_ok && tw + k < t_end) vr[k] = *reinterpret_cast<const vec_t *>(Vg + (size_t)(tw + k) * d + lane * EPL);
        }
        // scores of slot (pass i, row) against every head, in all 16 lanes of the row
        float sc[PASSES][GT];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const bool ok = tw + i * 4 + row < t_end;
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                float p = 0.f;
#pragma unroll
                for (int c = 0; c < EPL; ++c) p = dot4(qv[j][c], kr[i][c], p);
                p = row16_sum(p);
                sc[i][j] = ok ? p : -INFINITY;
            }
        }
        // wave-local running softmax: maximum and sum over the wave's 16 slots
#pragma unroll
        for (int j = 0; j < GT; ++j) {
            float mt = sc[0][j];
#pragma unroll
            for (int i = 1; i < PASSES; ++i) mt = fmaxf(mt, sc[i][j]);
            mt = fmaxf(fmaxf(lane_value(mt, 0), lane_value(mt, 16)), fmaxf(lane_value(mt, 32), lane_value(mt, 48)));
            const float m_new = fmaxf(m_run[j], mt);
            float ls = 0.f;
#pragma unroll
            for (int i = 0; i < PASSES; ++i) {
                sc[i][j] = (sc[i][j] == -INFINITY) ? 0.f : __expf(sc[i][j] - m_new);
                ls += sc[i][j];
            }
            ls = (lane_value(ls, 0) + lane_value(ls, 16)) + (lane_value(ls, 32) + lane_value(ls, 48));
            const float al = (m_run[j] == -INFINITY) ? 0.f : __expf(m_run[j] - m_new);
            l_run[j] = l_run[j] * al + ls;
            m_run[j] = m_new;
            float *ap = reinterpret_cast<float *>(&acc[j]);
#pragma unroll
            for (int i = 0; i < EPL; ++i) ap[i] *= al;
        }
        // values: slot k of the wave = (pass k / 4, row k % 4); its probability sits in lane 16 * row
#pragma unroll
        for (int k = 0; k < KPW; ++k) {
            const float *vp = reinterpret_cast<const float *>(&vr[k]);
#pragma unroll
            for (int j = 0; j < GT; ++j) {
                float pk = lane_value(sc[k / 4][j], 16 * (k % 4));
                float *ap = reinterpret_cast<float *>(&acc[j]);
#pragma unroll
                for (int i = 0; i < EPL; ++i) ap[i] = fmaf(pk, vp[i], ap[i]);
            }
        }
    }

    // the four waves' partials meet in LDS
#pragma unroll
    for (int j = 0; j < GT; ++j) {
        if (e_ok) *reinterpret_cast<vec_t *>(wacc + (size_t)(wave * GT + j) * d + lane * EPL) = acc[j];
        if (lane == 0) { wm[wave * GT + j] = m_run[j]; wl[wave * GT + j] = l_run[j]; }
    }
    __syncthreads();
    const int total = a.n_splits * n_ht;           // workgroups per KV head
    for (int i = tid; i < GT * d4; i += kBlock) {
        int j = i / d4, c = i - j * d4;
        if (ht * GT + j >= G) continue;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) M = fmaxf(M, wm[w * GT + j]);
        float L = 0.f;
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            float mw = wm[w * GT + j];
            float wt = (mw == -INFINITY) ? 0.f : __expf(mw - M);
            L = fmaf(wt, wl[w * GT + j], L);
            float4 v = *reinterpret_cast<const float4 *>(wacc + (size_t)(w * GT + j) * d + c * 4);
            o.x = fmaf(wt, v.x, o.x); o.y = fmaf(wt, v.y, o.y);
            o.z = fmaf(wt, v.z, o.z); o.w = fmaf(wt, v.w, o.w);
        }
        const int head = g * G + ht * GT + j;
        if (total == 1) {
            float inv = 1.0f / L;
            *reinterpret_cast<float4 *>(s.ws + a.ws_o + (size_t)head * d + c * 4) =
                make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
        } else {
            *reinterpret_cast<float4 *>(s.ws + a.ws_att_acc + ((size_t)head * kAttnMaxSplits + split) * d + c * 4) = o;
            if (c == 0) {
                s.ws[a.ws_att_m + head * kAttnMaxSplits + split] = M;
                s.ws[a.ws_att_l + head * kAttnMaxSplits + split] = L;
            }
        }
    }
    if (total == 1) return;

    // The last workgroup of this KV head to arrive merges the splits.  Release: every thread waits until its own
    // partial stores have been acknowledged (they are then in this die's L2), and behind the workgroup barrier one
    // thread writes the L2 back at device scope and takes the ticket.  Acquire: the thread that took the last ticket
    // invalidates at device scope before the barrier that lets the other waves read; the vector L1 is one per
    // compute unit and the L2 one per die, shared by all waves of the workgroup, so one thread's write-back and
    // invalidate serve them all (a fence per thread measured 1.6 us per layer more for the same effect).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        unsigned old = atomicAdd(s.ws_u32() + a.ws_cnt + g, 1u);
        s_last = (old == (unsigned)total - 1u);
        if (s_last) __threadfence();
    }
    __syncthreads();
    if (!s_last) return;
    for (int i = tid; i < G * d4; i += kBlock) {
        int j = i / d4, c = i - j * d4;
        int head = g * G + j;
        const float *mp = s.ws + a.ws_att_m + head * kAttnMaxSplits;
        const float *lp = s.ws + a.ws_att_l + head * kAttnMaxSplits;
        const float *ap = s.ws + a.ws_att_acc + (size_t)head * kAttnMaxSplits * d + c * 4;
        // every load of the merge is issued before any is used: the partials come from other compute units'
        // writes, each a trip to memory, and one trip is all the merge should wait for
        float wgt[kAttnMaxSplits], lv[kAttnMaxSplits];
        float4 v[kAttnMaxSplits];
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) {
            wgt[sp] = (sp < a.n_splits) ? mp[sp] : -INFINITY;
            lv[sp] = (sp < a.n_splits) ? lp[sp] : 0.f;
            v[sp] = (sp < a.n_splits) ? *reinterpret_cast<const float4 *>(ap + (size_t)sp * d)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        float M = -INFINITY;
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) M = fmaxf(M, wgt[sp]);
        float L = 0.f;
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int sp = 0; sp < kAttnMaxSplits; ++sp) {
            const float w = (sp < a.n_splits) ? __expf(wgt[sp] - M) : 0.f;
            L = fmaf(w, lv[sp], L);
            o.x = fmaf(w, v[sp].x, o.x); o.y = fmaf(w, v[sp].y, o.y);
            o.z = fmaf(w, v[sp].z, o.z); o.w = fmaf(w, v[sp].w, o.w);
        }
        float inv = 1.0f / L;
        *reinterpret_cast<float4 *>(s.ws + a.ws_o + (size_t)head * d + c * 4) =
            make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    }
    if (tid == 0) s.ws_u32()[a.ws_cnt + g] = 0u;  // ready for the next call
}

}  // namespace tpi
