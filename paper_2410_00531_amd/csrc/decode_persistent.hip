// Whole-token decode of ONE device's shard in a single persistent kernel.
//
// The per-stage kernels pay a launch, a ramp-up and a drain for each of the
// seven dependent steps of a layer; at batch 1 those floors cost as much as
// the streaming itself.  Here one cooperative grid of co-resident workgroups
// walks all layers of a token: the five stages of a layer are separated by
// grid barriers instead of kernel boundaries, the star reduce with the
// shortcut is folded into the epilogues of the two row-parallel stages (this
// device's partial comes from registers, the peers' partials from memory),
// and no activation leaves the chip's caches.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "../../include/tpi.h"
#include "decode_args.hpp"
#include "decode_stages.hpp"
#include "decode_wave.hpp"
#include "host_util.hpp"
#include "prof.hpp"

namespace tpi {

struct LayerPtrs {
    const float *attn_norm, *w_qkv, *w_o, *ffn_norm, *w_gate, *w_up, *w_down;
    float *k, *v;
};

struct TokenArgs {
    DecodeDims dm;                     // h_in is rewritten per stage on the device
    int n_layers;
    const LayerPtrs *layers;           // device table [n_layers]
    const float *h_in;                 // [h] input hidden state of layer 0
    float *h_out;                      // [h] output of the last layer
    float *ws;                         // per-shard decode workspace (q, attention partials, act, tickets)
    float *h_attn, *xa, *xb;           // [h] each, in the decoder workspace
    unsigned long long *bar_words;     // barrier tree: [0] generation flag, [16] root, [32 + 16 g] group g
    unsigned *bar_error;               // set when a barrier wait gave up
    unsigned long long bar_gen0;       // barrier generations completed before this launch
    int n_ranks, rank;
    int xs_floats;                     // LDS floats reserved for the stage input vector
    const float *const *peer_attn;     // device tables [n_ranks] of the peers' partial vectors
    const float *const *peer_ffn;      // (entry `rank` unused)
};

constexpr unsigned kSpinLimit = 1u << 22;   // polls before a barrier wait gives up (seconds of wall time)
constexpr int kBarGroup = 16;               // workgroups per leaf counter of the barrier tree

// Barrier over the whole (co-resident) grid.  Arrivals to one address are served one after the
// other by the memory side, so they are counted in a two-level tree: a workgroup adds to its
// group's counter (groups of 16, each counter on a cache line of its own), the last of a group
// adds to the root, the last at the root publishes the barrier's generation number, and everybody
// polls that one read-only word.  All counters are monotonic over the decoder's life (bar_gen0 is
// the generation before this launch), so nothing is ever reset.
// One thread per workgroup carries the release fence, the arrival, the bounded wait and the
// acquire fence; the workgroup barriers around it extend them to every wave.  Returns false when
// the wait gave up or another workgroup reported failure: the caller then leaves the kernel, so
// every wave reaches its exit whatever happens.
__device__ __forceinline__ void grid_arrive(const TokenArgs &t, unsigned &epoch)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        epoch += 1;
        const unsigned long long gen = t.bar_gen0 + epoch;          // generation this barrier publishes
        const int n_groups = (gridDim.x + kBarGroup - 1) / kBarGroup;
        const int grp = blockIdx.x / kBarGroup;
        const int gsize = min(kBarGroup, (int)gridDim.x - grp * kBarGroup);
        unsigned long long *leaf = t.bar_words + 16 * (2 + grp);    // 128-byte stride
        unsigned long long *root = t.bar_words + 16;
        unsigned long long *flag = t.bar_words;
        __threadfence();
        unsigned long long old = __hip_atomic_fetch_add(leaf, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == gen * (unsigned long long)gsize) {            // last of the group
            old = __hip_atomic_fetch_add(root, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old + 1 == gen * (unsigned long long)n_groups)       // last of all
                __hip_atomic_store(flag, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__device__ __forceinline__ bool grid_wait(const TokenArgs &t, unsigned epoch, int *s_flag)
{
    if (threadIdx.x == 0) {
        const unsigned long long gen = t.bar_gen0 + epoch;
        unsigned long long *flag = t.bar_words;
        int ok = 1;
        unsigned spins = 0;
        while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < gen) {
            __builtin_amdgcn_s_sleep(4);
            if ((++spins & 1023u) == 0) {
                if (spins >= kSpinLimit ||
                    __hip_atomic_load(t.bar_error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                    __hip_atomic_store(t.bar_error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = 0;
                    break;
                }
            }
        }
        __threadfence();
        *s_flag = ok;
    }
    __syncthreads();
    return *s_flag != 0;
}

// arrive and wait in one go
__device__ __forceinline__ bool grid_barrier(const TokenArgs &t, unsigned &epoch, int *s_flag)
{
    grid_arrive(t, epoch);
    return grid_wait(t, epoch, s_flag);
}

// XCH_*: 256-float chunks (rounded up to a power of two) of the hidden size, the shard's FFN
// width and the shard's query width; GT, EPL: attention head tile and elements per lane.
template <int XCH_H, int XCH_SL, int XCH_DQ, int GT, int EPL>
__global__ __launch_bounds__(kBlock, 1) void k_decode_token(TokenArgs t)
{
    extern __shared__ float smem[];                 // [xs: stage input vector | attention: wave partials]
    __shared__ float rope[2 * kRopeHalf];           // cos | sin of pos * theta_e, e < d/2
    __shared__ float red[kWavesPerBlock];
    __shared__ int s_flag;
    constexpr int kSaveUnits = 32;                  // units of a row-parallel stage one wave may own (checked at create)
    __shared__ float ysave[kWavesPerBlock * kSaveUnits * 16];
    float *xs = smem;
    float *attn_smem = smem + t.xs_floats;
    // a batch is kBatch float4 per lane (two batches in flight): CB chunks of ROWS rows
    constexpr int kBatch = 16;
    constexpr int CB_H = XCH_H < kBatch / 2 ? XCH_H : kBatch / 2, ROWS_H = kBatch / CB_H;
    constexpr int CB_SL = XCH_SL < kBatch / 2 ? XCH_SL : kBatch / 2, ROWS_SL = kBatch / CB_SL;
    constexpr int CB_DQ = XCH_DQ < kBatch / 2 ? XCH_DQ : kBatch / 2, ROWS_DQ = kBatch / CB_DQ;
    constexpr int PAIRS = ROWS_H / 2, COLS = ROWS_H / 2;

    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int vwg = blockIdx.x;
    const int vw = vwg * kWavesPerBlock + wave, nvw = gridDim.x * kWavesPerBlock;   // wave index in the grid
    unsigned epoch = 0;
    const DecodeDims &dm = t.dm;
    const int G = dm.nq / dm.nkv;
    const int n_ht = (G + GT - 1) / GT;
    const int n_attn_units = dm.nkv * n_ht * dm.n_splits;
    const int half = dm.d / 2, dq = dm.nq * dm.d;
    const int npairs = (dm.nq + 2 * dm.nkv) * half;

    // rotary table of this token (the angle is the same in every layer)
    fill_rope_table(dm, rope);
    __syncthreads();

    WaveStreamer<2 * PAIRS, CB_H> st_qkv;     // the only streamer alive across the layer loop's back edge

    const float *x = t.h_in;
    LayerPtrs lp = t.layers[0];
    QkvRows<PAIRS> r_qkv{lp.w_qkv, dm.d, dm.h, half, npairs};
    st_qkv.prefetch(vw, nvw, (npairs + PAIRS - 1) / PAIRS, dm.h, r_qkv);

    for (int l = 0; l < t.n_layers; ++l) {
        ShardView s;
        s.attn_norm = lp.attn_norm; s.w_qkv = lp.w_qkv; s.w_o = lp.w_o; s.ffn_norm = lp.ffn_norm;
        s.w_gate = lp.w_gate; s.w_up = lp.w_up; s.w_down = lp.w_down;
        s.k = lp.k; s.v = lp.v; s.partial_out = nullptr; s.ws = t.ws;
        float *x_next = (l == t.n_layers - 1) ? t.h_out : ((l & 1) ? t.xb : t.xa);
        PlainRows<ROWS_DQ> r_o{lp.w_o, dm.h, dq};
        GateUpRows<COLS> r_gu{lp.w_gate, lp.w_up, dm.sl, dm.h};
        PlainRows<ROWS_SL> r_dn{lp.w_down, dm.h, dm.sl};

#ifdef TPI_TRACE
#define TPI_TRACE_L(slot) do { if (l == 1) TPI_TRACE_AT(vwg, slot); } while (0)
#else
#define TPI_TRACE_L(slot) do { } while (0)
#endif
        TPI_TRACE_L(0);
        // ---- stage 1: RMSNorm + QKV + rotary + cache append --------------------------------
        {
            if (vwg == 0 && threadIdx.x < dm.nkv) s.ws_u32()[dm.ws_cnt + threadIdx.x] = 0u;   // attention tickets
            const float rinv = stage_x_norm(x, lp.attn_norm, dm.h, dm.eps, xs, red);
            auto epi = [&](int u, float (&y)[2 * PAIRS]) {
                float lo = y[0], hi = y[1];
#pragma unroll
                for (int q = 1; q < PAIRS; ++q) {
                    lo = (lane == q) ? y[2 * q] : lo;
                    hi = (lane == q) ? y[2 * q + 1] : hi;
                }
                const int p = u * PAIRS + lane;
                if (lane < PAIRS && p < npairs) {
                    int hd = p / half, e = p - hd * half;
                    lo *= rinv; hi *= rinv;
                    float cs = 1.f, sn = 0.f;
                    float *dst;
                    if (hd < dm.nq + dm.nkv) { cs = rope[e]; sn = rope[kRopeHalf + e]; }
                    if (hd < dm.nq) dst = s.ws + dm.ws_q + (size_t)hd * dm.d;
                    else if (hd < dm.nq + dm.nkv) dst = s.k + ((size_t)(hd - dm.nq) * dm.max_seq + dm.pos) * dm.d;
                    else dst = s.v + ((size_t)(hd - dm.nq - dm.nkv) * dm.max_seq + dm.pos) * dm.d;
                    dst[e] = lo * cs - hi * sn;
                    dst[e + half] = hi * cs + lo * sn;
                }
            };
            st_qkv.run(xs, r_qkv, epi);
        }
        TPI_TRACE_L(1);

        // ---- stage 2: attention on a few workgroups; everyone else already pulls W_o ---------
        WaveStreamer<ROWS_DQ, CB_DQ> st_o;
        if (vwg < n_attn_units) {
            if (!grid_barrier(t, epoch, &s_flag)) return;
            for (int u = vwg; u < n_attn_units; u += gridDim.x) {
                int split = u % dm.n_splits, gh = u / dm.n_splits;
                stage_attn<GT, EPL>(dm, s, split, gh / n_ht, gh % n_ht, attn_smem);
                __syncthreads();                       // LDS of the stage is reused by the next unit
            }
            TPI_TRACE_L(3);
            st_o.prefetch(vw, nvw, (dm.h + ROWS_DQ - 1) / ROWS_DQ, dq, r_o);
            if (!grid_barrier(t, epoch, &s_flag)) return;
        } else {
            grid_arrive(t, epoch);
            st_o.prefetch(vw, nvw, (dm.h + ROWS_DQ - 1) / ROWS_DQ, dq, r_o);
            if (!grid_wait(t, epoch, &s_flag)) return;
            if (!grid_barrier(t, epoch, &s_flag)) return;
        }

        TPI_TRACE_L(4);
        // ---- stage 3: output projection, reduce 1 + shortcut folded in -> H_attn -------------
        {
            FusedReduce rf;
            rf.n = t.n_ranks; rf.rank = t.rank; rf.residual = x; rf.out = t.h_attn;
#pragma unroll
            for (int i = 0; i < kMaxBatchShards; ++i) rf.peer[i] = t.peer_attn[i];
            stage_x_plain(s.ws + dm.ws_o, dq, xs);
            // sums wait in LDS; the rows are reduced after the last unit (no loads inside the pipeline)
            int n_saved = 0;
            auto epi = [&](int u, float (&y)[ROWS_DQ]) {
                const float mine = pick_own<ROWS_DQ>(y, lane);
                if (lane < ROWS_DQ && n_saved < kSaveUnits) ysave[(wave * kSaveUnits + n_saved) * 16 + lane] = mine;
                n_saved += 1;
            };
            st_o.run(xs, r_o, epi);
            for (int k = 0; k < n_saved && k < kSaveUnits; ++k) {
                const int row = (vw + k * nvw) * ROWS_DQ + lane;
                if (lane < ROWS_DQ && row < dm.h) emit_row(s, rf, row, ysave[(wave * kSaveUnits + k) * 16 + lane]);
            }
        }
        TPI_TRACE_L(5);
        WaveStreamer<2 * COLS, CB_H> st_gu;
        grid_arrive(t, epoch);
        st_gu.prefetch(vw, nvw, (dm.sl + COLS - 1) / COLS, dm.h, r_gu);
        if (!grid_wait(t, epoch, &s_flag)) return;

        TPI_TRACE_L(6);
        // ---- stage 4: RMSNorm + gate/up + SiLU gate -------------------------------------------
        {
            const float rinv = stage_x_norm(t.h_attn, lp.ffn_norm, dm.h, dm.eps, xs, red);
            auto epi = [&](int u, float (&y)[2 * COLS]) {
                float gt = y[0], up = y[1];
#pragma unroll
                for (int q = 1; q < COLS; ++q) {
                    gt = (lane == q) ? y[2 * q] : gt;
                    up = (lane == q) ? y[2 * q + 1] : up;
                }
                const int j = u * COLS + lane;
                if (lane < COLS && j < dm.sl) {
                    gt *= rinv; up *= rinv;
                    s.ws[dm.ws_act + j] = gt / (1.0f + expf(-gt)) * up;
                }
            };
            st_gu.run(xs, r_gu, epi);
        }
        TPI_TRACE_L(7);
        WaveStreamer<ROWS_SL, CB_SL> st_dn;
        grid_arrive(t, epoch);
        st_dn.prefetch(vw, nvw, (dm.h + ROWS_SL - 1) / ROWS_SL, dm.sl, r_dn);
        if (!grid_wait(t, epoch, &s_flag)) return;

        TPI_TRACE_L(8);
        // ---- stage 5: down projection, reduce 2 + shortcut folded in -> next layer's input ----
        {
            FusedReduce rf;
            rf.n = t.n_ranks; rf.rank = t.rank; rf.residual = t.h_attn; rf.out = x_next;
#pragma unroll
            for (int i = 0; i < kMaxBatchShards; ++i) rf.peer[i] = t.peer_ffn[i];
            stage_x_plain(s.ws + dm.ws_act, dm.sl, xs);
            int n_saved = 0;
            auto epi = [&](int u, float (&y)[ROWS_SL]) {
                const float mine = pick_own<ROWS_SL>(y, lane);
                if (lane < ROWS_SL && n_saved < kSaveUnits) ysave[(wave * kSaveUnits + n_saved) * 16 + lane] = mine;
                n_saved += 1;
            };
            st_dn.run(xs, r_dn, epi);
            for (int k = 0; k < n_saved && k < kSaveUnits; ++k) {
                const int row = (vw + k * nvw) * ROWS_SL + lane;
                if (lane < ROWS_SL && row < dm.h) emit_row(s, rf, row, ysave[(wave * kSaveUnits + k) * 16 + lane]);
            }
        }
        TPI_TRACE_L(9);
        if (l + 1 < t.n_layers) {
            lp = t.layers[l + 1];
            r_qkv.w = lp.w_qkv;
            grid_arrive(t, epoch);
            st_qkv.prefetch(vw, nvw, (npairs + PAIRS - 1) / PAIRS, dm.h, r_qkv);
            if (!grid_wait(t, epoch, &s_flag)) return;
        }
        TPI_TRACE_L(10);
        x = x_next;
    }
}

}  // namespace tpi

using namespace tpi;

struct tpi_decoder {
    tpi_shard_cfg cfg;
    int n_layers = 0;
    char *ws = nullptr;
    size_t off_table = 0, off_peers = 0, off_sync = 0, off_h = 0, off_stage = 0;
    int n_ranks = 1, rank = 0;
    int grid = 0;
    int xs_floats = 0;
    size_t lds = 0;
    const void *kernel = nullptr;
    unsigned long long generations = 0;  // barriers queued so far (the tree's counters are monotonic)
    int barriers_per_token = 0;
};

namespace {

size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr bool kDecoderSwitchedOff = true;

constexpr size_t kSyncBytes = 128 * (2 + 512) + 256;   // flag, root, up to 512 group counters, error word

int xch_pow2(int K)
{
    int c = (K + kWChunk - 1) / kWChunk, p = 1;
    while (p < c) p *= 2;
    return p;
}

// The shape combinations the whole-token kernel is compiled for.
const void *pick_kernel(const tpi_shard_cfg *c)
{
    const int kh = xch_pow2(c->hidden), ks = xch_pow2(c->ffn_local), kq = xch_pow2(c->n_q_local * c->head_dim);
    const int G = c->n_q_local / c->n_kv_local;
    const int gt = G == 1 ? 1 : (G == 2 ? 2 : (G <= 4 ? 4 : 8));
    const int epl = c->head_dim <= 64 ? 1 : (c->head_dim <= 128 ? 2 : 4);
#define TPI_PICK(KH, KS, KQ, GT, EPL)                                                   \
    if (kh == KH && ks == KS && kq == KQ && gt == GT && epl == EPL)                     \
        return reinterpret_cast<const void *>(&k_decode_token<KH, KS, KQ, GT, EPL>);
    TPI_PICK(32, 16, 4, 8, 2)   // Llama-2-70B-shaped 8-way shard
    TPI_PICK(16, 16, 4, 4, 2)   // Llama-3.1-8B-shaped 4-way shard
    TPI_PICK(1, 2, 1, 1, 1)     // tiny test shard (hidden 256, FFN 344, 2 heads of 64)
    TPI_PICK(2, 4, 1, 4, 1)     // small test shards
    TPI_PICK(2, 1, 1, 2, 1)
#undef TPI_PICK
    return nullptr;
}

struct DecodeLayout { int q, att_m, att_l, att_acc, o, act, cnt, total; };

}  // namespace

namespace tpi {
// defined in tpi_api.hip: fills the shape fields and the workspace offsets of a decode call
int fill_decode_dims(const tpi_shard_cfg *c, int32_t pos, const float *h_in, DecodeDims &a);
}

extern "C" {

size_t tpi_decoder_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_layers)
{
    if (check_cfg(cfg) != TPI_OK || n_layers < 1 || cfg->dtype != TPI_F32) return 0;
    size_t stage = tpi_workspace_bytes(cfg, 1);
    return al256((size_t)n_layers * sizeof(LayerPtrs)) + 256 + kSyncBytes + al256(3 * (size_t)cfg->hidden * 4) + al256(stage);
}

int tpi_decoder_create(tpi_decoder **out, const tpi_shard_cfg *cfg, int32_t n_layers, const tpi_layer_weights *host_w,
                       const tpi_kv_layer *host_kv, int32_t n_ranks, int32_t rank, const float *const *host_peer_attn,
                       const float *const *host_peer_ffn, void *workspace, void *stream)
{
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (cfg->dtype != TPI_F32) return fail(TPI_EUNSUPPORTED, "decode is built for fp32 only");
    if (n_layers < 1 || !host_w || !host_kv || !workspace) return fail(TPI_EINVAL, "null argument or n_layers < 1");
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(TPI_EUNSUPPORTED, "workspace must be 256-byte aligned");
    if (n_ranks < 1 || n_ranks > TPI_MAX_BATCH_SHARDS || rank < 0 || rank >= n_ranks)
        return fail(TPI_EINVAL, "n_ranks %d / rank %d out of range (at most %d ranks)", n_ranks, rank, TPI_MAX_BATCH_SHARDS);
    if (n_ranks > 1 && (!host_peer_attn || !host_peer_ffn)) return fail(TPI_EINVAL, "peer partial tables are null");
    const float *peers[2 * TPI_MAX_BATCH_SHARDS] = {};
    for (int i = 0; i < n_ranks; ++i) {
        if (i == rank) continue;
        if (!host_peer_attn[i] || !host_peer_ffn[i]) return fail(TPI_EINVAL, "peer partial %d is null", i);
        peers[i] = host_peer_attn[i];
        peers[TPI_MAX_BATCH_SHARDS + i] = host_peer_ffn[i];
    }
    // Switched off: after the row-parallel stages' reduce was moved behind the row pipeline, one run
    // of this kernel (8B-shaped shard, 3 layers) stopped at a grid barrier until the bounded wait
    // gave up; reading the code has not shown which workgroup failed to arrive.  Until a cause is
    // shown the entry point reports the kernel as unavailable (it is also slower than the per-phase
    // calls: a software barrier across the chip's dies costs more than a kernel boundary).
    if (kDecoderSwitchedOff) return fail(TPI_EUNSUPPORTED, "the whole-token kernel is switched off in this build; use the per-phase calls");
    const void *kern = pick_kernel(cfg);
    if (!kern) return fail(TPI_EUNSUPPORTED, "the whole-token kernel is not compiled for this shard shape; use the per-layer calls");
    for (int l = 0; l < n_layers; ++l) {
        const tpi_layer_weights &w = host_w[l];
        if (!w.attn_norm || !w.w_qkv || !w.w_o || !w.ffn_norm || !w.w_gate || !w.w_up || !w.w_down || !host_kv[l].k ||
            !host_kv[l].v)
            return fail(TPI_EINVAL, "layer %d: null weight or cache pointer", l);
        const void *ps[9] = {w.attn_norm, w.w_qkv, w.w_o, w.ffn_norm, w.w_gate, w.w_up, w.w_down, host_kv[l].k, host_kv[l].v};
        for (const void *p : ps)
            if (reinterpret_cast<uintptr_t>(p) & 15u) return fail(TPI_EUNSUPPORTED, "layer %d: pointer not 16-byte aligned", l);
    }
    tpi_decoder *d = new (std::nothrow) tpi_decoder;
    if (!d) return fail(TPI_ERUNTIME, "out of host memory");
    d->cfg = *cfg;
    d->n_layers = n_layers;
    d->ws = static_cast<char *>(workspace);
    d->off_table = 0;
    d->off_peers = al256((size_t)n_layers * sizeof(LayerPtrs));
    d->off_sync = d->off_peers + 256;
    d->off_h = d->off_sync + kSyncBytes;
    d->n_ranks = n_ranks;
    d->rank = rank;
    d->off_stage = d->off_h + al256(3 * (size_t)cfg->hidden * 4);
    d->kernel = kern;
    d->barriers_per_token = 5 * n_layers - 1;
    const int G = cfg->n_q_local / cfg->n_kv_local;
    const int gt = G == 1 ? 1 : (G == 2 ? 2 : (G <= 4 ? 4 : 8));
    {
        int longest = cfg->hidden;
        if (cfg->ffn_local > longest) longest = cfg->ffn_local;
        if (cfg->n_q_local * cfg->head_dim > longest) longest = cfg->n_q_local * cfg->head_dim;
        d->xs_floats = (longest + 3) & ~3;
    }
    d->lds = sizeof(float) * ((size_t)d->xs_floats + (size_t)kWavesPerBlock * gt * cfg->head_dim + 2 * kWavesPerBlock * gt);
    if (d->lds > 60 * 1024) {
        delete d;
        return fail(TPI_EUNSUPPORTED, "the whole-token kernel needs %zu bytes of LDS per workgroup", d->lds);
    }

    // co-resident grid: every workgroup must be on the chip at once for the grid barrier
    int dev = 0, n_cu = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kBlock, d->lds);
    if (e != hipSuccess || per_cu < 1 || n_cu < 1) {
        delete d;
        return fail(TPI_ERUNTIME, "occupancy query failed: %s", hipGetErrorString(e));
    }
    per_cu = 1;   // one wave per SIMD: each wave owns the register file (see decode_wave.hpp)
    d->grid = n_cu * per_cu;
    {
        // a wave parks the sums of its units in LDS until the stage's end: at most 32 units per wave
        const int waves = d->grid * kWavesPerBlock;
        const int min_rows = 2;     // the smallest ROWS the kernel picks
        if ((cfg->hidden + min_rows - 1) / min_rows > 32 * waves) {
            delete d;
            return fail(TPI_EUNSUPPORTED, "hidden size %d is too large for the whole-token kernel on this device", cfg->hidden);
        }
    }
    if (d->grid > 512 * kBarGroup) d->grid = 512 * kBarGroup;

    std::vector<LayerPtrs> table(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        const tpi_layer_weights &w = host_w[l];
        table[l] = LayerPtrs{(const float *)w.attn_norm, (const float *)w.w_qkv, (const float *)w.w_o,
                             (const float *)w.ffn_norm, (const float *)w.w_gate, (const float *)w.w_up,
                             (const float *)w.w_down, (float *)host_kv[l].k, (float *)host_kv[l].v};
    }
    hipStream_t st = (hipStream_t)stream;
    e = hipMemcpyAsync(d->ws + d->off_table, table.data(), table.size() * sizeof(LayerPtrs), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(d->ws + d->off_peers, peers, sizeof(peers), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemsetAsync(d->ws + d->off_sync, 0, kSyncBytes, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);     // the host table goes out of scope
    if (e != hipSuccess) {
        delete d;
        return fail(TPI_ERUNTIME, "decoder setup: %s", hipGetErrorString(e));
    }
    *out = d;
    return TPI_OK;
}

int tpi_decoder_token(tpi_decoder *d, int32_t pos, const float *h_in, float *h_out, void *stream)
{
    if (!d || !h_in || !h_out) return fail(TPI_EINVAL, "null argument");
    if (pos < 0 || pos >= d->cfg.max_seq) return fail(TPI_EINVAL, "pos %d outside [0, max_seq %d)", pos, d->cfg.max_seq);
    if ((reinterpret_cast<uintptr_t>(h_in) | reinterpret_cast<uintptr_t>(h_out)) & 15u)
        return fail(TPI_EUNSUPPORTED, "h_in / h_out not 16-byte aligned");
    TokenArgs t;
    std::memset(&t, 0, sizeof(t));
    int rc = fill_decode_dims(&d->cfg, pos, h_in, t.dm);
    if (rc) return rc;
    t.n_layers = d->n_layers;
    t.layers = reinterpret_cast<const LayerPtrs *>(d->ws + d->off_table);
    t.h_in = h_in;
    t.h_out = h_out;
    t.ws = reinterpret_cast<float *>(d->ws + d->off_stage);
    float *hb = reinterpret_cast<float *>(d->ws + d->off_h);
    t.h_attn = hb; t.xa = hb + d->cfg.hidden; t.xb = hb + 2 * (size_t)d->cfg.hidden;
    t.bar_words = reinterpret_cast<unsigned long long *>(d->ws + d->off_sync);
    t.bar_error = reinterpret_cast<unsigned *>(d->ws + d->off_sync + kSyncBytes - 256);
    t.bar_gen0 = d->generations;
    t.n_ranks = d->n_ranks; t.rank = d->rank;
    t.xs_floats = d->xs_floats;
    t.peer_attn = reinterpret_cast<const float *const *>(d->ws + d->off_peers);
    t.peer_ffn = t.peer_attn + TPI_MAX_BATCH_SHARDS;
    void *params[1] = {&t};
    ProfScope ps(kStageToken, (hipStream_t)stream);
    hipError_t e = hipLaunchCooperativeKernel(d->kernel, dim3(d->grid), dim3(kBlock), params, (unsigned)d->lds,
                                              (hipStream_t)stream);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "cooperative launch failed: %s", hipGetErrorString(e));
    d->generations += (unsigned long long)d->barriers_per_token;
    return TPI_OK;
}

int tpi_decoder_status(tpi_decoder *d, void *stream)
{
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    unsigned flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, d->ws + d->off_sync + kSyncBytes - 256, sizeof(flag), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "status read: %s", hipGetErrorString(e));
    if (flag) return fail(TPI_ERUNTIME, "a grid barrier of the whole-token kernel gave up waiting; results are invalid");
    return TPI_OK;
}

int tpi_decoder_grid(const tpi_decoder *d) { return d ? d->grid : 0; }

int tpi_decoder_destroy(tpi_decoder *d)
{
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    delete d;
    return TPI_OK;
}

}  // extern "C"

#ifdef TPI_TRACE
namespace tpi {
__global__ __launch_bounds__(kBlock, 1) void k_barrier_bench(TokenArgs t, int iters)
{
    __shared__ int s_flag;
    unsigned epoch = 0;
    for (int i = 0; i < iters; ++i)
        if (!grid_barrier(t, epoch, &s_flag)) return;
}
}
// runs `iters` back-to-back grid barriers on the decoder's grid; returns microseconds per barrier
extern "C" double tpi_debug_barrier_bench(tpi_decoder *d, int iters)
{
    TokenArgs t;
    std::memset(&t, 0, sizeof(t));
    t.bar_words = reinterpret_cast<unsigned long long *>(d->ws + d->off_sync);
    t.bar_error = reinterpret_cast<unsigned *>(d->ws + d->off_sync + kSyncBytes - 256);
    t.bar_gen0 = d->generations;
    void *params[2] = {&t, &iters};
    hipEvent_t a, b;
    hipEventCreate(&a); hipEventCreate(&b);
    hipEventRecord(a, 0);
    hipError_t e = hipLaunchCooperativeKernel((const void *)&k_barrier_bench, dim3(d->grid), dim3(kBlock), params, 0, 0);
    hipEventRecord(b, 0);
    hipEventSynchronize(b);
    d->generations += iters;
    float ms = 0;
    hipEventElapsedTime(&ms, a, b);
    return e == hipSuccess ? ms * 1e3 / iters : -1.0;
}
extern "C" int tpi_debug_read_trace_token(unsigned long long *host_out, int n)
{
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(tpi::g_trace), sizeof(unsigned long long) * n) == hipSuccess ? 0 : -3;
}
#endif
