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
    unsigned long long *bar_count;     // grid barrier arrivals, monotonic over the decoder's life
    unsigned *bar_error;               // set when a barrier wait gave up
    unsigned long long bar_base;       // arrivals before this launch
    int n_ranks, rank;
    const float *const *peer_attn;     // device tables [n_ranks] of the peers' partial vectors
    const float *const *peer_ffn;      // (entry `rank` unused)
};

constexpr unsigned kSpinLimit = 1u << 22;   // polls before a barrier wait gives up (seconds of wall time)

// Barrier over the whole (co-resident) grid.  One thread per workgroup carries the release fence,
// the arrival, the bounded wait and the acquire fence; the workgroup barriers around it extend
// them to every wave.  Returns false when the wait gave up or another workgroup reported failure:
// the caller then leaves the kernel, so every wave reaches its exit whatever happens.
__device__ __forceinline__ bool grid_barrier(const TokenArgs &t, unsigned &epoch, int *s_flag)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        epoch += 1;
        const unsigned long long target = t.bar_base + (unsigned long long)epoch * gridDim.x;
        __threadfence();
        __hip_atomic_fetch_add(t.bar_count, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int ok = 1;
        unsigned spins = 0;
        while (__hip_atomic_load(t.bar_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
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

template <int KCH_H, int KCH_SL, int KCH_DQ, int GT, int EPL>
__global__ __launch_bounds__(kBlock) void k_decode_token(TokenArgs t)
{
    extern __shared__ float smem[];                 // attention: wave partials
    __shared__ float red[64];
    __shared__ int s_flag;
    constexpr int UB_H = KCH_H == 1 ? 1 : 2, UB_SL = KCH_SL == 1 ? 1 : 2, UB_DQ = KCH_DQ == 1 ? 1 : 2;
    constexpr int PAIRS = KCH_H == 1 ? 4 : 2, COLS = PAIRS;
    constexpr int ROWS_DQ = KCH_DQ == 1 ? 8 : 4, ROWS_SL = KCH_SL == 1 ? 8 : 4;

    const int vwg = blockIdx.x, nvwg = gridDim.x;
    unsigned epoch = 0;
    DecodeDims dm = t.dm;
    const int G = dm.nq / dm.nkv;
    const int n_ht = (G + GT - 1) / GT;
    const int n_attn_units = dm.nkv * n_ht * dm.n_splits;
    const float *x = t.h_in;

    for (int l = 0; l < t.n_layers; ++l) {
        const LayerPtrs lp = t.layers[l];
        ShardView s;
        s.attn_norm = lp.attn_norm; s.w_qkv = lp.w_qkv; s.w_o = lp.w_o; s.ffn_norm = lp.ffn_norm;
        s.w_gate = lp.w_gate; s.w_up = lp.w_up; s.w_down = lp.w_down;
        s.k = lp.k; s.v = lp.v; s.partial_out = nullptr; s.ws = t.ws;
        float *x_next = (l == t.n_layers - 1) ? t.h_out : ((l & 1) ? t.xb : t.xa);

        dm.h_in = x;
        stage_qkv<PAIRS, KCH_H, UB_H>(dm, s, vwg, nvwg, red);
        if (!grid_barrier(t, epoch, &s_flag)) return;

        for (int u = vwg; u < n_attn_units; u += nvwg) {
            int split = u % dm.n_splits, gh = u / dm.n_splits;
            stage_attn<GT, EPL>(dm, s, split, gh / n_ht, gh % n_ht, smem);
            __syncthreads();                          // LDS of the stage is reused by the next unit
        }
        if (!grid_barrier(t, epoch, &s_flag)) return;

        {
            FusedReduce rf;
            rf.n = t.n_ranks; rf.rank = t.rank; rf.residual = x; rf.out = t.h_attn;
            rf.peer = t.peer_attn;
            stage_oproj<ROWS_DQ, KCH_DQ, UB_DQ>(dm, s, vwg, nvwg, red, rf);
        }
        if (!grid_barrier(t, epoch, &s_flag)) return;

        dm.h_in = t.h_attn;
        stage_gate_up<COLS, KCH_H, UB_H>(dm, s, vwg, nvwg, red);
        if (!grid_barrier(t, epoch, &s_flag)) return;

        {
            FusedReduce rf;
            rf.n = t.n_ranks; rf.rank = t.rank; rf.residual = t.h_attn; rf.out = x_next;
            rf.peer = t.peer_ffn;
            stage_down<ROWS_SL, KCH_SL, UB_SL>(dm, s, vwg, nvwg, red, rf);
        }
        if (l + 1 < t.n_layers && !grid_barrier(t, epoch, &s_flag)) return;
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
    size_t lds = 0;
    const void *kernel = nullptr;
    unsigned long long arrivals = 0;     // barrier arrivals queued so far
    int barriers_per_token = 0;
};

namespace {

size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

int kch_pow2(int K)
{
    int c = (K + kChunk - 1) / kChunk, p = 1;
    while (p < c) p *= 2;
    return p;
}

// The shape combinations the whole-token kernel is compiled for.
const void *pick_kernel(const tpi_shard_cfg *c)
{
    const int kh = kch_pow2(c->hidden), ks = kch_pow2(c->ffn_local), kq = kch_pow2(c->n_q_local * c->head_dim);
    const int G = c->n_q_local / c->n_kv_local;
    const int gt = G == 1 ? 1 : (G == 2 ? 2 : (G <= 4 ? 4 : 8));
    const int epl = c->head_dim <= 64 ? 1 : (c->head_dim <= 128 ? 2 : 4);
#define TPI_PICK(KH, KS, KQ, GT, EPL)                                                   \
    if (kh == KH && ks == KS && kq == KQ && gt == GT && epl == EPL)                     \
        return reinterpret_cast<const void *>(&k_decode_token<KH, KS, KQ, GT, EPL>);
    TPI_PICK(8, 4, 1, 8, 2)     // Llama-2-70B-shaped 8-way shard
    TPI_PICK(4, 4, 1, 4, 2)     // Llama-3.1-8B-shaped 4-way shard
    TPI_PICK(1, 1, 1, 1, 1)     // tiny test shard
    TPI_PICK(1, 1, 1, 2, 1)
    TPI_PICK(1, 1, 1, 4, 1)
    TPI_PICK(2, 1, 1, 4, 2)
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
    return al256((size_t)n_layers * sizeof(LayerPtrs)) + 256 + 256 + al256(3 * (size_t)cfg->hidden * 4) + al256(stage);
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
    d->off_h = d->off_sync + 256;
    d->n_ranks = n_ranks;
    d->rank = rank;
    d->off_stage = d->off_h + al256(3 * (size_t)cfg->hidden * 4);
    d->kernel = kern;
    d->barriers_per_token = 5 * n_layers - 1;
    const int G = cfg->n_q_local / cfg->n_kv_local;
    const int gt = G == 1 ? 1 : (G == 2 ? 2 : (G <= 4 ? 4 : 8));
    d->lds = sizeof(float) * ((size_t)kWavesPerBlock * gt * cfg->head_dim + 2 * kWavesPerBlock * gt);

    // co-resident grid: every workgroup must be on the chip at once for the grid barrier
    int dev = 0, n_cu = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kBlock, d->lds);
    if (e != hipSuccess || per_cu < 1 || n_cu < 1) {
        delete d;
        return fail(TPI_ERUNTIME, "occupancy query failed: %s", hipGetErrorString(e));
    }
    if (per_cu > 2) per_cu = 2;
    d->grid = n_cu * per_cu;

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
    if (e == hipSuccess) e = hipMemsetAsync(d->ws + d->off_sync, 0, 256, st);
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
    t.bar_count = reinterpret_cast<unsigned long long *>(d->ws + d->off_sync);
    t.bar_error = reinterpret_cast<unsigned *>(d->ws + d->off_sync + 64);
    t.bar_base = d->arrivals;
    t.n_ranks = d->n_ranks; t.rank = d->rank;
    t.peer_attn = reinterpret_cast<const float *const *>(d->ws + d->off_peers);
    t.peer_ffn = t.peer_attn + TPI_MAX_BATCH_SHARDS;
    void *params[1] = {&t};
    ProfScope ps(kStageToken, (hipStream_t)stream);
    hipError_t e = hipLaunchCooperativeKernel(d->kernel, dim3(d->grid), dim3(kBlock), params, (unsigned)d->lds,
                                              (hipStream_t)stream);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "cooperative launch failed: %s", hipGetErrorString(e));
    d->arrivals += (unsigned long long)d->barriers_per_token * d->grid;
    return TPI_OK;
}

int tpi_decoder_status(tpi_decoder *d, void *stream)
{
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    unsigned flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, d->ws + d->off_sync + 64, sizeof(flag), hipMemcpyDeviceToHost, (hipStream_t)stream);
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
