// extern "C" entry points of libtpi: argument checks and launches only.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/tpi.h"
#include "decode_args.hpp"
#include "decode_stages.hpp"
#include "host_util.hpp"
#include "prefill.hpp"
#include "star_reduce.hpp"

static_assert(TPI_MAX_BATCH_SHARDS == tpi::kMaxBatchShards, "limits out of sync");
static_assert(TPI_ATTN_MAX_SPLITS == tpi::kAttnMaxSplits, "limits out of sync");
static_assert(TPI_MAX_REDUCE_RANKS == tpi::kMaxReduceRanks, "limits out of sync");
static_assert(TPI_MAX_HEAD_DIM == 2 * tpi::kRopeHalf, "limits out of sync");

// Workspace of tpi_shard_layer_decode_static: device memory that belongs to the library's code object, one copy
// per GPU, alive until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// address the kernels get is asked for once per device (scratch_of_current_device).
constexpr size_t kStaticScratchBytes = TPI_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace tpi {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int round4(int x) { return (x + 3) & ~3; }

// Shape checks shared by every compute entry point.
int check_cfg(const tpi_shard_cfg *c)
{
    if (!c) return fail(TPI_EINVAL, "cfg is null");
    if (c->hidden < 1 || c->n_q_local < 1 || c->n_kv_local < 1 || c->head_dim < 2 || c->ffn_local < 1 ||
        c->max_seq < 1)
        return fail(TPI_EINVAL, "cfg: sizes must be positive (hidden %d, n_q %d, n_kv %d, head_dim %d, ffn %d, max_seq %d)",
                    c->hidden, c->n_q_local, c->n_kv_local, c->head_dim, c->ffn_local, c->max_seq);
    if (c->head_dim % 2) return fail(TPI_EINVAL, "cfg: head_dim %d is odd (rotary pairs need an even size)", c->head_dim);
    if (c->n_q_local % c->n_kv_local)
        return fail(TPI_EINVAL, "cfg: n_q_local %d is not a multiple of n_kv_local %d", c->n_q_local, c->n_kv_local);
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return fail(TPI_EINVAL, "cfg: rms_eps < 0 or rope_base <= 0");
    if (c->dtype != TPI_F32 && c->dtype != TPI_BF16) return fail(TPI_EINVAL, "cfg: unknown dtype %d", c->dtype);
    const int vec = (c->dtype == TPI_BF16) ? 8 : 4;      // elements per 16-byte load
    if (c->hidden % vec || c->ffn_local % vec || c->head_dim % vec)
        return fail(TPI_EUNSUPPORTED, "cfg: hidden, ffn_local and head_dim must be multiples of %d", vec);
    if (c->head_dim > TPI_MAX_HEAD_DIM) return fail(TPI_EUNSUPPORTED, "cfg: head_dim %d > %d", c->head_dim, TPI_MAX_HEAD_DIM);
    if ((int64_t)c->n_q_local * c->head_dim > (1 << 20) || c->hidden > (1 << 20) || c->ffn_local > (1 << 24))
        return fail(TPI_EUNSUPPORTED, "cfg: size beyond what this build indexes");
    return TPI_OK;
}

// Workspace layout of a decode call (offsets in floats).
static void decode_layout(const tpi_shard_cfg *c, DecodeDims &a)
{
    int off = 0;
    a.ws_q = off;        off += round4(c->n_q_local * c->head_dim);
    a.ws_att_m = off;    off += round4(c->n_q_local * kAttnMaxSplits);
    a.ws_att_l = off;    off += round4(c->n_q_local * kAttnMaxSplits);
    a.ws_att_acc = off;  off += round4(c->n_q_local * kAttnMaxSplits * c->head_dim);
    a.ws_o = off;        off += round4(c->n_q_local * c->head_dim);
    a.ws_act = off;      off += round4(c->ffn_local);
    a.ws_cnt = off;      off += round4(c->n_kv_local);
    a.ws_total = off;
}

int fill_decode_dims(const tpi_shard_cfg *c, int32_t pos, const float *h_in, DecodeDims &a)
{
    a.h = c->hidden; a.nq = c->n_q_local; a.nkv = c->n_kv_local; a.d = c->head_dim; a.sl = c->ffn_local;
    a.max_seq = c->max_seq; a.pos = pos; a.eps = c->rms_eps;
    a.log2_base = std::log2((double)c->rope_base);
    a.h_in = h_in;
    // split slots 0..pos into at most kAttnMaxSplits chunks of whole 64-slot tiles
    int n_valid = pos + 1;
    int per = (n_valid + kAttnMaxSplits - 1) / kAttnMaxSplits;
    a.chunk_len = ((per + 63) / 64) * 64;
    a.n_splits = (n_valid + a.chunk_len - 1) / a.chunk_len;
    decode_layout(c, a);
    return TPI_OK;
}

// rf_*: non-null host_peers folds the star reduce into the phase's last stage (single shard only)
static int decode_common(const tpi_shard_cfg *cfg, int32_t n_shards, const tpi_layer_weights *w,
                         const tpi_kv_layer *kv, int32_t pos, int phase, const float *h_in,
                         float *const *partial_out, void *const *workspace, void *stream,
                         int32_t rf_n = 0, int32_t rf_rank = 0, const float *const *rf_peers = nullptr,
                         float *rf_out = nullptr, bool rf_all = false)
{
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (phase != TPI_PHASE_ATTN && phase != TPI_PHASE_FFN) return fail(TPI_EINVAL, "unknown phase %d", phase);
    if (n_shards < 1) return fail(TPI_EINVAL, "n_shards %d < 1", n_shards);
    if (n_shards > TPI_MAX_BATCH_SHARDS) return fail(TPI_EINVAL, "n_shards %d > %d", n_shards, TPI_MAX_BATCH_SHARDS);
    if (!w || !h_in || (!partial_out && !rf_all) || !workspace) return fail(TPI_EINVAL, "null argument");
    if (phase == TPI_PHASE_ATTN && !kv) return fail(TPI_EINVAL, "kv is null in the attention phase");
    if (pos < 0 || pos >= cfg->max_seq) return fail(TPI_EINVAL, "pos %d outside [0, max_seq %d)", pos, cfg->max_seq);
    if (cfg->dtype != TPI_F32) return fail(TPI_EUNSUPPORTED, "decode is built for fp32 only");
    if (!aligned16(h_in)) return fail(TPI_EUNSUPPORTED, "h_in is not 16-byte aligned");
    // each stage keeps its thread's slice of the input vector in registers: at most 16 chunks of 1024 floats
    {
        int64_t longest = cfg->hidden;
        if (cfg->ffn_local > longest) longest = cfg->ffn_local;
        if ((int64_t)cfg->n_q_local * cfg->head_dim > longest) longest = (int64_t)cfg->n_q_local * cfg->head_dim;
        if (longest > 16 * 1024)
            return fail(TPI_EUNSUPPORTED, "rows of %lld floats: the GEMV stages are built for at most 16384", (long long)longest);
    }

    // the attention grid has one y index per (KV head, tile of its query heads)
    if (phase == TPI_PHASE_ATTN && (int64_t)cfg->n_kv_local * ((cfg->n_q_local / cfg->n_kv_local + 7) / 8) > 65535)
        return fail(TPI_EUNSUPPORTED, "n_kv_local %d: more head tiles than the attention grid can index", cfg->n_kv_local);

    DecodeArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_decode_dims(cfg, pos, h_in, a);
    if (rf_all) {
        // every rank's partial is formed by this call: nothing to read from peers
        if (!rf_out) return fail(TPI_EINVAL, "null argument");
        if (!aligned16(rf_out)) return fail(TPI_EUNSUPPORTED, "out is not 16-byte aligned");
        // a workgroup writes its rows of `out` while others still read h_in (as the stage's input or as the shortcut)
        {
            const uintptr_t o = reinterpret_cast<uintptr_t>(rf_out), x = reinterpret_cast<uintptr_t>(h_in);
            const uintptr_t len = (uintptr_t)cfg->hidden * sizeof(float);
            if (o < x + len && x < o + len) return fail(TPI_EINVAL, "out overlaps h_in");
        }
        a.rf.n = n_shards; a.rf.rank = 0; a.rf.all = 1; a.rf.residual = h_in; a.rf.out = rf_out;
    } else if (rf_n > 0) {
        if (rf_n > TPI_MAX_BATCH_SHARDS || rf_rank < 0 || rf_rank >= rf_n)
            return fail(TPI_EINVAL, "n_ranks %d / rank %d out of range (at most %d ranks)", rf_n, rf_rank, TPI_MAX_BATCH_SHARDS);
        if (!rf_out || (rf_n > 1 && !rf_peers)) return fail(TPI_EINVAL, "null argument");
        if (!aligned16(rf_out)) return fail(TPI_EUNSUPPORTED, "out is not 16-byte aligned");
        a.rf.n = rf_n; a.rf.rank = rf_rank; a.rf.residual = h_in; a.rf.out = rf_out;
        for (int i = 0; i < rf_n; ++i) {
            if (i == rf_rank) continue;
            if (!rf_peers[i]) return fail(TPI_EINVAL, "partial of rank %d is null", i);
            a.rf.peer[i] = rf_peers[i];
        }
    }
    for (int r = 0; r < n_shards; ++r) {
        const tpi_layer_weights &lw = w[r];
        ShardView &s = a.s[r];
        const bool stores_partial = rf_n == 0 && !rf_all;
        if ((stores_partial && !partial_out[r]) || !workspace[r]) return fail(TPI_EINVAL, "shard %d: null output or workspace", r);
        if (phase == TPI_PHASE_ATTN) {
            if (!lw.attn_norm || !lw.w_qkv || !lw.w_o || !kv[r].k || !kv[r].v)
                return fail(TPI_EINVAL, "shard %d: null attention weight or cache pointer", r);
            if (!aligned16(lw.attn_norm) || !aligned16(lw.w_qkv) || !aligned16(lw.w_o) || !aligned16(kv[r].k) ||
                !aligned16(kv[r].v))
                return fail(TPI_EUNSUPPORTED, "shard %d: pointer not 16-byte aligned", r);
        } else {
            if (!lw.ffn_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
                return fail(TPI_EINVAL, "shard %d: null FFN weight pointer", r);
            if (!aligned16(lw.ffn_norm) || !aligned16(lw.w_gate) || !aligned16(lw.w_up) || !aligned16(lw.w_down))
                return fail(TPI_EUNSUPPORTED, "shard %d: pointer not 16-byte aligned", r);
        }
        if ((stores_partial && !aligned16(partial_out[r])) || !aligned16(workspace[r]))
            return fail(TPI_EUNSUPPORTED, "shard %d: output or workspace not 16-byte aligned", r);
        s.attn_norm = (const float *)lw.attn_norm; s.w_qkv = (const float *)lw.w_qkv; s.w_o = (const float *)lw.w_o;
        s.ffn_norm = (const float *)lw.ffn_norm; s.w_gate = (const float *)lw.w_gate; s.w_up = (const float *)lw.w_up;
        s.w_down = (const float *)lw.w_down;
        s.k = kv ? (float *)kv[r].k : nullptr;
        s.v = kv ? (float *)kv[r].v : nullptr;
        s.partial_out = stores_partial ? partial_out[r] : nullptr;
        s.ws = (float *)workspace[r];
    }
    hipError_t e = (phase == TPI_PHASE_ATTN) ? launch_attn_phase(a, n_shards, (hipStream_t)stream)
                                             : launch_ffn_phase(a, n_shards, (hipStream_t)stream);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}

// Device address of `scratch` on the current device, asked for on the first call per device.
static int scratch_of_current_device(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(TPI_EUNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lk(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(TPI_ERUNTIME, "hipGetSymbolAddress: %s", hipGetErrorString(e));
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return TPI_OK;
}

}  // namespace tpi

using namespace tpi;

extern "C" {

const char *tpi_last_error(void) { return g_err; }

int tpi_abi_version(void) { return 1; }

size_t tpi_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_tokens)
{
    if (check_cfg(cfg) != TPI_OK || n_tokens < 1) return 0;
    if (cfg->dtype == TPI_BF16) return prefill_workspace_bytes(cfg, n_tokens);
    DecodeArgs a;
    decode_layout(cfg, a);
    return (size_t)a.ws_total * sizeof(float);
}

int tpi_shard_layer_decode(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w, const tpi_kv_layer *host_kv,
                           int32_t pos, int phase, const float *h_in, float *partial_out, void *workspace,
                           void *stream)
{
    float *po[1] = {partial_out};
    void *ws[1] = {workspace};
    return decode_common(cfg, 1, host_w, host_kv, pos, phase, h_in, po, ws, stream);
}

int tpi_shard_layer_decode_static(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                                  const tpi_kv_layer *host_kv, int32_t pos, int phase, const float *h_in,
                                  float *partial_out, void *stream)
{
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (cfg->dtype != TPI_F32) return fail(TPI_EUNSUPPORTED, "decode is built for fp32 only");
    DecodeArgs a;
    decode_layout(cfg, a);
    const size_t need = (size_t)a.ws_total * sizeof(float);
    if (need > kStaticScratchBytes)
        return fail(TPI_EUNSUPPORTED, "this shard needs %zu bytes of workspace, the built-in one holds %zu: "
                    "use tpi_shard_layer_decode with a workspace of the caller", need, kStaticScratchBytes);
    void *ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc) return rc;
    float *po[1] = {partial_out};
    void *wsv[1] = {ws};
    return decode_common(cfg, 1, host_w, host_kv, pos, phase, h_in, po, wsv, stream);
}

int tpi_shard_layer_decode_reduce(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                                  const tpi_kv_layer *host_kv, int32_t pos, int phase, const float *h_in,
                                  int32_t n_ranks, int32_t rank, const float *const *host_partials, float *out,
                                  void *workspace, void *stream)
{
    if (n_ranks < 1) return fail(TPI_EINVAL, "n_ranks %d < 1", n_ranks);
    float *po[1] = {nullptr};
    void *ws[1] = {workspace};
    return decode_common(cfg, 1, host_w, host_kv, pos, phase, h_in, po, ws, stream, n_ranks, rank, host_partials, out);
}

int tpi_shards_layer_decode(const tpi_shard_cfg *cfg, int32_t n_shards, const tpi_layer_weights *host_w,
                            const tpi_kv_layer *host_kv, int32_t pos, int phase, const float *h_in,
                            float *const *host_partial_out, void *const *host_workspace, void *stream)
{
    return decode_common(cfg, n_shards, host_w, host_kv, pos, phase, h_in, host_partial_out, host_workspace, stream);
}

int tpi_shards_layer_decode_reduce(const tpi_shard_cfg *cfg, int32_t n_shards, const tpi_layer_weights *host_w,
                                   const tpi_kv_layer *host_kv, int32_t pos, int phase, const float *h_in, float *out,
                                   void *const *host_workspace, void *stream)
{
    return decode_common(cfg, n_shards, host_w, host_kv, pos, phase, h_in, nullptr, host_workspace, stream, 0, 0, nullptr,
                         out, true);
}

static int star_reduce_common(const float *const *host_partials, int32_t n, int64_t len, const float *residual,
                              float *out, void *out_bf16, void *stream)
{
    if (!host_partials || !out) return fail(TPI_EINVAL, "null argument");
    if (n < 1) return fail(TPI_EINVAL, "n %d < 1", n);
    if (len < 0) return fail(TPI_EINVAL, "len %lld < 0", (long long)len);
    if (n > TPI_MAX_REDUCE_RANKS) return fail(TPI_EUNSUPPORTED, "n %d > %d", n, TPI_MAX_REDUCE_RANKS);
    ReduceArgs a;
    std::memset(&a, 0, sizeof(a));
    bool al = aligned16(out) && (!residual || aligned16(residual)) &&
              (!out_bf16 || (reinterpret_cast<uintptr_t>(out_bf16) & 7u) == 0);
    for (int r = 0; r < n; ++r) {
        if (!host_partials[r]) return fail(TPI_EINVAL, "partial %d is null", r);
        a.p[r] = host_partials[r];
        al = al && aligned16(host_partials[r]);
    }
    a.residual = residual; a.out = out; a.out_bf16 = (unsigned short *)out_bf16; a.len = len; a.n = n;
    a.vec_ok = al ? 1 : 0;
    hipError_t e = launch_star_reduce(a, (hipStream_t)stream);
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}

int tpi_star_reduce(const float *const *host_partials, int32_t n, int64_t len, const float *residual, float *out,
                    void *stream)
{
    return star_reduce_common(host_partials, n, len, residual, out, nullptr, stream);
}

int tpi_star_reduce_bf16(const float *const *host_partials, int32_t n, int64_t len, const float *residual, float *out,
                         void *out_bf16, void *stream)
{
    if (!out_bf16) return fail(TPI_EINVAL, "out_bf16 is null");
    return star_reduce_common(host_partials, n, len, residual, out, out_bf16, stream);
}

static int prefill_common(const tpi_shard_cfg *cfg, int32_t n_shards, const tpi_layer_weights *host_w,
                          const tpi_kv_layer *host_kv, int32_t pos0, int32_t n_tokens, int phase, const void *h_in,
                          float *const *partial_out, void *const *workspace, void *stream)
{
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (phase != TPI_PHASE_ATTN && phase != TPI_PHASE_FFN) return fail(TPI_EINVAL, "unknown phase %d", phase);
    if (n_shards < 1) return fail(TPI_EINVAL, "n_shards %d < 1", n_shards);
    if (n_shards > TPI_MAX_BATCH_SHARDS) return fail(TPI_EINVAL, "n_shards %d > %d", n_shards, TPI_MAX_BATCH_SHARDS);
    if (!host_w || !h_in || !partial_out || !workspace) return fail(TPI_EINVAL, "null argument");
    if (phase == TPI_PHASE_ATTN && !host_kv) return fail(TPI_EINVAL, "kv is null in the attention phase");
    if (n_tokens < 1) return fail(TPI_EINVAL, "n_tokens %d < 1", n_tokens);
    if (pos0 < 0 || (int64_t)pos0 + n_tokens > cfg->max_seq)
        return fail(TPI_EINVAL, "positions %d..%lld outside [0, max_seq %d)", pos0, (long long)pos0 + n_tokens - 1,
                    cfg->max_seq);
    if (cfg->dtype != TPI_BF16) return fail(TPI_EUNSUPPORTED, "prefill is built for bf16 only");
    return prefill_launch(cfg, n_shards, host_w, host_kv, pos0, n_tokens, phase, h_in, partial_out, workspace,
                          (hipStream_t)stream);
}

int tpi_shard_layer_prefill(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w, const tpi_kv_layer *host_kv,
                            int32_t pos0, int32_t n_tokens, int phase, const void *h_in, float *partial_out,
                            void *workspace, void *stream)
{
    float *po[1] = {partial_out};
    void *ws[1] = {workspace};
    return prefill_common(cfg, 1, host_w, host_kv, pos0, n_tokens, phase, h_in, po, ws, stream);
}

int tpi_shards_layer_prefill(const tpi_shard_cfg *cfg, int32_t n_shards, const tpi_layer_weights *host_w,
                             const tpi_kv_layer *host_kv, int32_t pos0, int32_t n_tokens, int phase, const void *h_in,
                             float *const *host_partial_out, void *const *host_workspace, void *stream)
{
    return prefill_common(cfg, n_shards, host_w, host_kv, pos0, n_tokens, phase, h_in, host_partial_out, host_workspace,
                          stream);
}

int tpi_probe_gemm_loop(int32_t leave_out, int32_t reps, tpi_gemm_probe_result *host_out, void *stream)
{
    if (!host_out) return fail(TPI_EINVAL, "host_out is null");
    if (leave_out < 0 || leave_out > 6) return fail(TPI_EINVAL, "leave_out %d outside [0, 6]", leave_out);
    if (reps < 1 || reps > 1000) return fail(TPI_EINVAL, "reps %d outside [1, 1000]", reps);
    return prefill_probe_gemm_loop(leave_out, reps, host_out, (hipStream_t)stream);
}

int tpi_set_prefill_concurrency(int32_t n_calls)
{
    if (n_calls < 1 || n_calls > TPI_MAX_BATCH_SHARDS)
        return fail(TPI_EINVAL, "n_calls %d outside [1, %d]", n_calls, TPI_MAX_BATCH_SHARDS);
    prefill_set_concurrency(n_calls);
    return TPI_OK;
}

}  // extern "C"
