// tpi_decoder_*: the whole-token decode of one device's shard (Alg. 2, the worker's loop) as ONE persistent
// launch.  This build has no such kernel: the entry points keep their place in the ABI, check their arguments
// and report TPI_EUNSUPPORTED.
//
// What stood here, and why it is gone.  A co-resident grid ran all stages of all layers of a token, its stages
// separated by a software barrier (counters per die, a root counter, bounded spins).  It was slower than the
// per-stage kernels (11-12 ms against 7.3 ms per token on the 70B-shaped shard), and one run ended with a
// bounded barrier wait giving up for a reason that reading the code did not show; it was switched off, and
// its device code has now been removed rather than shipped unexplained.  Measurements on this chip say the
// arrangement cannot win: a chip-wide hand-over inside a kernel -- results written through to memory, a
// two-level counter tree, a flag per die, the results read back -- takes 3.6-4.2 us from the last workgroup's
// result to the first use of the next stage's input, on top of 4.5-6 us in which the workgroups of a stage
// finish one after the other, while a kernel boundary costs 4.5 us all in; weights requested ahead across the
// hand-over (33 MB in flight) hide about half of it (tpi_probe_handover; bench.py's handover_probe object).
// The per-phase entry points cover every shape.
#include "../../include/tpi.h"
#include "host_util.hpp"

using tpi::fail;

struct tpi_decoder {
    int unused;
};

extern "C" {

size_t tpi_decoder_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_layers)
{
    if (tpi::check_cfg(cfg) != TPI_OK || n_layers < 1 || cfg->dtype != TPI_F32) return 0;
    return 256;   // nothing is kept there; a non-zero size keeps callers' allocation code on one path
}

int tpi_decoder_create(tpi_decoder **out, const tpi_shard_cfg *cfg, int32_t n_layers, const tpi_layer_weights *host_w,
                       const tpi_kv_layer *host_kv, int32_t n_ranks, int32_t rank, const float *const *host_peer_attn,
                       const float *const *host_peer_ffn, void *workspace, void *stream)
{
    (void)stream;
    if (!out) return fail(TPI_EINVAL, "out is null");
    *out = nullptr;
    int rc = tpi::check_cfg(cfg);
    if (rc) return rc;
    if (cfg->dtype != TPI_F32) return fail(TPI_EUNSUPPORTED, "decode is built for fp32 only");
    if (n_layers < 1 || !host_w || !host_kv || !workspace) return fail(TPI_EINVAL, "null argument or n_layers < 1");
    if (n_ranks < 1 || n_ranks > TPI_MAX_BATCH_SHARDS || rank < 0 || rank >= n_ranks)
        return fail(TPI_EINVAL, "n_ranks %d / rank %d out of range (at most %d ranks)", n_ranks, rank, TPI_MAX_BATCH_SHARDS);
    if (n_ranks > 1 && (!host_peer_attn || !host_peer_ffn)) return fail(TPI_EINVAL, "peer partial tables are null");
    return fail(TPI_EUNSUPPORTED, "the whole-token kernel is switched off in this build (no such kernel is compiled in); "
                                  "use the per-phase calls");
}

int tpi_decoder_token(tpi_decoder *d, int32_t pos, const float *h_in, float *h_out, void *stream)
{
    (void)pos; (void)h_in; (void)h_out; (void)stream;
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    return fail(TPI_EUNSUPPORTED, "the whole-token kernel is switched off in this build");
}

int tpi_decoder_status(tpi_decoder *d, void *stream)
{
    (void)stream;
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    return fail(TPI_EUNSUPPORTED, "the whole-token kernel is switched off in this build");
}

int tpi_decoder_grid(const tpi_decoder *d) { (void)d; return 0; }

int tpi_decoder_destroy(tpi_decoder *d)
{
    if (!d) return fail(TPI_EINVAL, "decoder is null");
    return TPI_OK;     // create never hands one out
}

}  // extern "C"
