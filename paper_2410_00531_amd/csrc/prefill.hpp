// bf16 prefill path (matrix cores): host interface used by the entry points.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/tpi.h"

namespace tpi {

size_t prefill_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_tokens);
void prefill_set_concurrency(int n);

// n_shards shards of one layer phase (arrays of n_shards entries; kv may be null in the FFN phase).  The
// configuration, token range, phase and h_in are already validated; the per-shard pointers are checked here.
int prefill_launch(const tpi_shard_cfg *cfg, int n_shards, const tpi_layer_weights *w, const tpi_kv_layer *kv, int32_t pos0,
                   int32_t n_tokens, int phase, const void *h_in, float *const *partial_out, void *const *workspace,
                   hipStream_t stream);

// tpi_probe_gemm_loop: leave_out in [0, 6], reps >= 1 and out non-null are already checked.
int prefill_probe_gemm_loop(int leave_out, int reps, tpi_gemm_probe_result *out, hipStream_t stream);

}  // namespace tpi
