// bf16 prefill path (matrix cores): host interface used by the entry points.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/tpi.h"

namespace tpi {

size_t prefill_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_tokens);
void prefill_set_concurrency(int n);

// Arguments are already validated (non-null, ranges, dtype == TPI_BF16).
int prefill_launch(const tpi_shard_cfg *cfg, const tpi_layer_weights *w, const tpi_kv_layer *kv, int32_t pos0,
                   int32_t n_tokens, int phase, const void *h_in, float *partial_out, void *workspace,
                   hipStream_t stream);

}  // namespace tpi
