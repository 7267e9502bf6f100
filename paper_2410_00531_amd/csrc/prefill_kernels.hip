// bf16 prefill path -- not built yet: the entry point reports TPI_EUNSUPPORTED.
#include "prefill.hpp"

#include "host_util.hpp"

namespace tpi {

size_t prefill_workspace_bytes(const tpi_shard_cfg *, int32_t) { return 0; }

int prefill_launch(const tpi_shard_cfg *, const tpi_layer_weights *, const tpi_kv_layer *, int32_t, int32_t, int,
                   const void *, float *, void *, hipStream_t)
{
    return fail(TPI_EUNSUPPORTED, "prefill kernels are not built in this version");
}

}  // namespace tpi
