// Host-side helpers shared by the entry points.
#pragma once
#include "../../include/tpi.h"

namespace tpi {

// Stores a printf-style message for tpi_last_error() and returns `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// Validates a shard shape; TPI_OK or the failing status (message stored).
int check_cfg(const tpi_shard_cfg *c);

}  // namespace tpi
