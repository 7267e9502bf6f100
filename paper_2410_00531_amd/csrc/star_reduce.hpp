#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tpi {

constexpr int kMaxReduceRanks = 64;   // == TPI_MAX_REDUCE_RANKS

struct ReduceArgs {
    const float *p[kMaxReduceRanks];
    const float *residual;   // nullable
    float *out;
    unsigned short *out_bf16;   // nullable: result rounded to bf16 (nearest even)
    int64_t len;
    int n;
    int vec_ok;              // all pointers 16-byte aligned
};

hipError_t launch_star_reduce(const ReduceArgs &a, hipStream_t st);

}  // namespace tpi
