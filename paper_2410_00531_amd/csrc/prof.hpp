// Optional per-stage kernel timer: HIP events around every launch of ONE
// chosen stage, on the stream the kernel is launched on.  Off by default; a
// measurement aid for benchmarks, not thread-safe.
#pragma once
#include <hip/hip_runtime.h>

namespace tpi {

enum Stage { kStageNone = 0, kStageQkv = 1, kStageAttn = 2, kStageOproj = 3, kStageGateUp = 4, kStageDown = 5,
             kStageReduce = 6, kStagePrefillGemm = 7, kStageToken = 8, kStageCount };

void prof_begin(int stage, hipStream_t st);
void prof_end(int stage, hipStream_t st);

struct ProfScope {
    int stage;
    hipStream_t st;
    ProfScope(int s, hipStream_t t) : stage(s), st(t) { prof_begin(stage, st); }
    ~ProfScope() { prof_end(stage, st); }
};

}  // namespace tpi
