// Kernel argument block of the decode stages (passed by value).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tpi {

constexpr int kMaxBatchShards = 16;   // == TPI_MAX_BATCH_SHARDS
constexpr int kAttnMaxSplits = 32;    // == TPI_ATTN_MAX_SPLITS

// Pointers of one emulated shard.
struct ShardView {
    const float *attn_norm, *w_qkv, *w_o, *ffn_norm, *w_gate, *w_up, *w_down;
    float *k, *v;          // [nkv][max_seq][d]
    float *partial_out;    // [h]
    float *ws;             // workspace base
    __host__ __device__ unsigned *ws_u32() const { return reinterpret_cast<unsigned *>(ws); }
};

// Shape, position and workspace layout: everything but the per-shard pointers.
struct DecodeDims {
    int h, nq, nkv, d, sl, max_seq, pos;
    float eps;
    double log2_base;      // log2(rope_base)
    const float *h_in;     // [h], shared by all shards
    int n_splits, chunk_len;   // attention: splits of slots 0..pos, slots per split
    // workspace layout, offsets in floats from ShardView::ws
    int ws_q;              // [nq*d]                    rotated queries
    int ws_att_m;          // [nq][kAttnMaxSplits]      split maxima
    int ws_att_l;          // [nq][kAttnMaxSplits]      split sums
    int ws_att_acc;        // [nq][kAttnMaxSplits][d]   split unnormalised outputs
    int ws_o;              // [nq*d]                    merged, normalised attention output
    int ws_act;            // [sl]                      silu(gate) * up
    int ws_cnt;            // [nkv] uint32              attention merge tickets (zeroed by stage 1)
    int ws_total;          // floats
};



// Star reduce folded into the epilogue of a row-parallel stage (one device's view: its own partial
// is in registers, the peers' partials are in memory).  out[i] = sum in rank order, then + residual.
struct FusedReduce {
    int n = 0, rank = 0;                  // n == 0: no folding, the stage stores its partial
    int all = 0;                          // batched call: all n ranks' partials are formed by this launch (no peers)
    const float *residual = nullptr;
    float *out = nullptr;
    const float *peer[kMaxBatchShards] = {};   // partial vectors of the ranks; entry `rank` is not read
};

struct DecodeArgs : DecodeDims {
    ShardView s[kMaxBatchShards];
    FusedReduce rf;        // single-shard calls only: reduce folded into the row-parallel stage
};

hipError_t launch_attn_phase(const DecodeArgs &a, int n_shards, hipStream_t st);
hipError_t launch_ffn_phase(const DecodeArgs &a, int n_shards, hipStream_t st);

}  // namespace tpi