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
};

struct DecodeArgs {
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
    int ws_act;            // [sl]                      silu(gate) * up
    int ws_total;          // floats
    ShardView s[kMaxBatchShards];
};

hipError_t launch_attn_phase(const DecodeArgs &a, int n_shards, hipStream_t st);
hipError_t launch_ffn_phase(const DecodeArgs &a, int n_shards, hipStream_t st);

}  // namespace tpi
