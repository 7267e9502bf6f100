// The ends of the token loop, which only the master device runs (Alg. 1, "Preprocess" and
// "Postprocess"; Sec. 3.1 Step 4): the input embedding of the new token, and after the last
// layer's reduce the final RMSNorm, the task head, softmax and the choice of the next token.
//
// The task head is one more streaming GEMV (vocab rows of length hidden, read once): it uses
// the row streamer of the decode stages with the RMSNorm folded in.  The token choice is a
// single workgroup: softmax over the vocabulary, then either the largest logit or the inverse
// CDF at a uniform draw supplied by the caller.
#include <hip/hip_runtime.h>

#include <cmath>

#include "decode_stages.hpp"
#include "host_util.hpp"

namespace tpi {

struct LmHeadArgs {
    const float *norm, *w_head, *h_in;
    float *logits;
    int vocab, h;
    float eps;
};

template <int ROWS, int KCH, int UB>
__global__ __launch_bounds__(kBlock) void k_lm_head(LmHeadArgs a)
{
    __shared__ float red[ROWS * kWavesPerBlock + kWavesPerBlock];
    const int n_units = (a.vocab + ROWS - 1) / ROWS;
    auto rowfn = [&](int u, const float *(&rows)[ROWS]) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) rows[r] = a.w_head + (size_t)min(u * ROWS + r, a.vocab - 1) * a.h;
    };
    RowStreamer<ROWS, KCH, UB> st;
    st.prefetch(blockIdx.x, gridDim.x, n_units, a.h, rowfn);   // weights first: they do not depend on h_in
    float4 xr[KCH];
    const float rinv = norm_slice<KCH>(a.h_in, a.norm, a.h, a.eps, xr, red);
    auto epi = [&](int u, float (&y)[ROWS]) {
        const int r = threadIdx.x;
        const float mine = pick_own<ROWS>(y, r);
        if (r < ROWS && u * ROWS + r < a.vocab) a.logits[u * ROWS + r] = mine * rinv;
    };
    st.run(xr, red, rowfn, epi);
}

__global__ __launch_bounds__(256) void k_embed(const float *__restrict__ w_emb, int h, int token, float *__restrict__ out)
{
    const float *row = w_emb + (size_t)token * h;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < h; i += gridDim.x * blockDim.x) out[i] = row[i];
}

constexpr int kChoiceThreads = 1024;

// One workgroup.  Thread t owns the contiguous index range [t * chunk, (t + 1) * chunk).
__global__ __launch_bounds__(kChoiceThreads) void k_next_token(const float *__restrict__ logits, int vocab, float u,
                                                               float *__restrict__ probs, int *__restrict__ token_out)
{
    __shared__ float s_val[kChoiceThreads];
    __shared__ int s_idx[kChoiceThreads];
    __shared__ float s_prefix[kChoiceThreads + 1];
    const int t = threadIdx.x;
    const int chunk = (vocab + kChoiceThreads - 1) / kChoiceThreads;
    const int lo = min(t * chunk, vocab), hi = min(lo + chunk, vocab);

    // largest logit and its lowest index.  A range without a logit above -inf (all -inf, or NaN, which
    // compares as neither) still names its first index, so the token is always inside [0, vocab).
    float best = -INFINITY;
    int best_i = lo < hi ? lo : vocab;
    for (int i = lo; i < hi; ++i) {
        float z = logits[i];
        if (z > best) { best = z; best_i = i; }
    }
    s_val[t] = best; s_idx[t] = best_i;
    __syncthreads();
    for (int w = kChoiceThreads / 2; w > 0; w >>= 1) {
        if (t < w) {
            float ov = s_val[t + w]; int oi = s_idx[t + w];
            if (ov > s_val[t] || (ov == s_val[t] && oi < s_idx[t])) { s_val[t] = ov; s_idx[t] = oi; }
        }
        __syncthreads();
    }
    const float m = s_val[0];
    const int arg = s_idx[0];
    __syncthreads();

    // sum of exp(z - m): per-thread partial sums, then their prefix in thread order (fixed order of additions)
    float part = 0.f;
    for (int i = lo; i < hi; ++i) part += expf(logits[i] - m);
    s_val[t] = part;
    __syncthreads();
    if (t == 0) {
        float acc = 0.f;
        for (int k = 0; k < kChoiceThreads; ++k) { s_prefix[k] = acc; acc += s_val[k]; }
        s_prefix[kChoiceThreads] = acc;
    }
    __syncthreads();
    const float total = s_prefix[kChoiceThreads];
    if (probs) {
        const float inv = 1.0f / total;
        for (int i = lo; i < hi; ++i) probs[i] = expf(logits[i] - m) * inv;
    }
    if (u < 0.f) {                       // greedy
        if (t == 0) *token_out = arg;
        return;
    }
    // inverse CDF: the first index whose cumulative sum exceeds u * total
    const float target = u * total;
    if (t == 0) *token_out = vocab - 1;  // if rounding leaves every cumulative sum at or below the target
    __syncthreads();
    if (lo < hi && s_prefix[t] <= target && s_prefix[t + 1] > target) {
        float acc = s_prefix[t];
        int pick = hi - 1;               // the partial sums place the crossing in this range
        for (int i = lo; i < hi; ++i) {
            acc += expf(logits[i] - m);
            if (acc > target) { pick = i; break; }
        }
        *token_out = pick;
    }
}

namespace {

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

template <int KCH, int UB>
void launch_lm_head(const LmHeadArgs &a, hipStream_t st)
{
    constexpr int ROWS = 4;
    const int n_units = cdiv(a.vocab, ROWS);
    const int per = cdiv(n_units, 2048);                 // at most 8 workgroups per compute unit
    hipLaunchKernelGGL((k_lm_head<ROWS, KCH, UB>), dim3(cdiv(n_units, per)), dim3(kBlock), 0, st, a);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace tpi

using tpi::fail;

extern "C" {

int tpi_embed_token(const float *w_emb, int32_t vocab, int32_t hidden, int32_t token, float *h_out, void *stream)
{
    if (!w_emb || !h_out) return fail(TPI_EINVAL, "null argument");
    if (vocab < 1 || hidden < 1) return fail(TPI_EINVAL, "vocab %d / hidden %d < 1", vocab, hidden);
    if (token < 0 || token >= vocab) return fail(TPI_EINVAL, "token %d outside [0, %d)", token, vocab);
    hipLaunchKernelGGL(tpi::k_embed, dim3(tpi::cdiv(hidden, 256)), dim3(256), 0, (hipStream_t)stream, w_emb, hidden, token,
                       h_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}

int tpi_lm_head(const float *final_norm, const float *w_head, int32_t vocab, int32_t hidden, float rms_eps,
                const float *h_in, float *logits, void *stream)
{
    if (!final_norm || !w_head || !h_in || !logits) return fail(TPI_EINVAL, "null argument");
    if (vocab < 1) return fail(TPI_EINVAL, "vocab %d < 1", vocab);
    if (hidden < 4 || hidden % 4 != 0) return fail(TPI_EINVAL, "hidden %d must be a positive multiple of 4", hidden);
    if (!(rms_eps > 0.f)) return fail(TPI_EINVAL, "rms_eps must be positive");
    if (hidden > 16 * tpi::kChunk) return fail(TPI_EUNSUPPORTED, "hidden %d > %d", hidden, 16 * tpi::kChunk);
    if (!tpi::aligned16(final_norm) || !tpi::aligned16(w_head) || !tpi::aligned16(h_in))
        return fail(TPI_EUNSUPPORTED, "pointer not 16-byte aligned");
    tpi::LmHeadArgs a{final_norm, w_head, h_in, logits, vocab, hidden, rms_eps};
    hipStream_t st = (hipStream_t)stream;
    int kch = 1;
    while (kch * tpi::kChunk < hidden) kch *= 2;
    switch (kch) {
    case 1: tpi::launch_lm_head<1, 1>(a, st); break;
    case 2: tpi::launch_lm_head<2, 2>(a, st); break;
    case 4: tpi::launch_lm_head<4, 2>(a, st); break;
    case 8: tpi::launch_lm_head<8, 2>(a, st); break;
    default: tpi::launch_lm_head<16, 2>(a, st); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}

int tpi_next_token(const float *logits, int32_t vocab, float u, float *probs, int32_t *token_out, void *stream)
{
    if (!logits || !token_out) return fail(TPI_EINVAL, "null argument");
    if (vocab < 1) return fail(TPI_EINVAL, "vocab %d < 1", vocab);
    if (!(u < 1.0f)) return fail(TPI_EINVAL, "u must be below 1 (negative selects the largest logit)");
    hipLaunchKernelGGL(tpi::k_next_token, dim3(1), dim3(tpi::kChoiceThreads), 0, (hipStream_t)stream, logits, vocab, u, probs,
                       token_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e));
    return TPI_OK;
}

}  // extern "C"
