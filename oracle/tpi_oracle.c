/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Plain, slow CPU oracle for one device's tensor-parallel shard of a
 * Llama-style decoder layer as used by TPI-LLM (arxiv 2410.00531), for the
 * fixed-order star all-reduce sum, and for the prefill variant.  Only the test
 * suite, the smoke check and the benchmark's cpu_baseline leg may use it.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * Arithmetic: inputs are fp32 (bf16 inputs arrive already widened to fp32,
 * which is exact); every sum, product, square root, exponential and
 * trigonometric value is taken in fp64; values are rounded to fp32 only where
 * the method stores them at an interface: KV-cache entries and the output of
 * the sequential fp32 reduce.
 *
 * What follows the paper (Sec. 3.1 Step 3, Eq. 1, Eq. 2, Alg. 1 and Alg. 2)
 * and what is a reading of it:
 *   - attention block on the device's own heads, local KV cache, all-reduce
 *     plus shortcut (Eq. 1); FFN block with SiLU gate on the device's own
 *     columns, all-reduce plus shortcut (Eq. 2);
 *   - "norm" is read as RMSNorm (Llama / Yi models), eps inside the root;
 *   - the output projection W_O is absent from Eq. 1 but counted in the
 *     attention block's parameters (appendix parameter-count table), so the
 *     block's partial is W_O^h * concat(head outputs);
 *   - position embeddings (Alg. 1 "Preprocess") are read as rotary embeddings
 *     with rotate-half pairing and theta_i = base^(-2i/d);
 *   - the new token's K/V are stored at slot pos ("cache position") first and
 *     attention runs over slots 0..pos; K is cached after rotation, V raw;
 *   - the reduce sums ranks 0..N-1 left to right and then adds the shortcut.
 *
 * Loops are written in the order of the definitions; the only parallelism is
 * an OpenMP "parallel for" over independent output rows / heads / tokens.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t hidden;     /* h                                   */
    int32_t n_q;        /* query heads held by this shard      */
    int32_t n_kv;       /* KV heads held by this shard         */
    int32_t head_dim;   /* d                                   */
    int32_t ffn;        /* FFN columns held by this shard      */
    int32_t max_seq;    /* slots per KV head in the cache      */
    double  rms_eps;
    double  rope_base;
} orc_cfg;

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* RMSNorm: out_i = x_i / sqrt(mean(x^2) + eps) * g_i. */
void orc_rmsnorm(const float *x, const float *g, int32_t h, double eps, double *out)
{
    double ss = 0.0;
    for (int32_t i = 0; i < h; ++i) ss += (double)x[i] * (double)x[i];
    double ms = ss / (double)h;
    double r = sqrt(ms + eps);
    for (int32_t i = 0; i < h; ++i) out[i] = (double)x[i] / r * (double)g[i];
}

/* y = W x with W row-major [rows][cols] (fp32) and x, y fp64. */
void orc_matvec(const float *W, int64_t rows, int64_t cols, const double *x, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < rows; ++o) {
        const float *w = W + o * cols;
        double acc = 0.0;
        for (int64_t i = 0; i < cols; ++i) acc += (double)w[i] * x[i];
        y[o] = acc;
    }
}

/* Rotary embedding at integer position pos, in place on n_heads vectors of
 * length d laid out back to back.  Pair (i, i + d/2), angle pos * base^(-2i/d):
 *   out_i       = x_i cos - x_{i+d/2} sin
 *   out_{i+d/2} = x_{i+d/2} cos + x_i sin
 * At pos == 0 the angle is exactly 0, cos == 1, sin == 0: identity. */
void orc_rope(double *v, int32_t n_heads, int32_t d, int32_t pos, double base)
{
    int32_t half = d / 2;
    for (int32_t hd = 0; hd < n_heads; ++hd) {
        double *x = v + (int64_t)hd * d;
        for (int32_t i = 0; i < half; ++i) {
            double theta = pow(base, -2.0 * (double)i / (double)d);
            double ang = (double)pos * theta;
            double c = cos(ang), s = sin(ang);
            double a = x[i], b = x[i + half];
            x[i] = a * c - b * s;
            x[i + half] = b * c + a * s;
        }
    }
}

/* softmax(q.K^T / sqrt(d)) V for one query head against slots 0..last of one
 * KV head (cache rows are fp32).  probs (nullable) receives the last+1
 * probabilities. */
static void attend_one(const double *q, const float *Kg, const float *Vg, int32_t d,
                       int32_t last, double *o, double *probs)
{
    int32_t n = last + 1;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    double scale = 1.0 / sqrt((double)d);
    for (int32_t t = 0; t < n; ++t) {
        const float *k = Kg + (int64_t)t * d;
        double acc = 0.0;
        for (int32_t i = 0; i < d; ++i) acc += q[i] * (double)k[i];
        s[t] = acc * scale;
        if (s[t] > m) m = s[t];
    }
    double z = 0.0;
    for (int32_t t = 0; t < n; ++t) { s[t] = exp(s[t] - m); z += s[t]; }
    for (int32_t t = 0; t < n; ++t) s[t] /= z;
    for (int32_t i = 0; i < d; ++i) o[i] = 0.0;
    for (int32_t t = 0; t < n; ++t) {
        const float *v = Vg + (int64_t)t * d;
        for (int32_t i = 0; i < d; ++i) o[i] += s[t] * (double)v[i];
    }
    if (probs) memcpy(probs, s, sizeof(double) * (size_t)n);
    free(s);
}

static int cfg_ok(const orc_cfg *c)
{
    if (!c) return 0;
    if (c->hidden < 1 || c->n_q < 1 || c->n_kv < 1 || c->head_dim < 2 || c->ffn < 1) return 0;
    if (c->head_dim % 2) return 0;
    if (c->n_q % c->n_kv) return 0;
    if (c->max_seq < 1) return 0;
    return 1;
}

/*
 * Attention block of one shard for n_tokens consecutive tokens at positions
 * pos0 .. pos0+n_tokens-1 (decode is n_tokens == 1).   Eq. 1, inside the
 * all_reduce: the value this device contributes.
 *
 *   g1      [h]                  RMSNorm gain
 *   w_qkv   [(n_q+2 n_kv) d][h]  rows: Q heads, then K heads, then V heads
 *   w_o     [h][n_q d]
 *   K, V    [n_kv][max_seq][d]   fp32 caches, slots < pos0 already filled;
 *                                slots pos0.. are written here (K rotated)
 *   h_in    [n_tokens][h]
 *   partial [n_tokens][h]        fp64 out
 *   q_out   nullable [n_tokens][n_q d]   rotated queries
 *   o_out   nullable [n_tokens][n_q d]   per-head attention outputs
 *   probs   nullable [n_q][pos0+n_tokens] softmax row of the LAST token
 * returns 0, or -1 on a bad argument.
 */
int orc_attn_block(const orc_cfg *c, const float *g1, const float *w_qkv, const float *w_o,
                   float *K, float *V, int32_t pos0, int32_t n_tokens, const float *h_in,
                   double *partial, double *q_out, double *o_out, double *probs)
{
    if (!cfg_ok(c) || !g1 || !w_qkv || !w_o || !K || !V || !h_in || !partial) return -1;
    if (pos0 < 0 || n_tokens < 1 || (int64_t)pos0 + n_tokens > c->max_seq) return -1;
    const int32_t h = c->hidden, d = c->head_dim, nq = c->n_q, nkv = c->n_kv;
    const int64_t dq = (int64_t)nq * d, dkv = (int64_t)nkv * d;
    const int32_t group = nq / nkv;
    double *xn = (double *)malloc(sizeof(double) * (size_t)h);
    double *qkv = (double *)malloc(sizeof(double) * (size_t)(dq + 2 * dkv));
    double *q_all = (double *)malloc(sizeof(double) * (size_t)(dq * n_tokens));

    /* projections, rotation and cache append, token by token */
    for (int32_t i = 0; i < n_tokens; ++i) {
        int32_t pos = pos0 + i;
        orc_rmsnorm(h_in + (int64_t)i * h, g1, h, c->rms_eps, xn);
        orc_matvec(w_qkv, dq + 2 * dkv, h, xn, qkv);
        double *q = qkv, *k = qkv + dq, *v = qkv + dq + dkv;
        orc_rope(q, nq, d, pos, c->rope_base);
        orc_rope(k, nkv, d, pos, c->rope_base);
        for (int32_t g = 0; g < nkv; ++g)
            for (int32_t e = 0; e < d; ++e) {
                int64_t slot = ((int64_t)g * c->max_seq + pos) * d + e;
                K[slot] = (float)k[(int64_t)g * d + e];
                V[slot] = (float)v[(int64_t)g * d + e];
            }
        memcpy(q_all + (int64_t)i * dq, q, sizeof(double) * (size_t)dq);
    }
    if (q_out) memcpy(q_out, q_all, sizeof(double) * (size_t)(dq * n_tokens));

    /* causal attention: token i sees slots 0 .. pos0+i */
    double *o_all = (double *)malloc(sizeof(double) * (size_t)(dq * n_tokens));
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int32_t i = 0; i < n_tokens; ++i)
        for (int32_t j = 0; j < nq; ++j) {
            int32_t g = j / group;
            double *pr = (probs && i == n_tokens - 1)
                             ? probs + (int64_t)j * (pos0 + n_tokens) : NULL;
            attend_one(q_all + (int64_t)i * dq + (int64_t)j * d,
                       K + (int64_t)g * c->max_seq * d, V + (int64_t)g * c->max_seq * d,
                       d, pos0 + i, o_all + (int64_t)i * dq + (int64_t)j * d, pr);
        }
    if (o_out) memcpy(o_out, o_all, sizeof(double) * (size_t)(dq * n_tokens));

    /* row-parallel output projection: this shard's partial sum */
    for (int32_t i = 0; i < n_tokens; ++i)
        orc_matvec(w_o, h, dq, o_all + (int64_t)i * dq, partial + (int64_t)i * h);

    free(o_all); free(q_all); free(qkv); free(xn);
    return 0;
}

/*
 * FFN block of one shard (Eq. 2, inside the all_reduce):
 *   partial = W_down ( silu(W_gate xn) * (W_up xn) ),  xn = rmsnorm(h_in, g2)
 *   w_gate, w_up [ffn][h];  w_down [h][ffn];  h_in, partial [n_tokens][h]
 *   act_out nullable [n_tokens][ffn]
 */
int orc_ffn_block(const orc_cfg *c, const float *g2, const float *w_gate, const float *w_up,
                  const float *w_down, int32_t n_tokens, const float *h_in, double *partial,
                  double *act_out)
{
    if (!cfg_ok(c) || !g2 || !w_gate || !w_up || !w_down || !h_in || !partial) return -1;
    if (n_tokens < 1) return -1;
    const int32_t h = c->hidden, s = c->ffn;
    double *xn = (double *)malloc(sizeof(double) * (size_t)h);
    double *gt = (double *)malloc(sizeof(double) * (size_t)s);
    double *up = (double *)malloc(sizeof(double) * (size_t)s);
    for (int32_t i = 0; i < n_tokens; ++i) {
        orc_rmsnorm(h_in + (int64_t)i * h, g2, h, c->rms_eps, xn);
        orc_matvec(w_gate, s, h, xn, gt);
        orc_matvec(w_up, s, h, xn, up);
        for (int32_t j = 0; j < s; ++j) gt[j] = gt[j] / (1.0 + exp(-gt[j])) * up[j];
        if (act_out) memcpy(act_out + (int64_t)i * s, gt, sizeof(double) * (size_t)s);
        orc_matvec(w_down, h, s, gt, partial + (int64_t)i * h);
    }
    free(up); free(gt); free(xn);
    return 0;
}

/* Star all-reduce sum as the master performs it, in fp32, rank 0 first:
 * out_i = (((p0_i + p1_i) + p2_i) + ... + p_{n-1,i}) + residual_i.
 * volatile keeps every partial sum rounded to fp32 and blocks reassociation. */
int orc_reduce_seq_f32(const float *const *partials, int32_t n, int64_t len,
                       const float *residual, float *out)
{
    if (!partials || n < 1 || len < 0 || !out) return -1;
    for (int64_t i = 0; i < len; ++i) {
        volatile float acc = partials[0][i];
        for (int32_t r = 1; r < n; ++r) acc = acc + partials[r][i];
        if (residual) acc = acc + residual[i];
        out[i] = acc;
    }
    return 0;
}

/* The same sum in fp64 (for identity checks against an unsharded layer). */
int orc_reduce_f64(const double *const *partials, int32_t n, int64_t len,
                   const float *residual, double *out)
{
    if (!partials || n < 1 || len < 0 || !out) return -1;
    for (int64_t i = 0; i < len; ++i) {
        double acc = partials[0][i];
        for (int32_t r = 1; r < n; ++r) acc += partials[r][i];
        if (residual) acc += (double)residual[i];
        out[i] = acc;
    }
    return 0;
}
