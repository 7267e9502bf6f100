/*
 * libtpi -- MI355X (gfx950) hot path of TPI-LLM tensor-parallel inference
 * (arxiv 2410.00531): one device's shard of a Llama-style decoder layer, the
 * star all-reduce sum of the N shards' partial outputs, a sliding window of
 * layer shards (or attention / FFN blocks) streamed from pinned host memory
 * into HBM, the bf16 prefill of the same shard, and the master's embedding,
 * task head and token choice.
 *
 * Conventions for every entry point
 *   - C ABI, plain pointers and sizes.  A pointer is a DEVICE pointer unless
 *     its name starts with host_ or its comment says "host".
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute entry points only enqueue work on that stream and return; they
 *     never synchronise, allocate or free.
 *   - The caller owns every buffer (weights, KV cache, activations,
 *     workspace, pinned host blobs, window slots).  The library owns only
 *     tpi_window and tpi_decoder objects.
 *   - Return value: TPI_OK (0) or a negative tpi_status.  Argument errors are
 *     detected before anything is queued; tpi_last_error() returns a
 *     thread-local description of the last failure.
 *   - Weight matrices are row-major [out][in], so y = W x reads rows of W.
 *   - Alignment: every device pointer 16-byte aligned; hidden, ffn_local and
 *     head_dim multiples of 4 for fp32 shards, of 8 for bf16 shards
 *     (TPI_EUNSUPPORTED otherwise).
 */
#ifndef TPI_H
#define TPI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TPI_OK = 0,
    TPI_EINVAL = -1,        /* null pointer, size or position out of range, unknown enum   */
    TPI_EUNSUPPORTED = -2,  /* valid request that this build has no kernel for             */
    TPI_ERUNTIME = -3,      /* a HIP call failed; text in tpi_last_error()                 */
    TPI_ESTATE = -4         /* window protocol violated (acquire before prefetch, ...)     */
} tpi_status;

enum { TPI_F32 = 0, TPI_BF16 = 1 };

/* The all-reduce sits between the two phases of a layer (Alg. 1 / Alg. 2 loop
 * body: attention, allreduce, FFN, allreduce). */
enum { TPI_PHASE_ATTN = 1, TPI_PHASE_FFN = 2 };

/* Upper limits of this build. */
#define TPI_MAX_REDUCE_RANKS 64   /* partial vectors one tpi_star_reduce call can sum   */
#define TPI_MAX_HEAD_DIM 256
#define TPI_ATTN_MAX_SPLITS 32    /* KV-length splits of the decode attention            */
#define TPI_MAX_BATCH_SHARDS 16   /* shards one batched call can take                    */
#define TPI_MAX_ROW 16384         /* decode: hidden, ffn_local and n_q_local * head_dim  */
#define TPI_STATIC_WORKSPACE_BYTES (1u << 20)   /* built-in workspace of tpi_shard_layer_decode_static */

/* Shape of ONE device's shard of one decoder layer (Sec. 3.1 Step 1: attention
 * heads and FFN columns are divided among devices). */
typedef struct tpi_shard_cfg {
    int32_t hidden;       /* h: hidden size, replicated on every device             */
    int32_t n_q_local;    /* query heads on this device                             */
    int32_t n_kv_local;   /* KV heads on this device; must divide n_q_local         */
    int32_t head_dim;     /* d                                                      */
    int32_t ffn_local;    /* FFN columns on this device                             */
    int32_t max_seq;      /* slots per KV head in the cache                         */
    float   rms_eps;      /* RMSNorm epsilon (inside the square root)               */
    float   rope_base;    /* rotary base; theta_i = base^(-2i/d), rotate-half pairs */
    int32_t dtype;        /* TPI_F32 (decode) or TPI_BF16 (prefill weights/inputs)  */
} tpi_shard_cfg;

/* Weights of one layer of one shard: the attention block (norm gain, W_Q, W_K,
 * W_V, W_O slices) and the FFN block (norm gain, gate, up, down slices) of the
 * appendix parameter-count table.  Element type is cfg.dtype except the two
 * gains, which are always fp32. */
typedef struct tpi_layer_weights {
    const void *attn_norm;  /* [h] fp32                                               */
    const void *w_qkv;      /* [(n_q+2 n_kv) d][h]: Q-head rows, then K, then V rows  */
    const void *w_o;        /* [h][n_q d]   (row-parallel: yields a partial sum)      */
    const void *ffn_norm;   /* [h] fp32                                               */
    const void *w_gate;     /* [ffn_local][h]                                         */
    const void *w_up;       /* [ffn_local][h]                                         */
    const void *w_down;     /* [h][ffn_local] (row-parallel: yields a partial sum)    */
} tpi_layer_weights;

/* This device's KV cache of one layer: only its own heads (Sec. 3.1, the
 * distributed KV cache).  [n_kv_local][max_seq][head_dim], element type
 * cfg.dtype.  K is stored after rotation, V as projected. */
typedef struct tpi_kv_layer {
    void *k;
    void *v;
} tpi_kv_layer;

/* Bytes of workspace a decode (n_tokens = 1) or prefill call needs.  The
 * workspace carries no state between calls, needs no initialisation, and may
 * be shared by calls on the same stream.  Returns 0 on a bad cfg. */
size_t tpi_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_tokens);

/*
 * One phase of one layer for one shard, one token (batch 1 decode), fp32.
 *
 * TPI_PHASE_ATTN -- the term inside all_reduce() of Eq. 1:
 *   xn = rmsnorm(h_in, attn_norm); q,k,v = W_qkv xn; rotate q and k at `pos`;
 *   store k,v in cache slot `pos` (exactly that slot, nothing else in the
 *   cache is written); softmax(q K^T / sqrt(d)) V over slots 0..pos for each
 *   local head (query head j uses KV head j / (n_q_local / n_kv_local));
 *   partial_out = W_o o.
 * TPI_PHASE_FFN -- the term inside all_reduce() of Eq. 2:
 *   xn = rmsnorm(h_in, ffn_norm);
 *   partial_out = W_down (silu(W_gate xn) * (W_up xn)).
 *
 * h_in [h] fp32: H_ffn of the previous layer (ATTN) or H_attn (FFN).
 * partial_out [h] fp32.  kv may be NULL for TPI_PHASE_FFN.
 * Errors: TPI_EINVAL for null pointers, pos < 0, pos >= max_seq, odd or
 * non-positive sizes, n_q_local % n_kv_local != 0, unknown phase;
 * TPI_EUNSUPPORTED for cfg.dtype != TPI_F32 or sizes outside the limits above.
 */
int tpi_shard_layer_decode(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                           const tpi_kv_layer *host_kv, int32_t pos, int phase,
                           const float *h_in, float *partial_out, void *workspace,
                           void *stream);

/*
 * tpi_shard_layer_decode for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same computation, same kernels and same bits, but the workspace
 * is a device array inside the library (TPI_STATIC_WORKSPACE_BYTES = 1 MiB per
 * GPU, held until the process ends) instead of an argument; the call allocates
 * and frees nothing (the first call on a device looks the array's address up).
 * TPI_EUNSUPPORTED: tpi_workspace_bytes(cfg, 1) > TPI_STATIC_WORKSPACE_BYTES
 * (the 70B-shaped shard needs 156 KB).  All calls on one GPU share the one
 * array: calls that overlap in time on one GPU (different streams, different
 * threads) race -- queue them on one stream, or give all but one of them
 * tpi_shard_layer_decode with workspaces of their own.  The array keeps the
 * last call's contents; nothing in it needs clearing between calls.
 * Other arguments and errors as for tpi_shard_layer_decode.
 */
int tpi_shard_layer_decode_static(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                                  const tpi_kv_layer *host_kv, int32_t pos, int phase,
                                  const float *h_in, float *partial_out, void *stream);

/*
 * One phase for one shard with the star reduce and the shortcut folded into
 * its last (row-parallel) stage, as one device of the system sees it: the
 * device's own partial never leaves the chip's registers, the other ranks'
 * partials are read from host_partials[i] (device pointers to [h] fp32, entry
 * `rank` ignored; they must be complete before the call), and
 *   out[i] = (((p0[i] + p1[i]) + ...) + p_{n-1}[i]) + h_in[i]
 * with this device's partial at position `rank`: bit for bit what
 * tpi_shard_layer_decode followed by tpi_star_reduce(residual = h_in) yields.
 * out [h] fp32 may alias h_in.  1 <= n_ranks <= TPI_MAX_BATCH_SHARDS.
 */
int tpi_shard_layer_decode_reduce(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                                  const tpi_kv_layer *host_kv, int32_t pos, int phase,
                                  const float *h_in, int32_t n_ranks, int32_t rank,
                                  const float *const *host_partials, float *out, void *workspace,
                                  void *stream);

/*
 * The same phase for n_shards emulated devices in one set of launches (the
 * shards of a layer are independent between all-reduces, Sec. 3.1 Step 3).
 * host_w, host_kv, host_partial_out and host_workspace are HOST arrays of
 * n_shards entries; all shards share cfg, pos and h_in.  Results are
 * identical to n_shards calls of tpi_shard_layer_decode.
 * 1 <= n_shards <= TPI_MAX_BATCH_SHARDS.
 */
int tpi_shards_layer_decode(const tpi_shard_cfg *cfg, int32_t n_shards,
                            const tpi_layer_weights *host_w, const tpi_kv_layer *host_kv,
                            int32_t pos, int phase, const float *h_in,
                            float *const *host_partial_out, void *const *host_workspace,
                            void *stream);

/*
 * The batched phase with the star reduce and the shortcut folded in (the whole
 * step between two layer inputs of Alg. 1: every device's block, then
 * all_reduce + shortcut): all n_shards ranks' partials are formed by this
 * call and
 *   out[i] = (((p0[i] + p1[i]) + ...) + p_{n-1}[i]) + h_in[i]
 * bit for bit what tpi_shards_layer_decode followed by
 * tpi_star_reduce(residual = h_in) yields; the partial vectors are not written
 * to memory (the last, row-parallel stage walks the ranks in order for its
 * rows of the output).  out [h] fp32, must not alias h_in.  Arguments and
 * errors otherwise as for tpi_shards_layer_decode.
 */
int tpi_shards_layer_decode_reduce(const tpi_shard_cfg *cfg, int32_t n_shards,
                                   const tpi_layer_weights *host_w, const tpi_kv_layer *host_kv,
                                   int32_t pos, int phase, const float *h_in, float *out,
                                   void *const *host_workspace, void *stream);

/*
 * Prefill: the same two phases for n_tokens consecutive prompt tokens at
 * positions pos0 .. pos0+n_tokens-1 with causal attention (token i sees slots
 * 0..pos0+i), filling cache slots pos0..pos0+n_tokens-1 and no others.
 * Weights, h_in [n_tokens][h] and the KV cache are bf16; accumulation is fp32
 * on the matrix cores; partial_out [n_tokens][h] is fp32.  (The decode entry
 * points take fp32 caches: tpi_kv_widen carries a prefilled cache over.)
 * Errors as for decode; pos0 + n_tokens > max_seq is TPI_EINVAL;
 * cfg.dtype != TPI_BF16 is TPI_EUNSUPPORTED.
 */
int tpi_shard_layer_prefill(const tpi_shard_cfg *cfg, const tpi_layer_weights *host_w,
                            const tpi_kv_layer *host_kv, int32_t pos0, int32_t n_tokens,
                            int phase, const void *h_in, float *partial_out, void *workspace,
                            void *stream);

/*
 * From prefill to decode on one cache (Sec. 3.1: the KV cache a device keeps
 * for its heads serves every later token).  The prefill entry points fill a
 * bf16 cache and the decode entry points read an fp32 one, so a prompt that
 * was prefilled through this library continues like this: tpi_kv_widen copies
 * slots 0 .. n_slots-1 of every local KV head from the bf16 cache
 * [n_kv_local][src_max_seq][head_dim] into the fp32 cache
 * [n_kv_local][dst_max_seq][head_dim] (exact: every bf16 value is an fp32
 * value); slots from n_slots on are left alone.  Decode then appends at
 * pos = n_slots.  TPI_EINVAL: null pointers, sizes < 1, odd head_dim, n_slots
 * outside either cache.
 */
int tpi_kv_widen(int32_t n_kv_local, int32_t head_dim, int32_t n_slots,
                 const tpi_kv_layer *host_src_bf16, int32_t src_max_seq,
                 const tpi_kv_layer *host_dst_f32, int32_t dst_max_seq, void *stream);

/*
 * The same prefill phase for n_shards emulated devices in one set of launches
 * (every kernel takes the shard from a grid dimension; the GEMM plans size
 * their tiles for the batch).  host_w, host_kv (may be NULL in the FFN
 * phase), host_partial_out and host_workspace are HOST arrays of n_shards
 * entries; h_in is shared (it is replicated, Sec. 3.1).  Every shard has the
 * shape cfg; shards must not share a workspace.  Per shard the results agree
 * with tpi_shard_layer_prefill within the bf16 tolerance (the plans, and with
 * them the order of the sums, can differ).
 * Errors as above, plus TPI_EINVAL for n_shards outside
 * [1, TPI_MAX_BATCH_SHARDS].
 */
int tpi_shards_layer_prefill(const tpi_shard_cfg *cfg, int32_t n_shards,
                             const tpi_layer_weights *host_w, const tpi_kv_layer *host_kv,
                             int32_t pos0, int32_t n_tokens, int phase, const void *h_in,
                             float *const *host_partial_out, void *const *host_workspace,
                             void *stream);

/*
 * Hint for the prefill's GEMM plans, for callers that run several prefill
 * calls side by side on different streams (the emulated shards of one layer
 * are independent between the all-reduces of Eq. 1 and Eq. 2): each call then
 * sizes its grids for 1/n_calls of the chip (wider tiles, fewer K splits).
 * A workspace sized by tpi_workspace_bytes fits every value of the hint.
 * Process-wide, takes effect for later calls, default 1.  The sum of one
 * output element runs over the contraction index in an order that depends on
 * the plan, so results under different hints agree within the bf16 tolerance,
 * not bit for bit; under one hint they are reproducible.
 * Errors: TPI_EINVAL outside [1, TPI_MAX_BATCH_SHARDS].
 */
int tpi_set_prefill_concurrency(int32_t n_calls);

/*
 * Star all-reduce sum as the master performs it (Sec. 3.2, Prop. 2; the
 * "+ H" shortcut of Eq. 1 and Eq. 2):
 *   out[i] = (((p0[i] + p1[i]) + p2[i]) + ... + p_{n-1}[i]) + residual[i]
 * in fp32, ranks in index order, shortcut last, no fused multiply-add and no
 * reassociation: exactly one bit pattern is correct.
 * host_partials: HOST array of n device pointers to [len] fp32.  residual may
 * be NULL.  out may alias residual or any partial.
 * Errors: TPI_EINVAL for n < 1, len < 0, null pointers; TPI_EUNSUPPORTED for
 * n > TPI_MAX_REDUCE_RANKS.
 */
int tpi_star_reduce(const float *const *host_partials, int32_t n, int64_t len,
                    const float *residual, float *out, void *stream);

/* The same sum (same bits in `out`); additionally stores the result rounded
 * to bf16 (nearest, ties to even) in out_bf16 [len]: the fp32 copy stays the
 * shortcut of the next reduce, the bf16 copy is the h_in of the next prefill
 * phase.  out_bf16 must not be NULL. */
int tpi_star_reduce_bf16(const float *const *host_partials, int32_t n, int64_t len,
                         const float *residual, float *out, void *out_bf16, void *stream);

/*
 * Sliding window of layer shards (Sec. 3.3; appendix "A simple-to-use memory
 * scheduler").  All n_layers blobs live in pinned host memory; `window_layers`
 * slots of layer_bytes each live in HBM and are used in ring order: the k-th
 * prefetch lands in slot k % window_layers, so the window slides over the
 * layers of one token and on into the next token's first layers.  The library
 * owns one copy stream and two events per slot; copies run on the copy stream
 * and overlap with whatever the compute stream is doing.
 *
 *   prefetch(l): enqueue the host-to-device copy of layer l into the next ring
 *                slot, after that slot's previous tenant was released.
 *                Non-blocking.
 *   acquire(l):  make compute_stream wait until the oldest prefetched copy of
 *                layer l is resident; returns its device address ("wait" of
 *                wait_and_release).
 *   release(l):  mark that slot reusable once compute_stream has finished what
 *                was queued so far ("release" of wait_and_release).
 *
 * TPI_ESTATE: prefetch while the next ring slot's tenant is prefetched or
 * acquired and not yet released (the window is full), acquire of a layer with
 * no prefetched copy in the window, release of a layer that was not acquired.
 * TPI_EINVAL: layer out of range, window_layers < 1, null pointers.
 */
typedef struct tpi_window tpi_window;

int tpi_window_create(tpi_window **out, int32_t n_layers, int32_t window_layers,
                      size_t layer_bytes, const void *const *host_layer_blobs,
                      void *device_slots);
int tpi_window_prefetch(tpi_window *w, int32_t layer);
int tpi_window_acquire(tpi_window *w, int32_t layer, void *compute_stream,
                       const void **dev_blob);
int tpi_window_release(tpi_window *w, int32_t layer, void *compute_stream);
/* Blocks until every queued copy has finished, then frees the object. */
int tpi_window_destroy(tpi_window *w);

/*
 * The same window at the paper's granularity (Sec. 3.3: the unit that is
 * loaded ahead is one attention block or one FFN block, and the window size
 * counts blocks, Prop. 5) and with block retention (Prop. 6: one FFN block out
 * of every T stays in memory for good).
 *
 * A block is any contiguous run of bytes in pinned host memory; in the usual
 * arrangement blocks 2l and 2l+1 are the attention block (attn_norm | w_qkv |
 * w_o) and the FFN block (ffn_norm | w_gate | w_up | w_down) of layer l.
 * Blocks of one slot class pass through that class's ring of equally sized
 * HBM slots (class 0: attention blocks, class 1: FFN blocks; a window of w
 * blocks, w even, is w/2 slots in each).  A retained block has a device home of
 * its own (`resident`, caller-owned, `bytes` long): its first prefetch copies
 * it there, later prefetches do nothing, acquire waits for that one copy and
 * returns `resident`, release only checks the pairing.
 *
 * prefetch / acquire / release / copy_stats / destroy above take block indices
 * for a window created here; ring order, states and errors are per slot class.
 * The arrays are copied; host and device memory stay with the caller.
 * TPI_EINVAL: counts < 1, null pointers, a block larger than its class's slot,
 * slot class out of range, a retained block without `resident`.
 */
typedef struct tpi_window_block {
    const void *host;     /* pinned host memory */
    size_t bytes;
    int32_t slot_class;   /* ignored for a retained block */
    int32_t retained;     /* nonzero: copied once into `resident`, never evicted */
    void *resident;       /* device memory for a retained block, NULL otherwise */
} tpi_window_block;

typedef struct tpi_window_slots {
    void *base;           /* device memory, n_slots * slot_bytes */
    size_t slot_bytes;
    int32_t n_slots;
} tpi_window_slots;

int tpi_window_create_blocks(tpi_window **out, int32_t n_blocks, const tpi_window_block *blocks,
                             int32_t n_classes, const tpi_window_slots *classes);

/*
 * The paper's own source tier: the weights stay in files and are loaded and
 * dropped as the layers go by (Sec. 3.3; there the scheduler runs on a
 * background thread of its own).  Blocks are byte ranges of files; the window owns a loader thread
 * and n_staging pinned staging buffers of the largest block's size; a block of
 * 1 MiB or more is read by n_readers threads (1..64), a contiguous part each.  prefetch
 * only queues the request and returns; the loader reads the block into the
 * next staging buffer (pread) and forwards it to its HBM slot on the window's
 * copy stream, strictly in request order.  acquire blocks the CALLING THREAD
 * until the loader has queued that copy (not until it has finished: the
 * compute stream waits for that, as with the other windows), so a prefetch
 * issued well ahead costs the caller nothing.  Slot classes, retention,
 * states and errors are those of tpi_window_create_blocks.  Files are read
 * through the page cache; they must not change while the window exists.
 * tpi_window_read_stats: time the loader has spent reading files so far.
 * TPI_EINVAL also for a file that cannot be opened; a read error or a short
 * file surfaces as TPI_ERUNTIME at the next prefetch / acquire / copy_stats.
 */
typedef struct tpi_window_file_block {
    const char *path;     /* host string, copied */
    uint64_t offset;      /* byte offset of the block in the file */
    size_t bytes;
    int32_t slot_class;
    int32_t retained;
    void *resident;
} tpi_window_file_block;

int tpi_window_create_files(tpi_window **out, int32_t n_blocks, const tpi_window_file_block *blocks,
                            int32_t n_classes, const tpi_window_slots *classes, int32_t n_staging,
                            int32_t n_readers);
int tpi_window_read_stats(tpi_window *w, double *read_ms);
/*
 * Optional, once, before the first prefetch: makes sure that the window's
 * copies overlap with the kernels of compute_stream.  A process has only a few
 * hardware queues (four here) which its streams share; if the window's copy
 * stream happens to share one with compute_stream, the marker behind every
 * copy holds back the kernels queued after it, and copies and compute take
 * turns instead of overlapping (the window then still computes the right
 * thing, in compute + copy time).  The call probes for that with a 16 MiB copy
 * against a 4-byte fill on compute_stream and moves the window to a further
 * stream until the two are independent (at most 8 tries; *tried, nullable,
 * receives their number).  It allocates its probe buffers, synchronises both
 * streams and frees again -- a set-up call.  TPI_ESTATE after a prefetch.
 */
int tpi_window_calibrate(tpi_window *w, void *compute_stream, int32_t *tried);
/* Total time (ms) the copy stream spent in copies between the first prefetch
 * and the last one completed so far, and the bytes requested so far.  Either
 * output may be NULL; asking for the time synchronises the copy stream, asking
 * for the bytes alone waits for nothing. */
int tpi_window_copy_stats(tpi_window *w, double *copy_ms, uint64_t *bytes);

/*
 * A host model of the device side of the window, for checking a schedule of
 * prefetch / acquire / release calls without a GPU.  It models queues that run
 * in order, events, asynchronous copies and "kernels" that read memory; nothing
 * runs when it is queued -- tpi_sim_run (and every call of the window that has
 * to wait) executes what is queued, always picking at random (by `seed`) among
 * the queues whose next operation may run.  Any order the device could choose,
 * given queue order and event waits alone, can occur; a reader that is not
 * ordered after the copy it needs, or a copy not ordered after the readers of
 * the slot it overwrites, reads the wrong bytes in some of these orders.
 *
 * tpi_window_create_blocks_sim / _files_sim: the same windows running on the
 *   model; every "device" pointer (slots, resident homes) is plain host memory
 *   and host blocks need not be pinned.  The window must be destroyed before
 *   the model.  compute_stream arguments of acquire / release are handles from
 *   tpi_sim_stream (NULL: the model's null stream).
 * tpi_sim_read: queues a kernel on `stream` that reads [ptr, ptr + bytes) and
 *   takes cost_ms; when the model executes it, *host_hash receives tpi_sim_hash
 *   of what it saw and *host_start_ms (nullable) the time it started.  bytes = 0
 *   queues a kernel that only takes time (an all-reduce, say).
 * tpi_sim_run: executes everything queued; TPI_ESTATE if operations are left
 *   that wait for an event nobody recorded.
 * Time: every queue has a clock in model milliseconds, starting at 0; a copy
 *   takes bytes / rate (tpi_sim_set_copy_rate, default 1e6 bytes per ms), a
 *   wait moves the clock up to the recording's time, so the times follow from
 *   the dependencies alone and not from the order drawn.  tpi_sim_stream_time
 *   reads a queue's clock.
 * Calls may come from several host threads.  TPI_EINVAL: null arguments, a
 * stream of another model.
 */
typedef struct tpi_sim tpi_sim;
int tpi_sim_create(tpi_sim **out, uint64_t seed);
void *tpi_sim_stream(tpi_sim *sim);
int tpi_sim_read(tpi_sim *sim, void *stream, const void *ptr, size_t bytes, double cost_ms,
                 uint64_t *host_hash, double *host_start_ms);
int tpi_sim_set_copy_rate(tpi_sim *sim, double bytes_per_ms);
int tpi_sim_stream_time(tpi_sim *sim, void *stream, double *host_ms);
int tpi_sim_run(tpi_sim *sim);
uint64_t tpi_sim_hash(const void *ptr, size_t bytes);   /* FNV-1a, 64 bit */
int tpi_sim_destroy(tpi_sim *sim);
int tpi_window_create_blocks_sim(tpi_window **out, tpi_sim *sim, int32_t n_blocks,
                                 const tpi_window_block *blocks, int32_t n_classes,
                                 const tpi_window_slots *classes);
int tpi_window_create_files_sim(tpi_window **out, tpi_sim *sim, int32_t n_blocks,
                                const tpi_window_file_block *blocks, int32_t n_classes,
                                const tpi_window_slots *classes, int32_t n_staging, int32_t n_readers);

/*
 * The ends of the token loop, run by the master device only (Alg. 1,
 * "Preprocess" and "Postprocess"; Sec. 3.1 Step 4).  All pointers are device
 * pointers; nothing is allocated, nothing synchronises.
 *
 * tpi_embed_token: h_out[hidden] = row `token` of w_emb [vocab][hidden] (fp32),
 *   the input embedding of the token that was just chosen.
 * tpi_lm_head: logits[v] = w_head[v] . rmsnorm(h_in; final_norm, rms_eps) for
 *   v < vocab; w_head [vocab][hidden] fp32 row-major, read once (a streaming
 *   GEMV like the decode stages).  hidden a multiple of 4, at most 16384;
 *   final_norm, w_head, h_in 16-byte aligned (else TPI_EUNSUPPORTED).
 * tpi_next_token: softmax over logits[vocab]; probs (nullable) receives the
 *   distribution; *token_out (device int32) receives the next token:
 *   u < 0  -> the index of the largest logit, the lowest index among equals;
 *   0 <= u < 1 -> inverse-CDF sampling with the caller's uniform draw u: the
 *   first index whose cumulative probability exceeds u (sums in fp32, index
 *   order).  The library draws no random numbers.
 * TPI_EINVAL: null pointers, vocab < 1, token outside [0, vocab), hidden not a
 * positive multiple of 4, rms_eps <= 0, u >= 1.
 */
int tpi_embed_token(const float *w_emb, int32_t vocab, int32_t hidden, int32_t token,
                    float *h_out, void *stream);
int tpi_lm_head(const float *final_norm, const float *w_head, int32_t vocab, int32_t hidden,
                float rms_eps, const float *h_in, float *logits, void *stream);
int tpi_next_token(const float *logits, int32_t vocab, float u, float *probs,
                   int32_t *token_out, void *stream);

/*
 * Whole-token decode of ONE device's shard (Alg. 2, the worker's loop over all
 * decoder layers of one token) in a single persistent launch.  NOT AVAILABLE in
 * this build: tpi_decoder_create checks its arguments and returns
 * TPI_EUNSUPPORTED, tpi_decoder_workspace_bytes returns a token size (0 on a
 * bad cfg), token / status on a handle return TPI_EUNSUPPORTED.  The names keep
 * their place in the ABI; the per-phase calls above cover every shape.  (A
 * chip-wide hand-over between the stages inside one kernel costs more on this
 * chip than the kernel boundary it replaces -- see the source file.)
 */
typedef struct tpi_decoder tpi_decoder;
size_t tpi_decoder_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_layers);
int tpi_decoder_create(tpi_decoder **out, const tpi_shard_cfg *cfg, int32_t n_layers,
                       const tpi_layer_weights *host_w /* [n_layers] */,
                       const tpi_kv_layer *host_kv /* [n_layers] */, int32_t n_ranks, int32_t rank,
                       const float *const *host_peer_attn /* [n_ranks] device ptrs to [h] */,
                       const float *const *host_peer_ffn /* [n_ranks] device ptrs to [h] */,
                       void *workspace, void *stream);
int tpi_decoder_token(tpi_decoder *dec, int32_t pos, const float *h_in, float *h_out, void *stream);
int tpi_decoder_status(tpi_decoder *dec, void *stream);
int tpi_decoder_grid(const tpi_decoder *dec);   /* workgroups of the persistent grid */
int tpi_decoder_destroy(tpi_decoder *dec);

/*
 * Measurement aid (not part of the method): time every launch of one stage
 * with HIP events recorded on the stream the kernel is launched on.
 *   stage: 0 off, 1 QKV+rotary, 2 attention, 3 output projection,
 *          4 gate/up, 5 down projection, 6 star reduce, 7 prefill GEMMs,
 *          8 whole-token kernel.
 * tpi_prof_enable allocates `capacity` event pairs (launches beyond that are
 * not timed) and clears earlier records; tpi_prof_read waits for the recorded
 * launches, returns the sum of their durations and their count, and clears
 * the records.  Not thread-safe; leave it off in production loops.
 */
enum { TPI_STAGE_NONE = 0, TPI_STAGE_QKV = 1, TPI_STAGE_ATTN = 2, TPI_STAGE_OPROJ = 3,
       TPI_STAGE_GATE_UP = 4, TPI_STAGE_DOWN = 5, TPI_STAGE_REDUCE = 6, TPI_STAGE_PREFILL_GEMM = 7, TPI_STAGE_TOKEN = 8 };
int tpi_prof_enable(int stage, int32_t capacity);
int tpi_prof_read(double *total_ms, int32_t *launches);

/*
 * Measurement aid (not part of the method): the cost of a hand-over between
 * two dependent streaming stages on this chip.  256 workgroups stream a buffer
 * of total_bytes once, cut into segments of segment_kib_per_wave KiB per wave
 * (2048 waves: 32 KiB per wave = 67 MB per segment); a segment stands for a
 * stage and may be consumed only once the previous segment's results are
 * known:
 *   mode 0  no hand-over (the streaming rate)
 *   mode 1  hand-over inside the workgroup (through LDS)
 *   mode 2  hand-over across the chip inside one kernel: results written
 *           through to memory, a two-level counter tree, one flag per group
 *           of workgroups, all results read back; requests for the next
 *           segment's data stay in flight meanwhile (16 KiB per wave)
 *   mode 3  hand-over by kernel boundary: one launch per segment
 * The best of `reps` runs is reported.  spread_us: first to last workgroup to
 * finish a segment; chain_us: from the last workgroup's result to the first
 * use of the next segment's data (mode 2 only).  results_ok: the exchanged
 * results were the right ones in every run.
 * Unlike the entry points of the method this call allocates (total_bytes and
 * small tables), synchronises `stream` and frees again.
 * TPI_EINVAL: total_bytes not a multiple of 2048 waves x the segment, segment
 * not a positive multiple of 16 KiB, more than 4096 segments, mode or reps out
 * of range; TPI_ERUNTIME: a HIP call failed, or a bounded wait inside the
 * probe gave up (the kernel still ends).
 */
typedef struct tpi_probe_result {
    double us_total, tb_per_s, us_per_segment, segment_mb, spread_us, chain_us;
    int32_t segments, results_ok, gave_up;
} tpi_probe_result;
int tpi_probe_handover(uint64_t total_bytes, int32_t segment_kib_per_wave, int32_t mode, int32_t reps,
                       tpi_probe_result *host_out, void *stream);

/*
 * Measurement aid (not part of the method): what paces the K loop of the
 * prefill's 256x256 GEMM tile (Sec. 3.1's linear layers at prompt length).
 * One launch is the down projection of a Llama-2-70B-shaped 8-way shard for a
 * 512-token prompt, 8 shards per launch ([512 x 3584] . [8192 x 3584]^T,
 * bf16 in, fp32 out: 512 tiles, 0.24 TFLOP), on buffers the call allocates,
 * fills with a fixed pseudo-random pattern and frees.  leave_out is a bit mask of the loop's
 * three activities to take out of the kernel: 1 the loads into LDS after the
 * first fill of the stages, 2 the fragment reads from LDS, 4 the matrix
 * instructions (0: the kernel as the library runs it; 7 is not offered).  A
 * variant with something left out computes nothing meaningful: only its time
 * is of interest.  us_per_launch: mean over `reps` launches after one untimed
 * launch; tflops: for leave_out = 0, else 0; result_ok: for leave_out = 0
 * whether the first and the last output element equal the same sums taken
 * on the host (1 / 0), -1 otherwise.
 * Unlike the entry points of the method this call allocates (0.63 GB),
 * synchronises `stream` and frees again.
 * TPI_EINVAL: host_out null, leave_out outside [0, 6], reps outside
 * [1, 1000]; TPI_ERUNTIME: a HIP call failed.
 */
typedef struct tpi_gemm_probe_result {
    double us_per_launch, tflop_per_launch, tflops;
    int32_t result_ok;
} tpi_gemm_probe_result;
int tpi_probe_gemm_loop(int32_t leave_out, int32_t reps, tpi_gemm_probe_result *host_out, void *stream);

const char *tpi_last_error(void);

/* ABI version of this header: bumped when a signature changes. */
int tpi_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TPI_H */
