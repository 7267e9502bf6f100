// bf16 prefill of one shard's decoder layer on gfx950: the GEMMs run on the
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation), the small
// element-wise steps and the causal attention run on the vector ALUs.
//
// ATTN phase: k_rmsnorm_bf16 -> gemm (QKV) -> k_rope_scatter (rotary, cache fill)
//             -> k_prefill_attn (causal GQA attention) -> gemm (output projection)
// FFN phase:  k_rmsnorm_bf16 -> gemm (gate | up) -> k_swiglu -> gemm (down projection)
#include "prefill.hpp"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <type_traits>

#include "host_util.hpp"
#include "prof.hpp"

namespace tpi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short bf16_t;   // storage type

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((unsigned)v << 16); }

// Round to nearest even; NaN stays NaN.  The conversion is the hardware's (two values per instruction where the
// compiler can pair them), not integer arithmetic on the bits.
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));
}

__device__ __forceinline__ float wsum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------------------
// RMSNorm of n tokens: out[t][k] = bf16( x[t][k] / sqrt(mean_k x^2 + eps) * g[k] ).  One workgroup per token.
// ---------------------------------------------------------------------------
constexpr int kMaxPrefillShards = 16;   // == TPI_MAX_BATCH_SHARDS

// Shards of one batched call differ in their gains and in where the result goes; the input is shared.
struct NormArgs {
    const bf16_t *x;
    int h;
    float eps;
    const float *g[kMaxPrefillShards];
    bf16_t *out[kMaxPrefillShards];
};

__global__ __launch_bounds__(256) void k_rmsnorm_bf16(NormArgs a)
{
    const bf16_t *__restrict__ x = a.x;
    const float *__restrict__ g = a.g[blockIdx.y];
    bf16_t *__restrict__ out = a.out[blockIdx.y];
    const int h = a.h;
    const float eps = a.eps;
    // the first kKeep * 2048 elements of the row stay in registers between the two passes (rows up to
    // 8192 elements are read once); longer rows read the rest again
    constexpr int kKeep = 4;
    __shared__ float red[4];
    const bf16_t *xr = x + (size_t)blockIdx.x * h;
    bf16_t *orow = out + (size_t)blockIdx.x * h;
    uint4 keep[kKeep];
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const int k = (c * 256 + threadIdx.x) * 8;
        keep[c] = (k < h) ? *reinterpret_cast<const uint4 *>(xr + k) : make_uint4(0, 0, 0, 0);
    }
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const bf16_t *e = reinterpret_cast<const bf16_t *>(&keep[c]);
#pragma unroll
        for (int i = 0; i < 8; ++i) { float v = bf16_to_f32(e[i]); ss = fmaf(v, v, ss); }
    }
    for (int k = (kKeep * 256 + threadIdx.x) * 8; k < h; k += 256 * 8) {
        uint4 raw = *reinterpret_cast<const uint4 *>(xr + k);
        const bf16_t *e = reinterpret_cast<const bf16_t *>(&raw);
#pragma unroll
        for (int i = 0; i < 8; ++i) { float v = bf16_to_f32(e[i]); ss = fmaf(v, v, ss); }
    }
    ss = wsum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rinv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)h + eps);
    auto emit = [&](int k, const uint4 &raw) {
        const bf16_t *e = reinterpret_cast<const bf16_t *>(&raw);
        float4 g0 = *reinterpret_cast<const float4 *>(g + k), g1 = *reinterpret_cast<const float4 *>(g + k + 4);
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        uint4 o;
        bf16_t *oe = reinterpret_cast<bf16_t *>(&o);
#pragma unroll
        for (int i = 0; i < 8; ++i) oe[i] = f32_to_bf16(bf16_to_f32(e[i]) * rinv * gg[i]);
        *reinterpret_cast<uint4 *>(orow + k) = o;
    };
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const int k = (c * 256 + threadIdx.x) * 8;
        if (k < h) emit(k, keep[c]);
    }
    for (int k = (kKeep * 256 + threadIdx.x) * 8; k < h; k += 256 * 8) emit(k, *reinterpret_cast<const uint4 *>(xr + k));
}

// ---------------------------------------------------------------------------
// C[m][n] = sum_k A[m][k] * B[n][k]   (bf16 in, fp32 out; both operands K-contiguous)
// ---------------------------------------------------------------------------
// Rows n < n_split of B come from B0, the rest from B1 (gate | up share one launch).
// Workgroup tile BM x BN, 4 waves as 2 x 2, each wave (BM/2) x (BN/2) in 32x32 MFMA tiles.
// K advances in steps of 64.  Step t is multiplied out of LDS stage (t+1) & 1 while the global
// loads of steps t+1 .. t+NS sit in a ring of NS register sets (set = step % NS); at the end of
// the step, set (t+1) % NS goes to the other LDS stage, one workgroup barrier per step.  With
// one workgroup per compute unit nothing else hides the latency of HBM, hence the deep ring.
// An LDS row is 64 elements = 8 chunks of 16 bytes, stored at
// chunk position (chunk ^ (row & 7)): the fragment reads of 8 consecutive rows then cover all
// banks without padding.
// blockIdx.z selects shard and K range (split-K): split z writes its partial product to C + z * c_split
// and the consumer adds the partials in split order.
struct GemmPtrs {
    const bf16_t *A;
    const bf16_t *B0, *B1;
    float *C;
    bf16_t *act;              // SWI kernels only: output of the fused SwiGLU, n_split columns, rows ldc apart
};

// One launch covers the shards of a batched call: blockIdx.z = shard * splits + K split.
struct GemmArgs {
    int M, N, K, n_split;
    int lda, ldb, ldc;
    int k_per_split;          // multiple of 64
    int splits;
    size_t c_split;           // floats between the partial products of consecutive splits
    GemmPtrs p[kMaxPrefillShards];
};

// KW = 2: eight waves; waves 4..7 repeat the 2 x 2 arrangement and take the second half of every
// K-step (a second wave per SIMD, so one wave's LDS and barrier waits are covered by the other's
// MFMAs); at the end the two waves of a pair exchange halves of their accumulators through LDS and
// each finishes one of the pair's two row tiles.
//
// SWI: the gate | up product with SwiGLU (the activation of Eq. 2) applied to the accumulators.  Column
// tile x then covers hidden units 64x .. 64x+63 of BOTH matrices, arranged so that each wave's first
// 32x32 tile holds gate columns and its second the up columns of the same 32 units: the product
// silu(gate) * up is taken lane by lane in registers and only the bf16 activation [M][n_split] is
// written (no fp32 product in memory, no separate elementwise pass).
constexpr int kSwzShift = 1;

//
// DIRECT: the tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane), never
// through registers: no ds_write, no register ring, and the loads' data does not compete with the fragment
// reads for the way back into the register file.  Such a load writes the 64 lanes' 16 bytes to consecutive
// LDS addresses (8 rows of 8 chunks), so the swizzle moves to the global side: the lane at chunk position p
// of its row fetches K chunk p ^ swizzle(row).  Three LDS stages, each a static array of its own (the
// compiler then knows that a fragment read of one stage cannot meet a load in flight to another and adds no
// waits of its own); step t + 2 is requested at the start of step t, and the step ends with an explicit
// wait for step t + 1's loads of this wave followed by a bare workgroup barrier (a fence would wait for
// every load in flight).  Needs whole K-steps (K range a multiple of 64) and the eight-wave tiles.
// NS = 2 is the same with two stages (step t + 1 requested at the start of step t): half the LDS, so that two
// workgroups fit a compute unit.
// LEAVE_OUT is for the loop probe only (tpi_probe_gemm_loop): bit 0 the loads after the first fill of the stages,
// bit 1 the fragment reads, bit 2 the matrix instructions.  The product kernels are the instantiations with 0.
template <int BM, int BN, int NS, int KW, bool SWI = false, bool DIRECT = false, int WM = 2, int LEAVE_OUT = 0>
__global__ __launch_bounds__(128 * WM * KW) void k_gemm_bf16_nt(GemmArgs g)
{
    static_assert(LEAVE_OUT == 0 || (DIRECT && !SWI && KW == 1), "the probe variants exist for the direct loop of the plain product");
    // SWI with a tile whose two wave columns do not hold whole (gate, up) pairs of 32-column tiles (BN = 192): the
    // left wave column takes the gate rows of the tile's units, the right one their up rows, and the two waves of a
    // row exchange halves of their accumulators through LDS before the activation.
    constexpr bool SWI_SPLIT = SWI && BN % 128 != 0;
    static_assert(!SWI_SPLIT || (DIRECT && KW == 1 && BM / (32 * WM) == 2 && BN % 64 == 0),
                  "gate and up in different waves: eight waves of two row tiles each, stages as separate arrays");
    static_assert(!DIRECT || NS == 3 || NS == 2, "the direct loads are written for two or three stages");
    static_assert(!DIRECT || KW == 2 || NS == 2, "four waves: two stages, every load waited for in each step");
    constexpr int BK = 64, NT = 128 * WM * KW;          // WM x 2 waves, KW times
    constexpr int MI = BM / (32 * WM), NI = BN / 64;    // 32x32 tiles per wave along m and n
    static_assert(WM == 2 || KW == 1, "the exchange between the waves of a pair is written for 2 x 2 waves");
    constexpr int ACH = BM * (BK / 8) / NT;             // 16-byte chunks per thread, A tile
    constexpr int BCH = BN * (BK / 8) / NT;
    constexpr int STAGE = (BM + BN) * 8;                // chunks per stage
    static_assert(ACH >= 1 && BCH >= 1, "tile too small for the thread count");
    constexpr int NP = NI > 2 ? 2 : NI;                 // column tiles per pass of the accumulator exchange
    static_assert(KW == 1 || NI % NP == 0, "whole passes");
    static_assert(KW == 1 || 8 * NP * 16 * 64 * 4 <= 2 * STAGE * 16, "an exchange pass must fit the LDS stages");
    static_assert(!DIRECT || 8 * 16 * 64 * 4 <= STAGE * 16, "one column tile of an exchange pass per stage");
    extern __shared__ uint4 lds[];                      // 2 * STAGE chunks, sized at launch (not DIRECT)
    __shared__ uint4 stage_a[DIRECT ? STAGE : 1], stage_b[DIRECT ? STAGE : 1], stage_c[DIRECT && NS == 3 ? STAGE : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) % (2 * WM), kh = tid / (128 * WM);
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups are dealt to the eight compute dies in turn (linear index mod 8) and every die has its own L2,
    // so the tiles are renumbered: each die works through a contiguous run of (z, band of kRowBand row tiles,
    // column tile, row tile of the band) with the row tile running fastest -- the workgroups that share a B
    // tile, and the neighbours that share A tiles, meet in one L2 instead of fetching the same rows into
    // several, and with many row tiles (long prompts) a band's A tiles are reused across the column tiles
    // before the next band starts.
    constexpr int kRowBand = 8;
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    {
        const unsigned gx = gridDim.x, gy = gridDim.y, total = gx * gy * gridDim.z;
        if (total % 8 == 0) {
            const unsigned lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
            const unsigned item = (lin % 8) * (total / 8) + lin / 8;
            bz = item / (gx * gy);
            unsigned r = item - bz * gx * gy;
            const unsigned band = min(r / (kRowBand * gx), (gy - 1) / kRowBand);    // the last band may be short
            const unsigned first = band * kRowBand, rows = min((unsigned)kRowBand, gy - first);
            r -= band * kRowBand * gx;
            bx = r / rows;
            by = first + r % rows;
        }
    }
    const int m0 = by * BM, n0 = bx * BN;
    const int shard = bz / g.splits, zs = bz - shard * g.splits;
    const GemmPtrs P = g.p[shard];
    const int k_begin = zs * g.k_per_split, k_end = min(g.K, k_begin + g.k_per_split);
    float *C = P.C + (size_t)zs * g.c_split;

    // this thread's chunks: row c >> 3, chunk c & 7 of the A tile and of the B tile.  Loads are
    // unconditional (straight-line code keeps the ring's loads in flight across K-steps): rows past
    // the edge are clamped to the last row (their products are never written), chunks past the end
    // of K are clamped to the last chunk and replaced by zeros after the load.
    const bf16_t *pa[ACH], *pb[BCH];
    // K offset of this thread's chunk within a step; DIRECT: the chunk that belongs at LDS position tid & 7
    const int kc = DIRECT ? ((tid & 7) ^ ((tid >> (3 + kSwzShift)) & 7)) * 8 : (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        int m = min(m0 + ((tid + i * NT) >> 3), g.M - 1);
        pa[i] = P.A + (size_t)m * g.lda;
    }
    // row `within` (0 .. BN - 1) of this workgroup's B tile
    auto b_row_of = [&](int within) -> const bf16_t * {
        if constexpr (SWI_SPLIT) {
            // tile column -> gate (left wave column) or up (right wave column) row of unit bx * (BN / 2) + ...
            const int up = within / (BN / 2);
            const int unit = min(bx * (BN / 2) + within % (BN / 2), g.n_split - 1);
            return (up ? P.B1 : P.B0) + (size_t)unit * g.ldb;
        } else if constexpr (SWI) {
            // tile column -> wave half, pair of 32-column tiles (gate, up), unit within the pair
            const int wh = within / (BN / 2), t32 = (within % (BN / 2)) >> 5;
            const int unit = min(bx * (BN / 2) + wh * (BN / 4) + (t32 >> 1) * 32 + (within & 31), g.n_split - 1);
            return ((t32 & 1) ? P.B1 : P.B0) + (size_t)unit * g.ldb;
        } else {
            const int n = min(n0 + within, g.N - 1);
            return (n < g.n_split) ? P.B0 + (size_t)n * g.ldb : P.B1 + (size_t)(n - g.n_split) * g.ldb;
        }
    };
#pragma unroll
    for (int i = 0; i < BCH; ++i) pb[i] = b_row_of((tid + i * NT) >> 3);
    // (row * 8 + chunk) -> swizzled LDS position; row & 7 == (tid >> 3) & 7 for every i
    const int st_off = (tid >> 3) * 8 + ((tid & 7) ^ ((tid >> (3 + kSwzShift)) & 7));

    // Workgroups of different column tiles walk K from different starting steps (wrapping around), so
    // that at any moment the chip's loads are spread over the memory channels instead of all sitting at
    // the same offset of rows a power of two apart.  Only when the K range is whole steps.
    const int span = k_end - k_begin;
    const int rot = (span % BK == 0 && span >= 32 * BK) ? (bx % 16) * BK : 0;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int a = 0; a < MI; ++a)
#pragma unroll
        for (int b = 0; b < NI; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int fr = lane & 31, hb = lane >> 5, sw = (fr >> kSwzShift) & 7;
    const int a_row = (wm * (BM / WM) + fr) * 8, b_row = (BM + wn * (BN / 2) + fr) * 8;

    // the fragments of one K-step (this wave's half of it when KW = 2) out of an LDS stage
    auto multiply = [&](const uint4 *base) {
#pragma unroll
        for (int s0 = 0; s0 < BK / 16 / KW; ++s0) {
            bf16x8 fa[MI], fb[NI];
            const int s = kh * (BK / 16 / KW) + s0;
            const int ch = (2 * s + hb) ^ sw;
#pragma unroll
            for (int a = 0; a < MI; ++a) fa[a] = *reinterpret_cast<const bf16x8 *>(base + a_row + a * 32 * 8 + ch);
#pragma unroll
            for (int b = 0; b < NI; ++b) fb[b] = *reinterpret_cast<const bf16x8 *>(base + b_row + b * 32 * 8 + ch);
#pragma unroll
            for (int a = 0; a < MI; ++a)
#pragma unroll
                for (int b = 0; b < NI; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    };

    if constexpr (DIRECT) {
        const int nsteps = span / BK;                   // whole steps (the launcher checks)
        const int w64 = (tid >> 6) * 64;                // this wave's 8 rows of a 64-row slab, in chunks
        // s_waitcnt immediates: at most n vector memory loads in flight (bits 3:0 and 15:14), no wait on the export
        // counter (bits 6:4), every LDS read returned (bits 11:8)
        auto wait_for_all_but = [](int n) constexpr { return (n & 15) | ((n >> 4) << 14) | 0x0070; };
        constexpr int kWaitAll = wait_for_all_but(0);
        // One 16-byte-per-lane load from global memory into LDS: the 64 lanes' data go to consecutive LDS addresses
        // starting at `to` (the same for the whole wave; it travels in M0).  Written out as an instruction rather
        // than through the compiler's builtin: the compiler counts such a load as one that may return on either of
        // the memory and LDS counters and from then on waits for EVERY LDS read in flight wherever it needs one of
        // them, which would undo the read-ahead below.  The waits that these loads need are the explicit ones of
        // this loop (the count of loads in flight before a barrier, all of them at the end).
        auto lds_address = [](const uint4 *p) { return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void *)p; };
        const unsigned w64_bytes = __builtin_amdgcn_readfirstlane(w64 * 16);     // the same for the whole wave: a scalar
        auto load_to_lds = [&](const bf16_t *from, unsigned at) {
            unsigned keep;      // M0 belongs to the compiler: it is put back before the statement ends
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "v"(from), "s"(at) : "memory");
        };
        auto request = [&](const uint4 *stage, int t) {
            if constexpr ((LEAVE_OUT & 1) != 0) {
                if (t >= NS) { __builtin_amdgcn_sched_barrier(0); return; }
            }
            int kk = k_begin + t * BK + rot;
            if (kk >= k_end) kk -= span;
            const int ko = kk + kc;
            const unsigned at = lds_address(stage) + w64_bytes;
#pragma unroll
            for (int i = 0; i < ACH; ++i) load_to_lds(pa[i] + ko, at + i * NT * 16);
#pragma unroll
            for (int i = 0; i < BCH; ++i) load_to_lds(pb[i] + ko, at + (BM * 8 + i * NT) * 16);
            __builtin_amdgcn_sched_barrier(0);          // keep the requests ahead of the step's arithmetic
        };
        // A step is four 16-wide slices; a wave multiplies SL of them (its half of the step with eight waves,
        // all four with four waves).  The fragments of a slice are read from LDS one slice ahead of the matrix
        // instructions that use them, into a second set of registers: while the matrix cores work through the
        // products of one slice, the next slice's reads are already on their way, also across the barrier between
        // two steps -- the first slice of step t + 1 is read right after the barrier that makes step t + 1 visible
        // and is used only after the last slice of step t has been multiplied.  The order of the products per
        // accumulator is unchanged.
        constexpr int SL = BK / 16 / KW;
        static_assert(SL == 2 || SL == 4, "an even number of slices: the two fragment sets alternate");
        bf16x8 fa0[MI], fb0[NI], fa1[MI], fb1[NI];
        if constexpr ((LEAVE_OUT & 2) != 0) {       // never read: give the fragments a value
#pragma unroll
            for (int a = 0; a < MI; ++a) fa0[a] = fa1[a] = *reinterpret_cast<const bf16x8 *>(P.A + (size_t)lane * 8);
#pragma unroll
            for (int b = 0; b < NI; ++b) fb0[b] = fb1[b] = *reinterpret_cast<const bf16x8 *>(P.B0 + (size_t)lane * 8);
        }
        auto read_slice = [&](const uint4 *base, int s0, bf16x8 (&fa)[MI], bf16x8 (&fb)[NI]) {
            if constexpr ((LEAVE_OUT & 2) != 0) { __builtin_amdgcn_sched_barrier(0); return; }
            const int ch = (2 * (kh * SL + s0) + hb) ^ sw;
#pragma unroll
            for (int a = 0; a < MI; ++a) fa[a] = *reinterpret_cast<const bf16x8 *>(base + a_row + a * 32 * 8 + ch);
#pragma unroll
            for (int b = 0; b < NI; ++b) fb[b] = *reinterpret_cast<const bf16x8 *>(base + b_row + b * 32 * 8 + ch);
            __builtin_amdgcn_sched_barrier(0);          // the reads stay ahead of the products that follow
        };
        auto multiply_slice = [&](const bf16x8 (&fa)[MI], const bf16x8 (&fb)[NI]) {
#pragma unroll
            for (int a = 0; a < MI; ++a)
#pragma unroll
                for (int b = 0; b < NI; ++b) {
                    if constexpr ((LEAVE_OUT & 4) != 0) {   // keep the fragments alive with one addition per product
                        union { bf16x8 v; float f[4]; } ua, ub;
                        ua.v = fa[a]; ub.v = fb[b];
                        acc[a][b][0] += ua.f[0] + ub.f[1] + ua.f[2] + ub.f[3];
                    } else {
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        };
        // Step t out of `cur`; its first slice is in fa0 / fb0 already.  Before the barrier this wave's loads of
        // step t + 1 have landed (kWaitStep leaves the younger requests in flight) and its reads of `cur` have
        // returned; after the barrier everybody's, so `cur` is free and takes step t + NS at once -- a request has
        // NS - 1 whole steps to land -- and the first slice of step t + 1 is read from `nxt`.
        // The last steps request the last step once more (cache hits into a free stage) instead of nothing, so
        // that the count of loads in flight is the same at every wait; the slice read after the last step's
        // barrier comes from such a repeat and is not used.
        constexpr int kWaitStep = wait_for_all_but((NS - 2) * (ACH + BCH)), kWaitFirst = wait_for_all_but((NS - 1) * (ACH + BCH));
        static_assert((NS - 1) * (ACH + BCH) <= 63, "the count of loads in flight has six bits in the immediate");
        auto direct_step = [&](uint4 *cur, const uint4 *nxt, int t) {
            read_slice(cur, 1, fa1, fb1);
            multiply_slice(fa0, fb0);
            if constexpr (SL == 4) {
                read_slice(cur, 2, fa0, fb0);
                multiply_slice(fa1, fb1);
                read_slice(cur, 3, fa1, fb1);
                multiply_slice(fa0, fb0);
            }
            __builtin_amdgcn_s_waitcnt(kWaitStep);
            __builtin_amdgcn_s_barrier();
            request(cur, min(t + NS, nsteps - 1));
            read_slice(nxt, 0, fa0, fb0);
            multiply_slice(fa1, fb1);
        };
        request(stage_a, 0);
        request(stage_b, min(1, nsteps - 1));
        if constexpr (NS == 3) request(stage_c, min(2, nsteps - 1));
        __builtin_amdgcn_s_waitcnt(kWaitFirst);
        __builtin_amdgcn_s_barrier();
        read_slice(stage_a, 0, fa0, fb0);
        // whole rounds of NS steps (a loop with exits between the steps makes the compiler add waits of its own at
        // its head); every round ends where it began, so the steps left over start in the first stage again
        int t = 0;
        if constexpr (NS == 2) {
            for (; t + 2 <= nsteps; t += 2) {
                direct_step(stage_a, stage_b, t);
                direct_step(stage_b, stage_a, t + 1);
            }
            if (t < nsteps) direct_step(stage_a, stage_b, t++);
        } else {
            for (; t + 3 <= nsteps; t += 3) {
                direct_step(stage_a, stage_b, t);
                direct_step(stage_b, stage_c, t + 1);
                direct_step(stage_c, stage_a, t + 2);
            }
            if (t < nsteps) direct_step(stage_a, stage_b, t++);
            if (t < nsteps) direct_step(stage_b, stage_c, t++);
        }
        __builtin_amdgcn_s_waitcnt(kWaitAll);           // the repeated requests and the unused slice, before the stages are reused
        __builtin_amdgcn_s_barrier();
    } else {
        uint4 ring[NS][ACH + BCH];
        auto load_tiles = [&](auto J, int k0) {
            constexpr int j = decltype(J)::value;
            int kk = k0 + rot;
            if (kk >= k_end) kk -= span;
            const int ko = min(kk + kc, g.K - 8);
    #pragma unroll
            for (int i = 0; i < ACH; ++i) ring[j][i] = *reinterpret_cast<const uint4 *>(pa[i] + ko);
    #pragma unroll
            for (int i = 0; i < BCH; ++i) ring[j][ACH + i] = *reinterpret_cast<const uint4 *>(pb[i] + ko);
        };
        // k0: the K-step the set was loaded for.  In a step that reaches past k_end the chunks of A at or
        // past k_end become zeros (B stays as loaded: finite values times zero); this happens here, where
        // the loaded value is needed anyway (touching it earlier would wait for the load).
        auto store_tiles = [&](auto J, int stage, int k0) {
            constexpr int j = decltype(J)::value;
            uint4 *base = lds + stage * STAGE;
            if (k0 + BK > k_end) {
                const unsigned keep = (k0 + kc < k_end) ? 0xffffffffu : 0u;
    #pragma unroll
                for (int i = 0; i < ACH; ++i) {
                    const uint4 v = ring[j][i];
                    base[st_off + i * NT] = make_uint4(v.x & keep, v.y & keep, v.z & keep, v.w & keep);
                }
            } else {
    #pragma unroll
                for (int i = 0; i < ACH; ++i) base[st_off + i * NT] = ring[j][i];
            }
    #pragma unroll
            for (int i = 0; i < BCH; ++i) base[BM * 8 + st_off + i * NT] = ring[j][ACH + i];
        };

        // multiplies the K-step at k0 = step t, with J = (t + 1) % NS: set J - 1 (step t, already in LDS) is
        // free and takes step t + NS; set J (step t + 1) goes to LDS afterwards
        auto step = [&](auto J, int k0) {
            constexpr int j = decltype(J)::value;
            constexpr int stage = j & 1;
            load_tiles(std::integral_constant<int, (j + NS - 1) % NS>{}, k0 + NS * BK);
            multiply(lds + stage * STAGE);
            store_tiles(J, stage ^ 1, k0 + BK);   // the other stage was last read before the previous barrier
            __syncthreads();
        };

        // sets 0 .. NS-1 <- steps 0 .. NS-1, step 0 on to LDS stage 1
        static_assert(NS % 2 == 0, "LDS stage parity follows the ring index");
        auto prologue = [&](auto self, auto I) {
            constexpr int i = decltype(I)::value;
            if constexpr (i < NS) {
                load_tiles(I, k_begin + i * BK);
                self(self, std::integral_constant<int, i + 1>{});
            }
        };
        prologue(prologue, std::integral_constant<int, 0>{});
        store_tiles(std::integral_constant<int, 0>{}, 1, k_begin);
        __syncthreads();
        // always whole rounds of NS steps (no exits inside the round: straight-line code keeps the waits on
        // the ring exact); steps past k_end multiply zeros
        auto round = [&](auto self, auto I, int k0) {
            constexpr int i = decltype(I)::value;
            if constexpr (i < NS) {
                step(std::integral_constant<int, (i + 1) % NS>{}, k0 + i * BK);
                self(self, std::integral_constant<int, i + 1>{}, k0);
            }
        };
        for (int k0 = k_begin; k0 < k_end; k0 += NS * BK) round(round, std::integral_constant<int, 0>{}, k0);

    }

    // KW = 2: the two waves of a pair hold partial sums of the same tiles.  Wave kh hands the other its
    // partial of row tile 1 - kh through LDS (NP column tiles per pass) and finishes row tile kh, so all
    // eight waves share the stores.
    // column tile b of a pass goes through its own 32 KB: the first two stages when they are separate arrays
    float *const xch[2] = {reinterpret_cast<float *>(DIRECT ? stage_a : lds),
                           reinterpret_cast<float *>(DIRECT ? stage_b : lds + 8 * 16 * 64 / 4)};
    auto give = [&](auto A, auto B0) {
        constexpr int a = decltype(A)::value, b0 = decltype(B0)::value;
#pragma unroll
        for (int b = 0; b < NP; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) xch[b][((wave * 2 + a) * 16 + r) * 64 + lane] = acc[a][b0 + b][r];
    };
    auto take = [&](auto A, auto B0) {
        constexpr int a = decltype(A)::value, b0 = decltype(B0)::value;
#pragma unroll
        for (int b = 0; b < NP; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b0 + b][r] += xch[b][((wave * 2 + a) * 16 + r) * 64 + lane];
    };
    // accumulator register r of lane l is element (8*(r/4) + 4*(l/32) + r%4, l%32) of its 32x32 tile
    auto finish = [&](auto A) {
        constexpr int a = decltype(A)::value;
        if constexpr (SWI) {
#pragma unroll
            for (int c = 0; c < NI / 2; ++c) {
                const int unit = bx * (BN / 2) + wn * (BN / 4) + c * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = m0 + wm * (BM / WM) + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const float gt = acc[a][2 * c][r], up = acc[a][2 * c + 1][r];
                    if (row < g.M && unit < g.n_split) P.act[(size_t)row * g.ldc + unit] = f32_to_bf16(gt / (1.0f + expf(-gt)) * up);
                }
            }
        } else {
#pragma unroll
            for (int b = 0; b < NI; ++b) {
                int col = n0 + wn * (BN / 2) + b * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = m0 + wm * (BM / WM) + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row < g.M && col < g.N) C[(size_t)row * g.ldc + col] = acc[a][b][r];
                }
            }
        }
    };
    if constexpr (KW == 2) {
        static_assert(MI == 2, "one row tile per wave of a pair");
        static_assert(NI <= 2 * NP, "at most two passes");
        // the K loop ended with a barrier: the stages are free
        if (kh == 0) give(std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
        else give(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        __syncthreads();
        if (kh == 0) take(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        else take(std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
        if constexpr (NI > NP) {
            __syncthreads();                    // the first pass has been read
            if (kh == 0) give(std::integral_constant<int, 1>{}, std::integral_constant<int, NP>{});
            else give(std::integral_constant<int, 0>{}, std::integral_constant<int, NP>{});
            __syncthreads();
            if (kh == 0) take(std::integral_constant<int, 0>{}, std::integral_constant<int, NP>{});
            else take(std::integral_constant<int, 1>{}, std::integral_constant<int, NP>{});
        }
        if (kh == 0) finish(std::integral_constant<int, 0>{});
        else finish(std::integral_constant<int, 1>{});
    } else if constexpr (SWI_SPLIT) {
        // Wave (wm, 0) holds the gate sums of its 64 rows x BN / 2 units, wave (wm, 1) the up sums.  Each hands the
        // other one of its two row tiles (the left wave its second, the right wave its first) and finishes the row
        // tile it kept: the stores are shared by all eight waves.  The K loop ended with a barrier: the stages are
        // free; a wave's slot is NI tiles of 16 x 64 floats, waves 0..3 in the first stage, 4..7 in the second.
        constexpr int kSlot = NI * 16 * 64;
        static_assert(4 * kSlot * 4 <= STAGE * 16, "four waves' slots per stage");
        auto slot_of = [&](int w) { return reinterpret_cast<float *>(w < 4 ? stage_a : stage_b) + (w & 3) * kSlot; };
        float *mine = slot_of(wave);
        const float *theirs = slot_of(wave ^ 1);
        auto hand_over = [&](auto A) {
            constexpr int a = decltype(A)::value;
#pragma unroll
            for (int b = 0; b < NI; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) mine[(b * 16 + r) * 64 + lane] = acc[a][b][r];
        };
        if (wn == 0) hand_over(std::integral_constant<int, 1>{});
        else hand_over(std::integral_constant<int, 0>{});
        __syncthreads();
        auto activate = [&](auto A) {
            constexpr int a = decltype(A)::value;       // the row tile this wave kept: gate if a == 0, up if a == 1
#pragma unroll
            for (int b = 0; b < NI; ++b) {
                const int unit = bx * (BN / 2) + b * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wm * (BM / WM) + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    const float other = theirs[(b * 16 + r) * 64 + lane];
                    const float gt = a == 0 ? acc[a][b][r] : other, up = a == 0 ? other : acc[a][b][r];
                    if (row < g.M && unit < g.n_split) P.act[(size_t)row * g.ldc + unit] = f32_to_bf16(gt / (1.0f + expf(-gt)) * up);
                }
            }
        };
        if (wn == 0) activate(std::integral_constant<int, 0>{});
        else activate(std::integral_constant<int, 1>{});
    } else {
        finish(std::integral_constant<int, 0>{});
        if constexpr (MI >= 2) finish(std::integral_constant<int, 1>{});
        if constexpr (MI >= 3) finish(std::integral_constant<int, 2>{});
        if constexpr (MI >= 4) finish(std::integral_constant<int, 3>{});
    }
}

// ---------------------------------------------------------------------------
// Rotary embedding + cache fill from the fp32 QKV product
// ---------------------------------------------------------------------------
// One thread per (token, head slot, pair index e); head slots are the nq query heads, the nkv key heads and
// the nkv value heads.  Query and key slots rotate element pair (e, e + d/2) at position pos0 + token (angle
// in fp64); q goes out as bf16 [n][nq*d], K and V into cache slot pos0 + token.
// The QKV product arrives as n_parts split-K partials, part_stride floats apart, added in split order.
// blockIdx.y selects the shard of a batched call.
struct RopeArgs {
    int n_parts;
    size_t part_stride;
    int n, nq, nkv, d, max_seq, pos0;
    double log2_base;
    const float *qkv[kMaxPrefillShards];
    bf16_t *q_out[kMaxPrefillShards], *Kc[kMaxPrefillShards], *Vc[kMaxPrefillShards];
};

__global__ __launch_bounds__(256) void k_rope_scatter(RopeArgs a)
{
    const float *__restrict__ qkv = a.qkv[blockIdx.y];
    bf16_t *__restrict__ q_out = a.q_out[blockIdx.y];
    bf16_t *__restrict__ Kc = a.Kc[blockIdx.y];
    bf16_t *__restrict__ Vc = a.Vc[blockIdx.y];
    const int n_parts = a.n_parts, n = a.n, nq = a.nq, nkv = a.nkv, d = a.d, max_seq = a.max_seq, pos0 = a.pos0;
    const size_t part_stride = a.part_stride;
    const double log2_base = a.log2_base;
    const int half = d / 2, nh = nq + 2 * nkv;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * nh * half) return;
    const int e = idx % half, hs = (idx / half) % nh, t = idx / (half * nh);
    const int pos = pos0 + t;
    const float *row0 = qkv + (size_t)t * nh * d + (size_t)hs * d;
    float lo = row0[e], hi = row0[e + half];
    for (int p = 1; p < n_parts; ++p) {
        lo += row0[(size_t)p * part_stride + e];
        hi += row0[(size_t)p * part_stride + e + half];
    }
    if (hs >= nq + nkv) {
        const size_t slot = ((size_t)(hs - nq - nkv) * max_seq + pos) * d;
        Vc[slot + e] = f32_to_bf16(lo);
        Vc[slot + e + half] = f32_to_bf16(hi);
        return;
    }
    float cs = 1.f, sn = 0.f;
    if (pos != 0) {
        double theta = exp2(-(2.0 * (double)e / (double)d) * log2_base);
        double sd, cd;
        sincos((double)pos * theta, &sd, &cd);
        cs = (float)cd;
        sn = (float)sd;
    }
    const bf16_t rlo = f32_to_bf16(lo * cs - hi * sn), rhi = f32_to_bf16(hi * cs + lo * sn);
    if (hs < nq) {
        q_out[((size_t)t * nq + hs) * d + e] = rlo;
        q_out[((size_t)t * nq + hs) * d + e + half] = rhi;
    } else {
        const size_t slot = ((size_t)(hs - nq) * max_seq + pos) * d;
        Kc[slot + e] = rlo;
        Kc[slot + e + half] = rhi;
    }
}

// act[t][j] = bf16( silu(gu[t][j]) * gu[t][sl + j] )
__global__ __launch_bounds__(256) void k_swiglu(const float *__restrict__ gu, bf16_t *__restrict__ act, int n, int sl)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * sl) return;
    const size_t t = idx / sl, j = idx - t * sl;
    float gt = gu[t * 2 * sl + j], up = gu[t * 2 * sl + sl + j];
    act[idx] = f32_to_bf16(gt / (1.0f + expf(-gt)) * up);
}

// ---------------------------------------------------------------------------
// Causal GQA attention over the bf16 cache (vector ALUs, fp32 arithmetic)
// ---------------------------------------------------------------------------
// One workgroup = one KV head x QT consecutive tokens; its rows are the (token, query head of the group)
// pairs, R = QT * G <= 64.  Keys and values pass through LDS in tiles of 64 slots; thread (r, c) with
// r = tid / 4 (row) and c = tid % 4 owns the scores of row r against slots c, c+4, ... of the tile and a
// quarter of the row's output vector; the running softmax state of a row lives in the registers of its 4
// threads.  Token i attends to slots 0 .. pos0 + i.
template <int DMAX>
__global__ __launch_bounds__(256) void k_prefill_attn(const bf16_t *__restrict__ q, const bf16_t *__restrict__ Kc,
                                                      const bf16_t *__restrict__ Vc, bf16_t *__restrict__ o, int n,
                                                      int nq, int nkv, int d, int max_seq, int pos0, int QT)
{
    constexpr int TK = 64;
    constexpr int DQ = DMAX / 4;                       // output elements per thread
    extern __shared__ float smem[];
    float *Ks = smem;                                  // [TK][d + 1]
    float *Vs = Ks + TK * (d + 1);                     // [TK][d]
    float *Qs = Vs + TK * d;                           // [64][d + 1]
    float *Ps = Qs + 64 * (d + 1);                     // [64][TK + 1]

    const int G = nq / nkv;
    const int gk = blockIdx.y;
    const int t_first = blockIdx.x * QT;
    const int tid = threadIdx.x, r = tid >> 2, c = tid & 3;
    const int R = QT * G;
    const int tok = t_first + r / G, hd = gk * G + r % G;
    const bool row_ok = r < R && tok < n;
    const float scale = 1.0f / sqrtf((float)d);

    for (int i = tid; i < 64 * d; i += 256) {
        int rr = i / d, e = i - rr * d;
        int tk = t_first + rr / G, hh = gk * G + rr % G;
        float v = 0.f;
        if (rr < R && tk < n) v = bf16_to_f32(q[(size_t)tk * nq * d + (size_t)hh * d + e]) * scale;
        Qs[rr * (d + 1) + e] = v;
    }
    float m_run = -INFINITY, l_run = 0.f;
    float acc[DQ];
#pragma unroll
    for (int i = 0; i < DQ; ++i) acc[i] = 0.f;
    const int last_tok = min(t_first + QT, n) - 1;
    const int n_keys = pos0 + last_tok + 1;            // slots any row of this workgroup may see
    const int my_last = pos0 + tok;                    // last slot this row sees
    const bf16_t *Kg = Kc + (size_t)gk * max_seq * d;
    const bf16_t *Vg = Vc + (size_t)gk * max_seq * d;
    const int dq4 = d / 4;                             // elements of the output this thread owns: [c*dq4, (c+1)*dq4)

    for (int k0 = 0; k0 < n_keys; k0 += TK) {
        __syncthreads();
        for (int i = tid; i < TK * d; i += 256) {
            int s = i / d, e = i - s * d;
            bool ok = k0 + s < n_keys;
            Ks[s * (d + 1) + e] = ok ? bf16_to_f32(Kg[(size_t)(k0 + s) * d + e]) : 0.f;
            Vs[s * d + e] = ok ? bf16_to_f32(Vg[(size_t)(k0 + s) * d + e]) : 0.f;
        }
        __syncthreads();
        // scores of this row against slots c, c+4, ...
        float sc[TK / 4];
#pragma unroll
        for (int j = 0; j < TK / 4; ++j) sc[j] = 0.f;
        for (int e = 0; e < d; ++e) {
            float qv = Qs[r * (d + 1) + e];
#pragma unroll
            for (int j = 0; j < TK / 4; ++j) sc[j] = fmaf(qv, Ks[(c + 4 * j) * (d + 1) + e], sc[j]);
        }
        float mt = -INFINITY;
#pragma unroll
        for (int j = 0; j < TK / 4; ++j) {
            int slot = k0 + c + 4 * j;
            if (!row_ok || slot > my_last) sc[j] = -INFINITY;
            mt = fmaxf(mt, sc[j]);
        }
        mt = fmaxf(mt, __shfl_xor(mt, 1, 64));
        mt = fmaxf(mt, __shfl_xor(mt, 2, 64));
        const float m_new = fmaxf(m_run, mt);
        float ls = 0.f;
#pragma unroll
        for (int j = 0; j < TK / 4; ++j) {
            float p = (sc[j] == -INFINITY) ? 0.f : expf(sc[j] - m_new);
            ls += p;
            Ps[r * (TK + 1) + c + 4 * j] = p;
        }
        ls += __shfl_xor(ls, 1, 64);
        ls += __shfl_xor(ls, 2, 64);
        const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
        l_run = l_run * alpha + ls;
        m_run = (m_new == -INFINITY) ? m_run : m_new;
#pragma unroll
        for (int i = 0; i < DQ; ++i) acc[i] *= alpha;
        __syncthreads();                               // a row's P entries come from its 4 threads
        for (int s = 0; s < TK; ++s) {
            float p = Ps[r * (TK + 1) + s];
#pragma unroll
            for (int i = 0; i < DQ; ++i)
                if (i < dq4) acc[i] = fmaf(p, Vs[s * d + c * dq4 + i], acc[i]);
        }
    }
    if (row_ok) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int i = 0; i < DQ; ++i)
            if (i < dq4) o[(size_t)tok * nq * d + (size_t)hd * d + c * dq4 + i] = f32_to_bf16(acc[i] * inv);
    }
}

// ---------------------------------------------------------------------------
// Causal GQA attention on the matrix cores (head_dim a multiple of 32, at most 128)
// ---------------------------------------------------------------------------
// Rows are the (token, query head of the group) pairs of one KV head, row = token * G + head.
// A workgroup owns 32 rows; its four waves share them and split the key tiles (32 slots each,
// tile t goes to wave t % 4), each with a running softmax of its own, merged through LDS at the end.
//
// Scores are formed transposed, S^T[key][row] = K . Q^T: both operands are then read along the
// head dimension, straight from global memory, and a lane ends up with 16 scores of ONE row
// (its column), so the running softmax is in-lane work plus one exchange between the two
// half-waves.  O^T[e][row] += V^T[e][key] . P^T[key][row]: P^T is exactly the score registers
// (cast to bf16), no data movement; V^T is read from a per-wave LDS tile laid out
// [key / 4][e][key % 4], in the key order the score registers hold (the contraction index may be
// permuted as long as both operands agree).
// blockIdx.z selects the shard of a batched call.
struct AttnArgs {
    int n, nq, nkv, max_seq, pos0;
    const bf16_t *q[kMaxPrefillShards], *Kc[kMaxPrefillShards], *Vc[kMaxPrefillShards];
    bf16_t *o[kMaxPrefillShards];
};

template <int D>
__global__ __launch_bounds__(256) void k_prefill_attn_mfma(AttnArgs a)
{
    const bf16_t *__restrict__ q = a.q[blockIdx.z];
    const bf16_t *__restrict__ Kc = a.Kc[blockIdx.z];
    const bf16_t *__restrict__ Vc = a.Vc[blockIdx.z];
    bf16_t *__restrict__ o = a.o[blockIdx.z];
    const int n = a.n, nq = a.nq, nkv = a.nkv, max_seq = a.max_seq, pos0 = a.pos0;
    constexpr int ET = D / 32, KS = D / 16, TK = 32;
    constexpr int VT = (TK / 4) * D * 4;                          // bf16 elements of one V tile
    constexpr int MERGE = 3 * ET * 16 * 64;                       // floats: three foreign shares of every output tile
    constexpr int LDS_BYTES = (4 * VT * 2 > MERGE * 4) ? 4 * VT * 2 : MERGE * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[LDS_BYTES];
    __shared__ float ml[2][4][32];                                // running max and sum of every wave's rows

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hb = lane >> 5;
    const int G = nq / nkv, gk = blockIdx.y;
    const int n_rows = n * G;
    const int row = blockIdx.x * 32 + col;                        // this lane's row (a column of S^T)
    const bool row_ok = row < n_rows;
    const int tok = row_ok ? row / G : n - 1, head = gk * G + (row_ok ? row % G : 0);
    const int my_last = pos0 + tok;                               // last slot this row attends to
    const int wg_last_key = pos0 + min(n - 1, (blockIdx.x * 32 + 31) / G);
    const float scale = 1.0f / sqrtf((float)D);
    const bf16_t *Kg = Kc + (size_t)gk * max_seq * D;
    const bf16_t *Vg = Vc + (size_t)gk * max_seq * D;
    bf16_t *Vt = reinterpret_cast<bf16_t *>(smem) + wave * VT;

    bf16x8 qf[KS];
    {
        const bf16_t *qp = q + ((size_t)tok * nq + head) * D + hb * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }
    f32x16 oacc[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[et][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // Loads of one key tile, always in bounds (slots past the workgroup's last key are clamped to it; their
    // probabilities are zero).  K: the lane's MFMA fragments, rows of the MFMA = keys k0 .. k0+31.  V: lane =
    // output element e (EP passes of 64), one 16-bit load per key, coalesced across the wave, packed in
    // pairs of keys: what the lane then writes to LDS is already transposed.
    constexpr int EP = (D + 63) / 64;
    bf16x8 kf_next[KS];
    unsigned v_next[EP][TK];      // raw 16-bit loads; packed only where they are stored (no use next to the loads)
    auto fetch = [&](int k0) {
        const int key = min(k0 + col, wg_last_key);
        const bf16_t *kp = Kg + (size_t)key * D + hb * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf_next[ks] = *reinterpret_cast<const bf16x8 *>(kp + ks * 16);
#pragma unroll
        for (int ep = 0; ep < EP; ++ep) {
            const int e = min(ep * 64 + lane, D - 1);
#pragma unroll
            for (int j = 0; j < TK; ++j) v_next[ep][j] = Vg[(size_t)min(k0 + j, wg_last_key) * D + e];
        }
    };
    if (wave * TK <= wg_last_key) fetch(wave * TK);

    for (int k0 = wave * TK; k0 <= wg_last_key; k0 += 4 * TK) {
        bf16x8 kf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = kf_next[ks];
        // V tile -> this wave's LDS tile [key / 4][e][key % 4].  Only this wave touches the tile and a wave's
        // LDS operations complete in order, so no workgroup barrier is needed around it.
#pragma unroll
        for (int ep = 0; ep < EP; ++ep) {
            const int e = ep * 64 + lane;
            if (e < D) {
#pragma unroll
                for (int kg = 0; kg < TK / 4; ++kg)
                    *reinterpret_cast<uint2 *>(Vt + (kg * D + e) * 4) =
                        make_uint2(v_next[ep][4 * kg] | (v_next[ep][4 * kg + 1] << 16),
                                   v_next[ep][4 * kg + 2] | (v_next[ep][4 * kg + 3] << 16));
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        fetch(min(k0 + 4 * TK, wg_last_key));                     // next round's tile, in flight during this one

        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], sacc, 0, 0, 0);
        // register r of this lane: key k0 + 8*(r/4) + 4*hb + r%4, row = this lane's column
        float mt = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int key = k0 + 8 * (r >> 2) + 4 * hb + (r & 3);
            float sv = (key <= my_last) ? sacc[r] * scale : -INFINITY;
            sacc[r] = sv;
            mt = fmaxf(mt, sv);
        }
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));                   // the other half-wave holds the row's other keys
        const float m_new = fmaxf(m_run, mt);
        float ls = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = (sacc[r] == -INFINITY) ? 0.f : __expf(sacc[r] - m_new);
            sacc[r] = p;
            ls += p;
        }
        ls += __shfl_xor(ls, 32, 64);
        const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
        l_run = l_run * alpha + ls;
        m_run = m_new;
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[et][r] *= alpha;
        // P^T fragments: registers 8s .. 8s+7 are the 8 keys this half-wave contributes to MFMA step s
        bf16x8 pf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            union { bf16x8 v; bf16_t u[8]; } cvt;
#pragma unroll
            for (int i = 0; i < 8; ++i) cvt.u[i] = f32_to_bf16(sacc[8 * s2 + i]);
            pf[s2] = cvt.v;
        }
#pragma unroll
        for (int et = 0; et < ET; ++et) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                // element i of the fragment: key 16*s2 + 8*(i/4) + 4*hb + i%4 -> groups 4*s2 + hb and 4*s2 + 2 + hb
                union { bf16x8 v; uint2 h[2]; } vf;
                const int e = et * 32 + col;
                vf.h[0] = *reinterpret_cast<const uint2 *>(Vt + ((4 * s2 + hb) * D + e) * 4);
                vf.h[1] = *reinterpret_cast<const uint2 *>(Vt + ((4 * s2 + 2 + hb) * D + e) * 4);
                oacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[s2], oacc[et], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the tile is rewritten by the next round
        __builtin_amdgcn_wave_barrier();
    }

    // merge the four waves: common maximum, rescale, waves 1..3 hand their partial outputs to wave 0
    if (hb == 0) { ml[0][wave][col] = m_run; ml[1][wave][col] = l_run; }
    __syncthreads();                                              // also: every wave is done with its V tile
    float m_all = fmaxf(fmaxf(ml[0][0][col], ml[0][1][col]), fmaxf(ml[0][2][col], ml[0][3][col]));
    float l_all = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float mw = ml[0][w][col];
        l_all += (mw == -INFINITY) ? 0.f : ml[1][w][col] * __expf(mw - m_all);
    }
    const float mine = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_all);
    // output tile et (32 elements of every row) is finished by wave et: the other three waves hand it their
    // share through LDS, slot [et][p], p = the source wave's rank among the waves other than et
    float *mg = reinterpret_cast<float *>(smem);
#pragma unroll
    for (int et = 0; et < ET; ++et) {
        if (wave != et) {
            const int pslot = et * 3 + (wave < et ? wave : wave - 1);
#pragma unroll
            for (int r = 0; r < 16; ++r) mg[(pslot * 16 + r) * 64 + lane] = oacc[et][r] * mine;
        }
    }
    __syncthreads();
#pragma unroll
    for (int et = 0; et < ET; ++et) {
        if (wave == et && row_ok) {
            const float inv = 1.0f / l_all;
            bf16_t *op = o + ((size_t)tok * nq + head) * D;
            float part[3][16];
#pragma unroll
            for (int w = 0; w < 3; ++w)
#pragma unroll
                for (int r = 0; r < 16; ++r) part[w][r] = mg[((et * 3 + w) * 16 + r) * 64 + lane];
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                // registers 4*r4 .. 4*r4+3: elements e = 32*et + 8*r4 + 4*hb + 0..3
                union { uint2 v; bf16_t u[4]; } pk;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 4 * r4 + i;
                    pk.u[i] = f32_to_bf16((oacc[et][r] * mine + part[0][r] + part[1][r] + part[2][r]) * inv);
                }
                *reinterpret_cast<uint2 *>(op + 32 * et + 8 * r4 + 4 * hb) = pk.v;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same attention with the key and value tiles shared by 128 rows (head_dim 64 or 128)
// ---------------------------------------------------------------------------
// A workgroup owns 128 consecutive rows of one KV head, 32 per wave; every wave walks ALL key tiles its rows can
// see, against tiles that the workgroup brings into LDS once (global_load_lds, three stages, as in the GEMM):
// a quarter of the traffic per row of the kernel above, and no merge of the waves at the end.  Scores
// transposed as above, K fragments read from LDS rows swizzled against bank conflicts, and the V^T fragments
// come out of the row-major V tile through the transposing LDS read (ds_read_b64_tr_b16: in a group of 16
// lanes, lane 4i + j receives element j of the 8-byte pieces that lanes i, i + 4, i + 8, i + 12 point at --
// with lane s pointing at key s / 4, elements 4 (s % 4) .. + 3, lane l ends up with 4 consecutive keys of
// element l).  Workgroups with the longest rows come first in the grid.
typedef short tr16x4 __attribute__((ext_vector_type(4)));

template <int D>
__global__ __launch_bounds__(256, 2) void k_prefill_attn_shared(AttnArgs a)
{
    static_assert(D == 64 || D == 128, "tile loads are laid out for these head sizes");
    constexpr int ET = D / 32, KS = D / 16, TK = 32;
    constexpr int CPR = D / 8;                                   // 16-byte chunks per row
    constexpr int TILE = TK * CPR;                               // chunks per K or V tile
    constexpr int NLD = TILE / 64 / 4;                           // loads per wave per tile (K, and again V)
    constexpr int kWaitNext = 0x0070 | (2 * NLD), kWaitAll = 0x0070;
    __shared__ uint4 k_a[TILE], k_b[TILE], k_c[TILE], v_a[TILE], v_b[TILE], v_c[TILE];

    const bf16_t *__restrict__ q = a.q[blockIdx.z];
    bf16_t *__restrict__ o = a.o[blockIdx.z];
    const int n = a.n, nq = a.nq, nkv = a.nkv, max_seq = a.max_seq, pos0 = a.pos0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hb = lane >> 5;
    const int G = nq / nkv, gk = blockIdx.y;
    const int n_rows = n * G;
    const int blk = gridDim.x - 1 - blockIdx.x;                  // longest rows first
    const int row = blk * 128 + wave * 32 + col;
    const bool row_ok = row < n_rows;
    const int tok = row_ok ? row / G : n - 1, head = gk * G + (row_ok ? row % G : 0);
    const int my_last = pos0 + tok;
    const int wave_last_key = pos0 + min(n - 1, (blk * 128 + wave * 32 + 31) / G);
    const int wg_last_key = pos0 + min(n - 1, (blk * 128 + 127) / G);
    const int ntiles = wg_last_key / TK + 1;
    const float scale = 1.0f / sqrtf((float)D);
    const bf16_t *Kg = a.Kc[blockIdx.z] + (size_t)gk * max_seq * D;
    const bf16_t *Vg = a.Vc[blockIdx.z] + (size_t)gk * max_seq * D;

    bf16x8 qf[KS];
    {
        const bf16_t *qp = q + ((size_t)tok * nq + head) * D + hb * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }
    f32x16 oacc[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[et][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // This lane's pieces of a tile: load i of the wave covers chunks (wave * NLD + i) * 64 .. + 63, i.e. tile row
    // c / CPR at chunk position c % CPR, which holds the row's chunk (position ^ swizzle(row)).
    // K rows: swizzle so that the 16 keys a fragment read serves at a time hit 16 different chunk columns;
    // V rows: so that the 4 keys of a transposing read hit different pairs of chunks.
    constexpr int RP = 128 / D;                                  // rows per 256 bytes of LDS
    auto swz_k = [](int r) { return (r / RP) % CPR; };
    auto swz_v = [](int r) { return 2 * (r & 3); };
    int ld_row[NLD], ld_kc[NLD], ld_vc[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int c = (wave * NLD + i) * 64 + lane;
        ld_row[i] = c / CPR;
        ld_kc[i] = ((c % CPR) ^ swz_k(ld_row[i])) * 8;
        ld_vc[i] = ((c % CPR) ^ swz_v(ld_row[i])) * 8;
    }
    // the load into LDS as an instruction, for the reason given in k_gemm_bf16_nt (the compiler's waits for LDS reads
    // stay exact); the waits these loads need are the explicit ones below
    auto lds_address = [](const uint4 *p) { return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void *)p; };
    const unsigned wave_bytes = __builtin_amdgcn_readfirstlane(wave * NLD * 1024);
    auto load_to_lds = [&](const bf16_t *from, unsigned at) {
        unsigned keep;      // M0 belongs to the compiler: it is put back before the statement ends
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "v"(from), "s"(at) : "memory");
    };
    auto request = [&](uint4 *ks, uint4 *vs, int t) {
        const int k0 = t * TK;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const size_t key = (size_t)min(k0 + ld_row[i], wg_last_key);     // always in bounds; masked below
            load_to_lds(Kg + key * D + ld_kc[i], lds_address(ks) + wave_bytes + i * 1024);
            load_to_lds(Vg + key * D + ld_vc[i], lds_address(vs) + wave_bytes + i * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // fragment addresses (bytes within a tile)
    const int k_off = col * (D * 2);                             // K fragment: row = key col, chunk 2 ks + hb
    const int k_sw = swz_k(col);
    // V^T fragment for output tile et, MFMA step s2, half hf: keys 16 s2 + 8 hf + 4 hb .. + 3 of elements
    // 32 et + 16 ((lane >> 4) & 1) + (lane & 15); this lane points at key .. + (lane & 15) / 4, elements 4 (lane & 3)
    const int v_key = 4 * hb + ((lane & 15) >> 2);
    const int v_el = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    auto compute = [&](const uint4 *ks, const uint4 *vs, int t) {
        const int k0 = t * TK;
        if (k0 > wave_last_key) return;                          // none of this wave's rows sees the tile
        const unsigned char *kb = reinterpret_cast<const unsigned char *>(ks);
        const unsigned char *vb = reinterpret_cast<const unsigned char *>(vs);
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kb + k_off + (((2 * s + hb) ^ k_sw) << 4));
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc, 0, 0, 0);
        }
        // register r of this lane: key k0 + 8*(r/4) + 4*hb + r%4, row = this lane's column
        float mt = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int key = k0 + 8 * (r >> 2) + 4 * hb + (r & 3);
            float sv = (key <= my_last) ? sacc[r] * scale : -INFINITY;
            sacc[r] = sv;
            mt = fmaxf(mt, sv);
        }
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float m_new = fmaxf(m_run, mt);
        float ls = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = (sacc[r] == -INFINITY) ? 0.f : __expf(sacc[r] - m_new);
            sacc[r] = p;
            ls += p;
        }
        ls += __shfl_xor(ls, 32, 64);
        const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
        l_run = l_run * alpha + ls;
        m_run = m_new;
        if (__any(alpha != 1.0f)) {                             // the maxima settle after the first tiles
#pragma unroll
            for (int et = 0; et < ET; ++et)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[et][r] *= alpha;
        }
        bf16x8 pf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            union { bf16x8 v; bf16_t u[8]; } cvt;
#pragma unroll
            for (int i = 0; i < 8; ++i) cvt.u[i] = f32_to_bf16(sacc[8 * s2 + i]);
            pf[s2] = cvt.v;
        }
#pragma unroll
        for (int et = 0; et < ET; ++et) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                union { bf16x8 v; tr16x4 h[2]; } vf;
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int key = 16 * s2 + 8 * hf + v_key, el = 32 * et + v_el;
                    const int off = key * (D * 2) + ((((el >> 3) ^ swz_v(key)) << 4) | ((el & 7) << 1));
                    vf.h[hf] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tr16x4 *)(vb + off));
                }
                oacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[s2], oacc[et], 0, 0, 0);
            }
        }
    };
    auto step = [&](const uint4 *ks, const uint4 *vs, uint4 *kn, uint4 *vn, int t) {
        request(kn, vn, min(t + 2, ntiles - 1));
        compute(ks, vs, t);
        __builtin_amdgcn_s_waitcnt(kWaitNext);
        __builtin_amdgcn_s_barrier();
    };
    request(k_a, v_a, 0);
    request(k_b, v_b, min(1, ntiles - 1));
    __builtin_amdgcn_s_waitcnt(kWaitNext);
    __builtin_amdgcn_s_barrier();
    int t = 0;
    for (; t + 3 <= ntiles; t += 3) {
        step(k_a, v_a, k_c, v_c, t);
        step(k_b, v_b, k_a, v_a, t + 1);
        step(k_c, v_c, k_b, v_b, t + 2);
    }
    if (t < ntiles) step(k_a, v_a, k_c, v_c, t++);
    if (t < ntiles) step(k_b, v_b, k_a, v_a, t++);
    __builtin_amdgcn_s_waitcnt(kWaitAll);

    if (row_ok) {
        const float inv = 1.0f / l_run;
        bf16_t *op = o + ((size_t)tok * nq + head) * D;
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                // registers 4*r4 .. 4*r4+3: elements e = 32*et + 8*r4 + 4*hb + 0..3
                union { uint2 v; bf16_t u[4]; } pk;
#pragma unroll
                for (int i = 0; i < 4; ++i) pk.u[i] = f32_to_bf16(oacc[et][4 * r4 + i] * inv);
                *reinterpret_cast<uint2 *>(op + 32 * et + 8 * r4 + 4 * hb) = pk.v;
            }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
namespace {

struct PrefillLayout {
    size_t xn, big, q, o, act, total;   // byte offsets
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Tile shape and K split of one GEMM.  128x128 tiles once there are more than 64 rows; when the
// tiles alone leave most of the compute units idle, smaller tiles, or (where the caller has
// room for partial products) a split along K.
struct GemmPlan {
    int bm, bn, splits, k_per_split;
};

constexpr int kMaxGemmSplits = 8;
std::atomic<int> g_concurrency{1};   // prefill calls the caller runs side by side (tpi_set_prefill_concurrency)

// share: the compute units the call can count on.  The launches pass the current share; the workspace is
// sized with the whole chip, which gives the largest number of K splits.
// Compute units of the current device, asked once (256 on an MI355X; also the answer when no device
// can be asked, so that the size queries stay usable on a host without one).
int compute_units()
{
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        return cus;
    }();
    return n;
}

int current_share() { return std::max(1, compute_units() / std::max(1, g_concurrency.load(std::memory_order_relaxed))); }

GemmPlan plan_gemm(int M, int N, int K, int max_splits, int share)
{
    GemmPlan p{128, 128, 1, cdiv(K, 64) * 64};
    // 128x256 tiles move a quarter less through LDS per flop; they are taken once they still occupy three
    // quarters of the compute units this call can count on (all of them, or its share when the caller has said
    // that several prefill calls run side by side on different streams).
    if (max_splits == 1 && M > 64 && N >= 256) {
        if (cdiv(M, 128) * cdiv(N, 256) >= (3 * share) / 4) {
            p.bn = 256;
            return p;
        }
    }
    // A K split over 256x256 tiles, when that fills the share to four fifths in one round: a third less traffic
    // per flop than the split over 128x128 tiles below.
    if (max_splits > 1 && M > 128 && N >= 256 && K % 64 == 0) {
        const int t256 = cdiv(M, 256) * cdiv(N, 256), ksteps = K / 64;
        const int want = t256 <= share ? std::min(std::min(max_splits, share / t256), std::max(1, ksteps / 16)) : 0;
        if (want > 1 && 5 * t256 * want >= 4 * share) {
            const int per = cdiv(ksteps, want);
            return GemmPlan{256, 256, cdiv(ksteps, per), per * 64};
        }
    }
    if (M <= 64) p.bm = 64;
    int tiles = cdiv(M, p.bm) * cdiv(N, p.bn);
    // K is split when the tiles alone leave most of the share idle (one round of workgroups, filled by the
    // splits), or when they make fewer than three rounds of it (a ragged last round then costs too much).
    if (max_splits > 1 && (tiles < share / 2 || tiles < 3 * share)) {
        const int ksteps = cdiv(K, 64);
        const int fill = tiles < share / 2 ? share / tiles : cdiv(3 * share, tiles);
        int want = std::min(std::min(max_splits, fill), std::max(1, ksteps / (tiles < share / 2 ? 4 : 16)));
        if (want > 1) {
            const int per = cdiv(ksteps, want);
            p.splits = cdiv(ksteps, per);
            p.k_per_split = per * 64;
            return p;
        }
    }
    if (tiles < share / 2 && p.bm == 128) {
        p.bm = 64;
        tiles = cdiv(M, 64) * cdiv(N, 128);
    }
    if (tiles < share / 2) p.bn = 64;
    return p;
}

PrefillLayout layout_of(const tpi_shard_cfg *c, int n)
{
    PrefillLayout L;
    const size_t dq = (size_t)c->n_q_local * c->head_dim, dkv = (size_t)c->n_kv_local * c->head_dim;
    size_t off = 0;
    L.xn = off;  off += align256((size_t)n * c->hidden * 2);
    // room for the largest number of K splits a plan can choose, whatever share of the chip the call has
    size_t qkv = (size_t)kMaxGemmSplits * n * (dq + 2 * dkv) * 4, gu = (size_t)n * 2 * c->ffn_local * 4;
    L.big = off; off += align256(qkv > gu ? qkv : gu);
    L.q = off;   off += align256((size_t)n * dq * 2);
    L.o = off;   off += align256((size_t)n * dq * 2);
    L.act = off; off += align256((size_t)n * c->ffn_local * 2);
    L.total = off;
    return L;
}

// Launches one instantiation with its LDS size; above 64 KB the kernel has to opt in once per device.
template <int BM, int BN, int NS, int KW, bool SWI, bool DIRECT = false, int WM = 2, int LEAVE_OUT = 0>
hipError_t launch_gemm_kernel(dim3 grid, const GemmArgs &g, hipStream_t st)
{
    // DIRECT: the stages are static arrays of the kernel
    constexpr size_t lds = DIRECT ? 0 : (size_t)2 * (BM + BN) * 8 * 16;
    constexpr size_t lds_total = DIRECT ? (size_t)NS * (BM + BN) * 8 * 16 : lds;
    auto *kern = k_gemm_bf16_nt<BM, BN, NS, KW, SWI, DIRECT, WM, LEAVE_OUT>;
    if constexpr (lds_total > 65536) {
        static std::atomic<bool> opted[64];
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (!opted[dev].load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            opted[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(128 * WM * KW), lds, st, g);
    return hipGetLastError();
}

// The eight-wave tiles load straight into LDS when every K range is whole 64-element steps.
inline bool direct_ok(const GemmArgs &g) { return g.K % 64 == 0 && g.k_per_split % 64 == 0; }

// 256x256 tiles (four waves, each a 128x128 quarter) fetch a third less per flop from L2 and from LDS than
// 128x256 tiles.  They are taken when there are at least two row tiles' worth of rows and the tiles fill the
// compute units this call can count on to at least four fifths, counted over whole rounds.
inline bool square_tiles_pay(int M, int col_tiles, int S)
{
    const long cus = std::max(1, current_share()), tiles = (long)cdiv(M, 256) * col_tiles * S;
    const long rounds = (tiles + cus - 1) / cus;
    return M > 128 && tiles >= cus && 5 * tiles >= 4 * rounds * cus;
}

// max_splits > 1: C must have room for that many partial products of M * ldc floats; the number
// actually written is returned in *n_parts.
// One GEMM launch for the S shards of a batched call (ptrs[s].C is the shard's output; with max_splits > 1 it
// must have room for that many partial products of M * ldc floats; the number written is returned in *n_parts).
hipError_t launch_gemm(const GemmPtrs *ptrs, int S, int lda, int n_split, int ldb, int ldc, int M, int N, int K,
                       hipStream_t st, int max_splits = 1, int *n_parts = nullptr)
{
    const GemmPlan p = plan_gemm(M, N, K, max_splits, std::max(1, current_share() / S));
    if (n_parts) *n_parts = p.splits;
    GemmArgs g{};
    g.M = M; g.N = N; g.K = K; g.n_split = n_split; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.k_per_split = p.k_per_split; g.splits = p.splits; g.c_split = (size_t)M * ldc;
    for (int s = 0; s < S; ++s) g.p[s] = ptrs[s];
    ProfScope ps(kStagePrefillGemm, st);
    dim3 grid(cdiv(N, p.bn), cdiv(M, p.bm), p.splits * S);
    if (p.bm == 256) return launch_gemm_kernel<256, 256, 2, 1, false, true, 4>(grid, g, st);   // whole steps by the plan
    if (p.bm == 128 && p.bn == 256) {
        if (direct_ok(g) && square_tiles_pay(M, cdiv(N, 256), S))
            return launch_gemm_kernel<256, 256, 2, 1, false, true, 4>(dim3(cdiv(N, 256), cdiv(M, 256), S), g, st);
        return direct_ok(g) ? launch_gemm_kernel<128, 256, 3, 2, false, true>(grid, g, st)
                            : launch_gemm_kernel<128, 256, 2, 2, false>(grid, g, st);
    }
    if (p.bm == 128) {
        if (!direct_ok(g)) return launch_gemm_kernel<128, 128, 4, 2, false>(grid, g, st);
        // With at least two workgroups per compute unit the two-stage variant (64 KB of LDS, two workgroups
        // resident) lets one workgroup's start and end overlap the other's K loop: QKV of 8 shards 126 -> 119 us.
        // With one workgroup per compute unit the deeper pipeline of the three-stage variant is what counts.
        if ((int)(grid.x * grid.y * grid.z) >= 2 * std::max(1, current_share()))
            return launch_gemm_kernel<128, 128, 2, 2, false, true>(grid, g, st);
        return launch_gemm_kernel<128, 128, 3, 2, false, true>(grid, g, st);
    }
    if (p.bn == 128) return launch_gemm_kernel<64, 128, 4, 1, false>(grid, g, st);
    return launch_gemm_kernel<64, 64, 4, 1, false>(grid, g, st);
}

// act[m][j] = bf16(silu(A . gate[j]) * (A . up[j])) in one launch (B0 = gate, B1 = up, act set, C unused).  False
// (nothing launched) when the plan for this shape uses 64-column tiles: the caller then multiplies and
// activates separately.
// When the wide tiles make several rounds of the compute units and the last round is less than 0.6 of one, the
// hidden units are divided between two launches: wide tiles for as many units as fill whole rounds, 128-column
// tiles (half the work each) for the rest, so that the chip is not half idle for the length of a wide tile.
bool launch_gemm_swiglu(const GemmPtrs *ptrs, int S, int lda, int sl, int ldb, int M, int K, hipStream_t st, hipError_t *err)
{
    const GemmPlan p = plan_gemm(M, 2 * sl, K, 1, std::max(1, current_share() / S));
    *err = hipSuccess;
    if (p.bn < 128) return false;
    GemmArgs g{};
    g.M = M; g.N = 2 * sl; g.K = K; g.n_split = sl; g.lda = lda; g.ldb = ldb; g.ldc = sl;
    g.k_per_split = p.k_per_split; g.splits = 1; g.c_split = 0;
    for (int s = 0; s < S; ++s) g.p[s] = ptrs[s];
    ProfScope ps(kStagePrefillGemm, st);
    if (p.bn == 256 && direct_ok(g) && square_tiles_pay(M, cdiv(sl, 128), S)) {
        // 256x256 tiles.  When they end with a ragged round and the units of that round divide into exactly one
        // round of 256x192 tiles (96 units each), the launch is divided: whole rounds of 256x256 tiles, then one
        // round of the narrower tiles, so that no compute unit idles through a tile's length (70B shape, 8 shards
        // x 512 tokens: 448 tiles = 256 + 192 become 256 tiles of 128 units + 256 tiles of 96).
        const int cus = std::max(1, current_share()), per_col = cdiv(M, 256) * S, cols = cdiv(sl, 128);
        int full_cols = cols;
        if ((per_col * cols) % cus != 0 && cus % per_col == 0) {
            const int whole = ((per_col * cols) / cus) * (cus / per_col);       // column tiles of the whole rounds
            const int rest = sl - whole * 128;
            if (whole >= 1 && rest > 0 && cdiv(rest, 96) * per_col == cus) full_cols = whole;
        }
        const int full_units = std::min(sl, full_cols * 128);
        g.n_split = full_units; g.N = 2 * full_units;
        *err = launch_gemm_kernel<256, 256, 2, 1, true, true, 4>(dim3(full_cols, cdiv(M, 256), S), g, st);
        if (*err != hipSuccess || full_units == sl) return true;
        g.n_split = sl - full_units; g.N = 2 * g.n_split;
        for (int s = 0; s < S; ++s) {
            g.p[s].B0 += (size_t)full_units * ldb;
            g.p[s].B1 += (size_t)full_units * ldb;
            g.p[s].act += full_units;
        }
        *err = launch_gemm_kernel<256, 192, 2, 1, true, true, 4>(dim3(cdiv(g.n_split, 96), cdiv(M, 256), S), g, st);
        return true;
    }
    if (p.bn == 256) {
        const int cus = std::max(1, current_share()), per_col = cdiv(M, p.bm) * S, cols = cdiv(sl, 128);
        int wide_cols = cols;
        const int ragged = (per_col * cols) % cus;
        if (per_col * cols > cus && ragged != 0 && 10 * ragged < 6 * cus) {
            for (int c = cols - 1; c >= 1; --c)
                if ((per_col * c) % cus == 0) { wide_cols = c; break; }
        }
        const int wide_units = std::min(sl, wide_cols * 128);
        g.n_split = wide_units; g.N = 2 * wide_units;
        dim3 grid(wide_cols, cdiv(M, p.bm), S);
        *err = direct_ok(g) ? launch_gemm_kernel<128, 256, 3, 2, true, true>(grid, g, st)
                            : launch_gemm_kernel<128, 256, 2, 2, true>(grid, g, st);
        if (*err != hipSuccess || wide_units == sl) return true;
        // the remaining units: gate and up rows from wide_units on, activation columns from wide_units on
        g.n_split = sl - wide_units; g.N = 2 * g.n_split;
        for (int s = 0; s < S; ++s) {
            g.p[s].B0 += (size_t)wide_units * ldb;
            g.p[s].B1 += (size_t)wide_units * ldb;
            g.p[s].act += wide_units;
        }
        dim3 rest(cdiv(g.n_split, 64), cdiv(M, p.bm), S);
        *err = direct_ok(g) ? launch_gemm_kernel<128, 128, 3, 2, true, true>(rest, g, st)
                            : launch_gemm_kernel<128, 128, 4, 2, true>(rest, g, st);
        return true;
    }
    dim3 grid(cdiv(sl, 64), cdiv(M, p.bm), S);
    if (p.bm == 128)
        *err = direct_ok(g) ? launch_gemm_kernel<128, 128, 3, 2, true, true>(grid, g, st)
                            : launch_gemm_kernel<128, 128, 4, 2, true>(grid, g, st);
    else *err = launch_gemm_kernel<64, 128, 4, 1, true>(grid, g, st);
    return true;
}

}  // namespace

size_t prefill_workspace_bytes(const tpi_shard_cfg *cfg, int32_t n_tokens) { return layout_of(cfg, n_tokens).total; }

void prefill_set_concurrency(int n) { g_concurrency.store(n, std::memory_order_relaxed); }

// S shards of one layer phase in one set of launches: every kernel takes the shard from a grid dimension.
int prefill_launch(const tpi_shard_cfg *c, int S, const tpi_layer_weights *w, const tpi_kv_layer *kv, int32_t pos0, int32_t n,
                   int phase, const void *h_in, float *const *partial_out, void *const *workspace, hipStream_t st)
{
    const int h = c->hidden, d = c->head_dim, nq = c->n_q_local, nkv = c->n_kv_local, sl = c->ffn_local;
    const int dq = nq * d, dkv = nkv * d;
    auto al = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    if (S < 1 || S > kMaxPrefillShards) return fail(TPI_EINVAL, "n_shards %d outside [1, %d]", S, kMaxPrefillShards);
    if (!al(h_in)) return fail(TPI_EUNSUPPORTED, "pointer not 16-byte aligned");
    const PrefillLayout L = layout_of(c, n);
    bf16_t *xn[kMaxPrefillShards], *qb[kMaxPrefillShards], *ob[kMaxPrefillShards], *act[kMaxPrefillShards];
    float *big[kMaxPrefillShards];
    for (int s = 0; s < S; ++s) {
        if (!partial_out[s] || !workspace[s]) return fail(TPI_EINVAL, "shard %d: null output or workspace", s);
        if (!al(partial_out[s]) || !al(workspace[s])) return fail(TPI_EUNSUPPORTED, "shard %d: pointer not 16-byte aligned", s);
        char *ws = static_cast<char *>(workspace[s]);
        xn[s] = reinterpret_cast<bf16_t *>(ws + L.xn);
        big[s] = reinterpret_cast<float *>(ws + L.big);
        qb[s] = reinterpret_cast<bf16_t *>(ws + L.q);
        ob[s] = reinterpret_cast<bf16_t *>(ws + L.o);
        act[s] = reinterpret_cast<bf16_t *>(ws + L.act);
    }
    hipError_t e = hipSuccess;
#define TPI_LAUNCH_OK()                                                                         \
    do {                                                                                        \
        e = hipGetLastError();                                                                  \
        if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e)); \
    } while (0)
#define TPI_GEMM_OK()                                                                           \
    do {                                                                                        \
        if (e != hipSuccess) return fail(TPI_ERUNTIME, "kernel launch failed: %s", hipGetErrorString(e)); \
    } while (0)

    NormArgs na{};
    na.x = (const bf16_t *)h_in; na.h = h; na.eps = c->rms_eps;
    GemmPtrs gp[kMaxPrefillShards];
    // The hidden state and the norm are replicated on every device (Sec. 3.1): when all shards of the call name the
    // SAME gain vector -- the emulated devices of one model -- the input is normalised once, into the first shard's
    // workspace, and every shard's first GEMM reads that one copy (the same values a copy per shard would hold).
    auto norm_launch = [&](int n_tok) {
        bool same = S > 1;
        for (int s = 1; s < S; ++s) same = same && na.g[s] == na.g[0];
        hipLaunchKernelGGL(k_rmsnorm_bf16, dim3(n_tok, same ? 1 : S), dim3(256), 0, st, na);
        if (same)
            for (int s = 1; s < S; ++s) xn[s] = xn[0];
    };

    if (phase == TPI_PHASE_ATTN) {
        for (int s = 0; s < S; ++s) {
            if (!w[s].attn_norm || !w[s].w_qkv || !w[s].w_o || !kv[s].k || !kv[s].v)
                return fail(TPI_EINVAL, "shard %d: null attention weight or cache pointer", s);
            if (!al(w[s].attn_norm) || !al(w[s].w_qkv) || !al(w[s].w_o) || !al(kv[s].k) || !al(kv[s].v))
                return fail(TPI_EUNSUPPORTED, "shard %d: pointer not 16-byte aligned", s);
            na.g[s] = (const float *)w[s].attn_norm; na.out[s] = xn[s];
        }
        if (d > 256) return fail(TPI_EUNSUPPORTED, "head_dim %d > 256", d);
        const int G = nq / nkv;
        if (G > 64) return fail(TPI_EUNSUPPORTED, "more than 64 query heads per KV head");
        norm_launch(n);
        TPI_LAUNCH_OK();
        int qkv_parts = 1;
        for (int s = 0; s < S; ++s) gp[s] = GemmPtrs{xn[s], (const bf16_t *)w[s].w_qkv, (const bf16_t *)w[s].w_qkv, big[s], nullptr};
        e = launch_gemm(gp, S, h, dq + 2 * dkv, h, dq + 2 * dkv, n, dq + 2 * dkv, h, st, kMaxGemmSplits, &qkv_parts);
        TPI_GEMM_OK();
        RopeArgs ra{};
        ra.n_parts = qkv_parts; ra.part_stride = (size_t)n * (dq + 2 * dkv);
        ra.n = n; ra.nq = nq; ra.nkv = nkv; ra.d = d; ra.max_seq = c->max_seq; ra.pos0 = pos0;
        ra.log2_base = std::log2((double)c->rope_base);
        for (int s = 0; s < S; ++s) { ra.qkv[s] = big[s]; ra.q_out[s] = qb[s]; ra.Kc[s] = (bf16_t *)kv[s].k; ra.Vc[s] = (bf16_t *)kv[s].v; }
        const int nthr = n * (nq + 2 * nkv) * (d / 2);
        hipLaunchKernelGGL(k_rope_scatter, dim3((nthr + 255) / 256, S), dim3(256), 0, st, ra);
        TPI_LAUNCH_OK();
        if (d % 32 == 0 && d <= 128) {
            AttnArgs aa{};
            aa.n = n; aa.nq = nq; aa.nkv = nkv; aa.max_seq = c->max_seq; aa.pos0 = pos0;
            for (int s = 0; s < S; ++s) { aa.q[s] = qb[s]; aa.Kc[s] = (const bf16_t *)kv[s].k; aa.Vc[s] = (const bf16_t *)kv[s].v; aa.o[s] = ob[s]; }
            dim3 grid((n * G + 31) / 32, nkv, S);
            // With at least one 128-row workgroup per compute unit the kernel that shares its key and value
            // tiles among 128 rows is ahead (one shard, 16 layers: 16384-token prompt 130 -> 96 ms, 4096 tokens
            // 23.4 -> 23.0 ms); below that the 32-row kernel, whose waves split the keys, has the shorter
            // critical path (2048 tokens: 11.85 against 12.2 ms; 512 tokens, one shard: 16 against 34 us).
            const long wg128 = (long)((n * G + 127) / 128) * nkv * S;
            if ((d == 64 || d == 128) && wg128 >= std::max(1, current_share())) {
                dim3 g2((n * G + 127) / 128, nkv, S);
                if (d == 64) hipLaunchKernelGGL((k_prefill_attn_shared<64>), g2, dim3(256), 0, st, aa);
                else hipLaunchKernelGGL((k_prefill_attn_shared<128>), g2, dim3(256), 0, st, aa);
            } else
            switch (d) {
            case 32: hipLaunchKernelGGL((k_prefill_attn_mfma<32>), grid, dim3(256), 0, st, aa); break;
            case 64: hipLaunchKernelGGL((k_prefill_attn_mfma<64>), grid, dim3(256), 0, st, aa); break;
            case 96: hipLaunchKernelGGL((k_prefill_attn_mfma<96>), grid, dim3(256), 0, st, aa); break;
            default: hipLaunchKernelGGL((k_prefill_attn_mfma<128>), grid, dim3(256), 0, st, aa); break;
            }
            TPI_LAUNCH_OK();
        } else {
            const int QT = 64 / G;                         // tokens per workgroup: QT * G <= 64 rows
            const size_t lds = sizeof(float) * ((size_t)64 * (d + 1) + (size_t)64 * d + (size_t)64 * (d + 1) + 64 * 65);
            dim3 grid((n + QT - 1) / QT, nkv);
            if (lds > 65536) {                             // opt in to more than 64 KB of LDS per workgroup
                int dev = 0, cap = 0;
                e = hipGetDevice(&dev);
                if (e == hipSuccess) e = hipDeviceGetAttribute(&cap, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
                if (e != hipSuccess) return fail(TPI_ERUNTIME, "device query failed: %s", hipGetErrorString(e));
                if ((size_t)cap < lds) return fail(TPI_EUNSUPPORTED, "attention tile needs %zu bytes of LDS, device allows %d", lds, cap);
                e = (d <= 64) ? hipFuncSetAttribute((const void *)k_prefill_attn<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                              : hipFuncSetAttribute((const void *)k_prefill_attn<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return fail(TPI_ERUNTIME, "hipFuncSetAttribute: %s", hipGetErrorString(e));
            }
            if (d > 128) return fail(TPI_EUNSUPPORTED, "prefill attention is built for head_dim <= 128");
            for (int s = 0; s < S; ++s) {                  // the vector-ALU attention takes one shard per launch
                if (d <= 64) {
                    hipLaunchKernelGGL((k_prefill_attn<64>), grid, dim3(256), lds, st, qb[s], (const bf16_t *)kv[s].k,
                                       (const bf16_t *)kv[s].v, ob[s], n, nq, nkv, d, c->max_seq, pos0, QT);
                } else {
                    hipLaunchKernelGGL((k_prefill_attn<128>), grid, dim3(256), lds, st, qb[s], (const bf16_t *)kv[s].k,
                                       (const bf16_t *)kv[s].v, ob[s], n, nq, nkv, d, c->max_seq, pos0, QT);
                }
                TPI_LAUNCH_OK();
            }
        }
        for (int s = 0; s < S; ++s) gp[s] = GemmPtrs{ob[s], (const bf16_t *)w[s].w_o, (const bf16_t *)w[s].w_o, partial_out[s], nullptr};
        e = launch_gemm(gp, S, dq, h, dq, h, n, h, dq, st);
        TPI_GEMM_OK();
    } else {
        for (int s = 0; s < S; ++s) {
            if (!w[s].ffn_norm || !w[s].w_gate || !w[s].w_up || !w[s].w_down)
                return fail(TPI_EINVAL, "shard %d: null FFN weight pointer", s);
            if (!al(w[s].ffn_norm) || !al(w[s].w_gate) || !al(w[s].w_up) || !al(w[s].w_down))
                return fail(TPI_EUNSUPPORTED, "shard %d: pointer not 16-byte aligned", s);
            na.g[s] = (const float *)w[s].ffn_norm; na.out[s] = xn[s];
        }
        norm_launch(n);
        TPI_LAUNCH_OK();
        for (int s = 0; s < S; ++s) gp[s] = GemmPtrs{xn[s], (const bf16_t *)w[s].w_gate, (const bf16_t *)w[s].w_up, big[s], act[s]};
        if (launch_gemm_swiglu(gp, S, h, sl, h, n, h, st, &e)) {
            TPI_GEMM_OK();
        } else {
            e = launch_gemm(gp, S, h, sl, h, 2 * sl, n, 2 * sl, h, st);
            TPI_GEMM_OK();
            const size_t tot = (size_t)n * sl;
            for (int s = 0; s < S; ++s) {
                hipLaunchKernelGGL(k_swiglu, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, big[s], act[s], n, sl);
                TPI_LAUNCH_OK();
            }
        }
        for (int s = 0; s < S; ++s) gp[s] = GemmPtrs{act[s], (const bf16_t *)w[s].w_down, (const bf16_t *)w[s].w_down, partial_out[s], nullptr};
        e = launch_gemm(gp, S, sl, h, sl, h, n, h, sl, st);
        TPI_GEMM_OK();
    }
#undef TPI_LAUNCH_OK
#undef TPI_GEMM_OK
    return TPI_OK;
}

// ---------------------------------------------------------------------------
// Loop probe: the 256x256 tile's K loop with one or two of its three activities left out
// ---------------------------------------------------------------------------
namespace {

struct ProbeBuffers {
    bf16_t *a = nullptr, *b = nullptr;
    float *c = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~ProbeBuffers()
    {
        if (a) (void)hipFree(a);
        if (b) (void)hipFree(b);
        if (c) (void)hipFree(c);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

// element i of a probe operand: sign and the low 7 mantissa bits from a hash of i, exponent fixed: +-[2^-7, 2^-6)
__host__ __device__ inline unsigned short probe_value_bits(size_t i, unsigned salt)
{
    unsigned x = (unsigned)i * 2654435761u + salt;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    return (unsigned short)((x & 0x8000u) | 0x3c00u | (x & 0x7fu));
}

__global__ __launch_bounds__(256) void k_probe_fill_bf16(bf16_t *p, size_t n, unsigned salt)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = probe_value_bits(i, salt);
}

template <int LEAVE_OUT>
hipError_t launch_probe_variant(dim3 grid, const GemmArgs &g, hipStream_t st)
{
    return launch_gemm_kernel<256, 256, 2, 1, false, true, 4, LEAVE_OUT>(grid, g, st);
}

}  // namespace

int prefill_probe_gemm_loop(int leave_out, int reps, tpi_gemm_probe_result *out, hipStream_t st)
{
#define TPI_PROBE_HIP(call)                                                                          \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess) return fail(TPI_ERUNTIME, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)
    // the down projection of the 70B-shaped 8-way shard for a 512-token prompt, 8 shards per launch:
    // 512 tiles of 256x256 with 56 K-steps each, two rounds of 256 compute units
    constexpr int S = 8, M = 512, N = 8192, K = 3584;
    constexpr unsigned kSaltA = 17u, kSaltB = 4099u;
    const size_t a_elems = (size_t)S * M * K, b_elems = (size_t)S * N * K, c_elems = (size_t)S * M * N;
    ProbeBuffers B;
    TPI_PROBE_HIP(hipMalloc(&B.a, a_elems * 2));
    TPI_PROBE_HIP(hipMalloc(&B.b, b_elems * 2));
    TPI_PROBE_HIP(hipMalloc(&B.c, c_elems * 4));
    TPI_PROBE_HIP(hipEventCreate(&B.e0));
    TPI_PROBE_HIP(hipEventCreate(&B.e1));
    hipLaunchKernelGGL(k_probe_fill_bf16, dim3(4096), dim3(256), 0, st, B.a, a_elems, kSaltA);
    hipLaunchKernelGGL(k_probe_fill_bf16, dim3(4096), dim3(256), 0, st, B.b, b_elems, kSaltB);
    TPI_PROBE_HIP(hipGetLastError());
    TPI_PROBE_HIP(hipMemsetAsync(B.c, 0, c_elems * 4, st));
    GemmArgs g{};
    g.M = M; g.N = N; g.K = K; g.n_split = N; g.lda = K; g.ldb = K; g.ldc = N;
    g.k_per_split = K; g.splits = 1; g.c_split = (size_t)M * N;
    for (int s = 0; s < S; ++s) {
        g.p[s].A = B.a + (size_t)s * M * K;
        g.p[s].B0 = B.b + (size_t)s * N * K;
        g.p[s].B1 = g.p[s].B0;
        g.p[s].C = B.c + (size_t)s * M * N;
        g.p[s].act = nullptr;
    }
    const dim3 grid(N / 256, M / 256, S);
    auto launch = [&]() -> hipError_t {
        switch (leave_out) {
        case 0: return launch_probe_variant<0>(grid, g, st);
        case 1: return launch_probe_variant<1>(grid, g, st);
        case 2: return launch_probe_variant<2>(grid, g, st);
        case 3: return launch_probe_variant<3>(grid, g, st);
        case 4: return launch_probe_variant<4>(grid, g, st);
        case 5: return launch_probe_variant<5>(grid, g, st);
        default: return launch_probe_variant<6>(grid, g, st);
        }
    };
    TPI_PROBE_HIP(launch());                                  // untimed: code load, first touch
    TPI_PROBE_HIP(hipEventRecord(B.e0, st));
    for (int r = 0; r < reps; ++r) TPI_PROBE_HIP(launch());
    TPI_PROBE_HIP(hipEventRecord(B.e1, st));
    TPI_PROBE_HIP(hipEventSynchronize(B.e1));
    float ms = 0.f;
    TPI_PROBE_HIP(hipEventElapsedTime(&ms, B.e0, B.e1));
    out->us_per_launch = 1e3 * (double)ms / reps;
    out->tflop_per_launch = 2.0 * S * M * (double)N * K * 1e-12;
    out->tflops = leave_out == 0 ? out->tflop_per_launch / (out->us_per_launch * 1e-6) : 0.0;
    // the complete loop must have multiplied: the first and the last output element against the same sums on the host
    out->result_ok = -1;
    if (leave_out == 0) {
        auto value = [](size_t i, unsigned salt) {
            const unsigned short b = probe_value_bits(i, salt);
            const double mag = std::ldexp(1.0 + (b & 0x7f) / 128.0, -7);
            return (b & 0x8000u) ? -mag : mag;
        };
        bool ok = true;
        const size_t where[2][3] = {{0, 0, 0}, {S - 1, M - 1, N - 1}};       // shard, row, column
        for (const auto &w : where) {
            double want = 0.0, scale = 0.0;
            for (int k = 0; k < K; ++k) {
                const double t = value((w[0] * M + w[1]) * (size_t)K + k, kSaltA) * value((w[0] * N + w[2]) * (size_t)K + k, kSaltB);
                want += t;
                scale += std::fabs(t);
            }
            float got = 0.f;
            TPI_PROBE_HIP(hipMemcpy(&got, B.c + (w[0] * M + w[1]) * (size_t)N + w[2], 4, hipMemcpyDeviceToHost));
            ok = ok && std::fabs(got - want) <= 1e-5 * scale;
        }
        out->result_ok = ok ? 1 : 0;
    }
    return TPI_OK;
#undef TPI_PROBE_HIP
}

}  // namespace tpi

