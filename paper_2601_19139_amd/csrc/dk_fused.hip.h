// One decode step as a single persistent kernel, for small batches of small
// dense models, where a step is a chain of ~5 tiny dependent stages per layer
// and the chip would otherwise spend its time at kernel boundaries.
//
// One block per compute unit stays resident for the whole step and walks through
// every stage of every layer.  A stage's weights do not depend on the previous
// stage, so each block requests its slice of the NEXT stage's weights before it
// waits for that stage's input: the HBM latency of the weight stream is hidden
// behind the hand-over.  The hand-over itself needs no barrier and no flag:
//
//   * every activation buffer of the step (per layer: q|k|v, attention partials,
//     the two residual vectors, the MLP activations) has its own place in a
//     set of buffers that holds a "not written yet" bit pattern (a NaN that no
//     arithmetic produces) when the step starts;
//   * producers write results with device-coherent stores; consumers read with
//     device-coherent loads and simply re-read until no element is the pattern
//     (the 8 compute dies do not share an L2, so ordinary loads could be stale);
//   * there are two sets; a step uses one and refills the other with the
//     pattern for the next step (the kernel boundary between steps orders that);
//   * the vectors that every block awaits (attention output, the two residual
//     vectors, the MLP activations) are written in kFusedReplicas copies and a
//     block polls copy blockIdx % kFusedReplicas: fewer blocks poll the same lines.
//
// Requests return in order, so whatever a wave has requested before it polls
// delays the poll's answer: a stage's weight rows are requested ahead of its
// wait on purpose (they stream during the hand-over), but a burst of such requests
// from all blocks at once makes the hand-over as long as the burst.  While
// attention runs most blocks are idle and HBM is too: those blocks request a word
// of every line of the MLP's rows then (their own and those of a partner block of
// their die that is busy), which brings the rows into the die's L2 before the
// MLP's stages ask for them.  Weight rows are requested as streaming loads.
//
// Every wait is bounded: after a spin limit a block raises an abort word tagged
// with the step's serial number, and every waiter that sees it stops waiting, so
// the kernel always terminates (with an error the host can read) even if
// blocks were not co-resident.
//
// Work split: the rows of a matrix are divided evenly over the blocks and, in a
// block, over its 4 waves; a wave owns whole rows (lanes stride K in 16-byte
// pieces) so no cross-wave reduction is needed.  Attention: one block per
// (row, kv head, 64-token chunk) with the K/V tiles requested ahead as well;
// the block of a sequence's first chunk collects the other chunks' partials and
// publishes the finished attention output, which the output projection awaits.
#pragma once
#include <type_traits>
#include "dk_attention.hip.h"

namespace dk {

constexpr uint32_t kNotYet = 0x7FFFFFFFu;   // "not written yet"
constexpr int kFusedThreads = 256;
constexpr int kFusedWaves = 4;
constexpr int kFusedMaxLayers = 40;
constexpr int kFusedChunk = 64;             // tokens per attention work item
constexpr int kFusedMergeRound = 12;        // chunk partials the collecting block awaits at a time
constexpr int kFusedWaveTiles = kFusedChunk / (16 * kFusedWaves);   // 16-token K/V tiles per wave
constexpr int kFusedStamps = 16;            // stage boundaries a block can stamp per layer (see FusedArgs::stamps)
constexpr int kFusedReplicas = 4;           // copies of a vector that every block awaits (block blk polls copy blk % kFusedReplicas)
constexpr int kFusedWarmDelay = 64;         // x 64 clocks between a layer's start and an idle block's L2 warming
constexpr int kFusedSpinLimit = 1 << 16;    // polls before a block gives up (each ~1 us)

struct FusedLayer {
    const uint16_t *g_attn, *w_qkv, *g_q, *g_k, *w_o, *g_mlp, *w_gate, *w_up, *w_down;
};

struct FusedArgs {
    int L, H, nq, nkv, F, V, B;
    float eps, scale;
    const uint16_t *embed, *lm_head, *g_final;
    int *tokens, *seq_lens;
    const int *block_tables;
    int max_blocks, num_blocks;
    uint16_t *pool;
    float *logits;         // [B][V] or null
    int *next;             // [B]
    int advance;
    float *set;            // this step's buffers (all "not yet")
    float *other_set;      // refilled with the pattern during this step
    long long set_floats;
    int nchunks;           // attention chunks per sequence the buffers have room for
    unsigned *status;      // [0] abort tag, [1] number of timeouts ever
    unsigned serial;       // this step's tag (never 0)
    int spin_limit;        // polls before a block gives up a wait
    long long *stamps;     // measurement aid, normally null: [blocks][kFusedStamps] device clock readings of layer stamp_layer
    int stamp_layer;
    double inv_freq[64];
    FusedLayer layers[kFusedMaxLayers];
};

// offsets (in floats) inside a buffer set
struct FusedLayout {
    long long qkv, part, attn, xmid, act, xout, per_layer, amax, total;
};
__host__ __device__ inline FusedLayout fused_layout(int L, int B, int H, int nq, int nkv, int d, int F,
                                                   int nchunks, int nblocks)
{
    FusedLayout o;
    const long long qkv_dim = (long long)(nq + 2 * nkv) * d;
    o.qkv = 0;
    o.part = o.qkv + B * qkv_dim;
    // the vectors that all blocks await at once come in kFusedReplicas copies ([copy][B][N]): the more blocks
    // poll the lines that 8 producers at a time are writing, the later the last word is seen
    o.attn = o.part + (long long)B * nq * nchunks * (d + 2);
    o.xmid = o.attn + (long long)kFusedReplicas * B * nq * d;
    o.act = o.xmid + (long long)kFusedReplicas * B * H;
    o.xout = o.act + (long long)kFusedReplicas * B * F;
    o.per_layer = o.xout + (long long)kFusedReplicas * B * H;
    o.amax = o.per_layer * L;
    o.total = o.amax + 2LL * nblocks * B;
    return o;
}

__device__ __forceinline__ uint32_t ldc_u32(const void *p)
{
    return __hip_atomic_load(static_cast<const uint32_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stc_f32(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Four consecutive words at base + byte_off by one device-scope load (a raw buffer load with the sc1 bit: the
// 16-byte form of ldc_u32; the words may come from different moments, which data-as-flag does not mind).
// base: uniform over the wave, 16-byte aligned; bytes: the extent that may be read from base.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 ldc_u32x4(const void *base, uint32_t bytes, uint32_t byte_off)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, 16);
}

// Warming the die's L2: one word of every 128-byte line of [p, p + bytes) is requested, LINES lines per thread
// (bytes <= LINES * 32 KB; lines past the end repeat the last).  The words are returned so that nothing waits
// for them here: the caller folds them into a sink once the loads have long returned.
template <int LINES>
struct WarmWords { uint32_t w[LINES]; };
template <int LINES>
__device__ __forceinline__ WarmWords<LINES> warm_l2(const void *p, int bytes)
{
    WarmWords<LINES> r;
    const uint32_t *q = static_cast<const uint32_t *>(p);
    const int lines = (bytes + 127) >> 7;
#pragma unroll
    for (int i = 0; i < LINES; i++) r.w[i] = q[(long long)min(i * kFusedThreads + (int)threadIdx.x, lines - 1) * 32];
    return r;
}

// Bounded wait shared by every hand-over: `ready` is this thread's verdict on
// the elements it just loaded.  Returns true when the whole block may stop
// polling (everything arrived, or the step was aborted).
struct Waiter {
    unsigned *status;
    unsigned serial;
    int spins;
    bool aborted;
    int limit;
    unsigned *slots;   // LDS [2][kFusedWaves]: the waves' verdicts, double-buffered so one barrier per poll suffices
    int phase;
    __device__ __forceinline__ bool done(bool ready)
    {
        const int wv = threadIdx.x >> 6;
        const bool wave_ok = __all(ready);
        if ((threadIdx.x & 63) == 0) slots[phase * kFusedWaves + wv] = wave_ok;
        __syncthreads();
        const unsigned *sl = slots + phase * kFusedWaves;
        const bool ok = (sl[0] & sl[1] & sl[2] & sl[3]) != 0;
        phase ^= 1;
        if (ok) return true;
        spins++;
        if ((spins & 63) == 0 || spins > limit) {
            bool stop = ldc_u32(status) == serial;
            if (spins > limit && !stop) {
                if (threadIdx.x == 0) {
                    __hip_atomic_store(status, serial, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    atomicAdd(status + 1, 1u);
                }
                stop = true;
            }
            if (__syncthreads_or(stop)) { aborted = true; return true; }
        }
        __builtin_amdgcn_s_sleep(1);
        return false;
    }
};

// Loads x[NB][K] (device-coherent, re-reading until complete) into LDS as
// x * gain (or x) and returns 1/rms per row when NORM.
template <int NB, bool NORM, int MAXE /*elements per thread and row: K <= 256 * MAXE*/>
__device__ __forceinline__ void stage_input_words(const float *src, int K, const uint16_t *gain, float eps,
                                            float *xs /*[NB][K]*/, float (&rinv)[NB], float *red /*[4][NB]*/,
                                            Waiter &w)
{
    const int tid = threadIdx.x;
    uint32_t v[NB][MAXE];
    float gn[MAXE];
#pragma unroll
    for (int e = 0; e < MAXE; e++) {
        // on its way during the wait.  (Unconditional, from a clamped index: a load inside a
        // condition is waited for on the spot, one after the other.)
        gn[e] = NORM ? bf16_to_f32(gain[min(e * kFusedThreads + tid, K - 1)]) : 1.f;
    }
    w.spins = 0;
    for (;;) {
        bool ready = true;
#pragma unroll
        for (int b = 0; b < NB; b++)
#pragma unroll
            for (int e = 0; e < MAXE; e++) {
                const int k = min(e * kFusedThreads + tid, K - 1);     // past the end: the last word again
                v[b][e] = ldc_u32(src + (long long)b * K + k);
                ready = ready && v[b][e] != kNotYet;
            }
        if (w.done(ready)) break;
    }
    float ss[NB];
#pragma unroll
    for (int b = 0; b < NB; b++) {
        ss[b] = 0.f;
#pragma unroll
        for (int e = 0; e < MAXE; e++) {
            const int k = e * kFusedThreads + tid;
            if (k < K) {
                const float x = __uint_as_float(v[b][e]);
                ss[b] += x * x;
                xs[b * K + k] = NORM ? x * gn[e] : x;
            }
        }
    }
    if (NORM) {
#pragma unroll
        for (int b = 0; b < NB; b++) {
            const float s = sum64(ss[b]);
            if ((tid & 63) == 0) red[(tid >> 6) * NB + b] = s;
        }
    }
    __syncthreads();
    if (NORM) {
#pragma unroll
        for (int b = 0; b < NB; b++)
            rinv[b] = rsqrtf((red[b] + red[NB + b] + red[2 * NB + b] + red[3 * NB + b]) / (float)K + eps);
    }
}

// The same with 16-byte requests (four consecutive words per thread): a quarter of the poll instructions.  For
// the long vectors of the wide classes (16 and more words per thread and row), where a poll round is as long as
// the compute unit's memory pipeline needs for its requests; K a multiple of 4.
template <int NB, bool NORM, int MAXE>
__device__ __forceinline__ void stage_input_quads(const float *src, int K, const uint16_t *gain, float eps,
                                                  float *xs /*[NB][K]*/, float (&rinv)[NB], float *red /*[4][NB]*/,
                                                  Waiter &w)
{
    constexpr int GROUPS = (MAXE + 3) / 4;
    const int tid = threadIdx.x;
    u32x4 v[NB][GROUPS];
    uint2 gn[GROUPS];
#pragma unroll
    for (int e = 0; e < GROUPS; e++)
        gn[e] = NORM ? *reinterpret_cast<const uint2 *>(gain + min((e * kFusedThreads + tid) * 4, K - 4)) : make_uint2(0u, 0u);
    w.spins = 0;
    for (;;) {
        bool ready = true;
#pragma unroll
        for (int b = 0; b < NB; b++)
#pragma unroll
            for (int e = 0; e < GROUPS; e++) {
                const int k = min((e * kFusedThreads + tid) * 4, K - 4);     // past the end: the last four words again
                v[b][e] = ldc_u32x4(src, (uint32_t)(NB * K) * 4u, (uint32_t)(b * K + k) * 4u);
                ready = ready && v[b][e].x != kNotYet && v[b][e].y != kNotYet && v[b][e].z != kNotYet && v[b][e].w != kNotYet;
            }
        if (w.done(ready)) break;
    }
    float ss[NB];
#pragma unroll
    for (int b = 0; b < NB; b++) {
        ss[b] = 0.f;
#pragma unroll
        for (int e = 0; e < GROUPS; e++) {
            const int k = (e * kFusedThreads + tid) * 4;
            if (k < K) {
                float4 x = make_float4(__uint_as_float(v[b][e].x), __uint_as_float(v[b][e].y), __uint_as_float(v[b][e].z),
                                       __uint_as_float(v[b][e].w));
                ss[b] += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
                if (NORM) {
                    x.x *= bf16lo(gn[e].x); x.y *= bf16hi(gn[e].x);
                    x.z *= bf16lo(gn[e].y); x.w *= bf16hi(gn[e].y);
                }
                *reinterpret_cast<float4 *>(xs + b * K + k) = x;
            }
        }
    }
    if (NORM) {
#pragma unroll
        for (int b = 0; b < NB; b++) {
            const float s = sum64(ss[b]);
            if ((tid & 63) == 0) red[(tid >> 6) * NB + b] = s;
        }
    }
    __syncthreads();
    if (NORM) {
#pragma unroll
        for (int b = 0; b < NB; b++)
            rinv[b] = rsqrtf((red[b] + red[NB + b] + red[2 * NB + b] + red[3 * NB + b]) / (float)K + eps);
    }
}

template <int NB, bool NORM, int MAXE>
__device__ __forceinline__ void stage_input(const float *src, int K, const uint16_t *gain, float eps, float *xs,
                                            float (&rinv)[NB], float *red, Waiter &w)
{
    if constexpr (MAXE >= 16) {
        if ((K & 3) == 0) return stage_input_quads<NB, NORM, MAXE>(src, K, gain, eps, xs, rinv, red, w);
    }
    stage_input_words<NB, NORM, MAXE>(src, K, gain, eps, xs, rinv, red, w);
}

// The rows [r0, r1) of a matrix that a wave owns: rows of the block split over
// its waves, rows of the matrix split over the blocks.
__device__ __forceinline__ void block_rows(int N, int &b0, int &n)
{
    const int nb = gridDim.x, blk = blockIdx.x;
    b0 = (int)((long long)N * blk / nb);
    n = (int)((long long)N * (blk + 1) / nb) - b0;
}
__device__ __forceinline__ void wave_rows(int N, int wv, int &r0, int &r1)
{
    int b0, n;
    block_rows(N, b0, n);
    r0 = b0 + n * wv / kFusedWaves;
    r1 = b0 + n * (wv + 1) / kFusedWaves;
}

// Weights of up to RW rows x KS 512-element pieces, one 16-byte piece per lane.
//
// Q4 (4-bit codes, a bf16 scale and bias per 64 columns; layout of dk_create_model_q4): a lane
// holds 8 bytes = the 16 codes of half a lane-group unit, which all belong to ONE group, plus that
// group's (scale, bias) pair.  Unit c of a row (c = 0 .. K/16-1) is step c/8, lane group (c/2)%4,
// half c%2, and covers the columns step*128 + half*64 + lg*8 + {0..7} and the same + 32.
template <int RW, int KS, bool Q4 = false>
struct RowRegs {
    uint4 w[RW][KS];
};
template <int RW, int KS>
struct RowRegs<RW, KS, true> {
    static constexpr int KQ = (KS + 1) / 2;   // pieces of 64 units = 1024 columns
    uint2 w[RW][KQ];
    uint32_t sb[RW][KQ];
};
// N: rows of the whole matrix (Q4: the scale/bias tiles follow the N rows of codes)
template <int RW, int KS, bool Q4>
__device__ __forceinline__ void load_rows(RowRegs<RW, KS, Q4> &r, const uint16_t *W, int N, int K, int row0,
                                          int row_end, int lane)
{
    if constexpr (Q4) {
        const uint8_t *Wb = reinterpret_cast<const uint8_t *>(W);
        const int units = K >> 4, nks = K >> 7;
        const uint8_t *sbase = Wb + (long long)N * (K >> 1);
#pragma unroll
        for (int i = 0; i < RW; i++) {
            const int row = max(min(row0 + i, row_end - 1), 0);
            const uint8_t *codes = Wb + (long long)row * (K >> 1);
            const long long tile_off = (long long)(row >> 4) * nks * 128 + ((row & 15) >> 2) * 32 + (row & 3) * 4;
#pragma unroll
            for (int s = 0; s < RowRegs<RW, KS, true>::KQ; s++) {
                const int c = min(s * 64 + lane, units - 1);   // units past the row: a valid address, not used
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(codes + c * 8));   // used once per step
                r.w[i][s] = make_uint2(t.x, t.y);
                r.sb[i][s] = *reinterpret_cast<const uint32_t *>(sbase + tile_off + (c >> 3) * 128 + (c & 1) * 16);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < RW; i++)
#pragma unroll
            for (int s = 0; s < KS; s++) {
                const int k = s * 512 + lane * 8;
                // rows / pieces outside the matrix read a valid address and are not used
                const int row = min(row0 + i, row_end - 1);
                // used once per step: a streaming (non-temporal) request, so that the row does not push the rows
                // that were warmed for the coming stages out of the L2
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(W + (long long)max(row, 0) * K + min(k, K - 8)));
                r.w[i][s] = make_uint4(t.x, t.y, t.z, t.w);
            }
    }
}
// acc[i][b] = sum_k W[row0+i][k] * xs[b][k]   (all lanes get the sums)
template <int NB, int RW, int KS, bool Q4>
__device__ __forceinline__ void dot_rows(const RowRegs<RW, KS, Q4> &r, const float *xs, int K, int lane,
                                         float (&acc)[RW][NB])
{
#pragma unroll
    for (int i = 0; i < RW; i++)
#pragma unroll
        for (int b = 0; b < NB; b++) acc[i][b] = 0.f;
    if constexpr (Q4) {
#pragma unroll
        for (int s = 0; s < RowRegs<RW, KS, true>::KQ; s++) {
            const int c = s * 64 + lane;
            if (c < (K >> 4)) {
                const int k0 = (c >> 3) * 128 + (c & 1) * 64 + ((c >> 1) & 3) * 8;
                float xv[NB][16], sx[NB];
#pragma unroll
                for (int b = 0; b < NB; b++) {
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        const float4 lo = *reinterpret_cast<const float4 *>(xs + b * K + k0 + h * 32);
                        const float4 hi = *reinterpret_cast<const float4 *>(xs + b * K + k0 + h * 32 + 4);
                        xv[b][h * 8 + 0] = lo.x; xv[b][h * 8 + 1] = lo.y; xv[b][h * 8 + 2] = lo.z; xv[b][h * 8 + 3] = lo.w;
                        xv[b][h * 8 + 4] = hi.x; xv[b][h * 8 + 5] = hi.y; xv[b][h * 8 + 6] = hi.z; xv[b][h * 8 + 7] = hi.w;
                    }
                    float t = 0.f;
#pragma unroll
                    for (int e = 0; e < 16; e++) t += xv[b][e];
                    sx[b] = t;
                }
#pragma unroll
                for (int i = 0; i < RW; i++) {
                    const uint32_t cw[2] = {r.w[i][s].x, r.w[i][s].y};
                    float qf[16];
#pragma unroll
                    for (int h = 0; h < 2; h++)
#pragma unroll
                        for (int j = 0; j < 8; j++) qf[h * 8 + j] = (float)((cw[h] >> (4 * j)) & 15u);
                    const float sc = __uint_as_float(r.sb[i][s] << 16);
                    const float bi = __uint_as_float(r.sb[i][s] & 0xFFFF0000u);
#pragma unroll
                    for (int b = 0; b < NB; b++) {
                        float dq = 0.f;
#pragma unroll
                        for (int e = 0; e < 16; e++) dq += qf[e] * xv[b][e];
                        acc[i][b] += sc * dq + bi * sx[b];
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < KS; s++) {
            const int k = s * 512 + lane * 8;
            // long rows: the LDS reads of all pieces, hoisted to the top, would not fit the registers
            if (KS > 8 && (s & 3) == 0) __builtin_amdgcn_sched_barrier(0);
            if (k < K) {
                float xv[NB][8];
#pragma unroll
                for (int b = 0; b < NB; b++) {
                    const float4 lo = *reinterpret_cast<const float4 *>(xs + b * K + k);
                    const float4 hi = *reinterpret_cast<const float4 *>(xs + b * K + k + 4);
                    xv[b][0] = lo.x; xv[b][1] = lo.y; xv[b][2] = lo.z; xv[b][3] = lo.w;
                    xv[b][4] = hi.x; xv[b][5] = hi.y; xv[b][6] = hi.z; xv[b][7] = hi.w;
                }
#pragma unroll
                for (int i = 0; i < RW; i++) {
                    float wf[8];
                    unpack8(r.w[i][s], wf);
#pragma unroll
                    for (int b = 0; b < NB; b++)
#pragma unroll
                        for (int e = 0; e < 8; e++) acc[i][b] += wf[e] * xv[b][e];
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < RW; i++)
#pragma unroll
        for (int b = 0; b < NB; b++) acc[i][b] = sum64(acc[i][b]);
}

// A block hands a stage's result over with ONE coalesced store: the waves put
// their rows into LDS (`sm_y`, [NB][kFusedMaxBlockRows]) and, after a barrier,
// thread b*n + r stores element (batch row b, block row r).  Scattered 4-byte
// stores from 1024 waves made the hand-over measurably slower.
constexpr int kFusedMaxBlockRows = 64;

// sm_y[b][row - b0] = scale_b * W[row] . xs[b] for the wave's rows; the first RW
// rows come from `pre` (requested before the input was awaited).
template <int NB, int RW, int KS, bool Q4>
__device__ __forceinline__ void gemv_rows(RowRegs<RW, KS, Q4> &pre, const uint16_t *W, int N, int K, int r0, int r1,
                                          int b0, const float *xs, const float (&scale)[NB], float *sm_y, int lane)
{
    for (int rb = r0; rb < r1; rb += RW) {
        if (rb != r0) load_rows<RW, KS, Q4>(pre, W, N, K, rb, r1, lane);
        float acc[RW][NB];
        dot_rows<NB, RW, KS, Q4>(pre, xs, K, lane, acc);
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < RW; i++)
#pragma unroll
            for (int b = 0; b < NB; b++)
                if (lane == i * NB + b) v = acc[i][b] * scale[b];
        const int li = lane / NB, lb = lane - li * NB;
        if (lane < RW * NB && rb + li < r1) sm_y[lb * kFusedMaxBlockRows + rb + li - b0] = v;
    }
}

// The block's n rows starting at b0, for every batch row: out[copy][b][b0 + r] = sm_y[b][r] + rv, COPIES copies.
template <int NB, int COPIES = kFusedReplicas>
__device__ __forceinline__ void publish_rows(float *out, int N, int b0, int n, const float *sm_y, float rv)
{
    __syncthreads();
    const int tid = threadIdx.x;
    if (tid < n * NB) {
        const int b = tid / n, r = tid - b * n;
        const float y = sm_y[b * kFusedMaxBlockRows + r] + rv;
#pragma unroll
        for (int c = 0; c < COPIES; c++) stc_f32(out + ((long long)c * NB + b) * N + b0 + r, y);
    }
}

// Dynamic LDS of an instance: the stage input xs[NB][512 * max(KSH, KSQ, KSF)].
constexpr size_t fused_xs_bytes(int NB, int KSH, int KSQ, int KSF)
{
    return (size_t)NB * 512 * (KSF > KSQ ? (KSF > KSH ? KSF : KSH) : (KSQ > KSH ? KSQ : KSH)) * 4;
}

// STAMPS: the instance that records stage stamps (FusedArgs::stamps); the ordinary one has no trace of them
template <int NB, int D, int G, int KSH, int KSQ, int KSF, bool Q4 = false, bool STAMPS = false>
__global__ __launch_bounds__(kFusedThreads) void fused_step_kernel(FusedArgs a)
{
    constexpr int BS = 16, TPR = D / 8, TPW = 64 / TPR, NI = BS / TPW;
    // rows per wave in flight (registers: a row of K = 512 * KS columns is KS 16-byte pieces per lane)
    constexpr int RW_H = (KSH <= 2) ? 4 : (KSH <= 4 ? 2 : 1);   // K = hidden
    constexpr int RW_GU = (KSH <= 2) ? 3 : 1;                   // gate and up: two matrices
    constexpr int RW_Q = 1, RW_F = 1;                           // output and down projection
    constexpr int EP = (G * D + kFusedThreads - 1) / kFusedThreads;   // elements of a query group's output per thread
    constexpr int MERGE_ROUND = kFusedMergeRound / EP > 0 ? kFusedMergeRound / EP : 1;
    static_assert(D % 64 == 0, "a query head's elements fill whole waves (the collecting block fetches a chunk's maximum and sum once per wave)");
    extern __shared__ __attribute__((aligned(16))) float xs[];   // [NB][512 * max(KSH, KSQ, KSF)]: the stage's input (fused_xs_bytes)
    __shared__ float red[kFusedWaves * NB];
    __shared__ float sm_o[kFusedWaves][G][D];
    __shared__ float sm_ml[kFusedWaves][G][2];
    __shared__ float sm_qkv[(G + 2) * D];
    __shared__ unsigned wslots[2 * kFusedWaves];
    __shared__ float sm_y[NB * kFusedMaxBlockRows];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = blockIdx.x, nblk = gridDim.x;
    const int H = a.H, F = a.F, V = a.V, QD = a.nq * D, QKV = (a.nq + 2 * a.nkv) * D;
    const FusedLayout lay = fused_layout(a.L, NB, H, a.nq, a.nkv, D, F, a.nchunks, nblk);
    Waiter w{a.status, a.serial, 0, false, a.spin_limit, wslots, 0};
    const int copy = blk % kFusedReplicas;
    // stage stamps of one layer (100 MHz device clock), when the host asked for them: one flag per
    // layer, tested at every boundary
    long long *const stamp_to = a.stamps != nullptr ? a.stamps + (long long)blk * kFusedStamps : nullptr;
    bool stamp_on = false;
    auto stamp = [&](int i) {
        if constexpr (STAMPS) {
            if (stamp_on) stamp_to[i] = wall_clock64();
        }
    };
    // (12..15: the step itself - kernel entry, first layer begins, lm_head begins, lm_head streamed)
    auto stamp_step = [&](int i) {
        if constexpr (STAMPS) {
            if (stamp_to != nullptr && tid == 0) stamp_to[i] = wall_clock64();
        }
    };
    stamp_step(12);

    // refill the other buffer set for the next step
    {
        // (16 bytes per store; the set is 256-byte aligned, a block's share starts at a multiple of four words)
        uint32_t *o = reinterpret_cast<uint32_t *>(a.other_set);
        const long long per = ((a.set_floats + nblk - 1) / nblk + 3) & ~3LL;
        const long long lo = per * blk, hi = min(a.set_floats, lo + per);
        const long long hi4 = lo + ((hi - lo) & ~3LL);
        for (long long i = lo + 4 * tid; i < hi4; i += 4 * kFusedThreads)
            *reinterpret_cast<uint4 *>(o + i) = make_uint4(kNotYet, kNotYet, kNotYet, kNotYet);
        for (long long i = hi4 + tid; i < hi; i += kFusedThreads) o[i] = kNotYet;
    }

    // sequence state of the step (constant until the very end)
    int T[NB], nact[NB];
#pragma unroll
    for (int b = 0; b < NB; b++) {
        T[b] = min(max(a.seq_lens[b], 0), a.max_blocks * BS - 1);
        nact[b] = min((T[b] + 1 + kFusedChunk - 1) / kFusedChunk, a.nchunks);
    }

    // ---- stage 0: x0 = embedding rows, straight into LDS; q|k|v weights ahead ----
    int r0, r1, qkv_b0, qkv_n, h_b0, h_n, f_b0, f_n;
    wave_rows(QKV, wv, r0, r1);
    block_rows(QKV, qkv_b0, qkv_n);
    block_rows(H, h_b0, h_n);
    block_rows(F, f_b0, f_n);
    // The embedding rows are requested before the first weight rows (requests return in order: behind the 8 MB
    // that all blocks ask for at once they would arrive microseconds later), all of a thread's elements together.
    constexpr int EM = 2 * KSH;                    // H <= 256 * EM
    uint16_t ex[NB][EM], eg[EM];
#pragma unroll
    for (int e = 0; e < EM; e++) {
        const int k = min(e * kFusedThreads + tid, H - 1);
        eg[e] = a.layers[0].g_attn[k];
#pragma unroll
        for (int b = 0; b < NB; b++) ex[b][e] = a.embed[(long long)min(max(a.tokens[b], 0), V - 1) * H + k];
    }
    RowRegs<RW_H, KSH, Q4> pre_h;
    load_rows<RW_H, KSH, Q4>(pre_h, a.layers[0].w_qkv, QKV, H, r0, r1, lane);
    float rinv[NB], ones[NB];
#pragma unroll
    for (int b = 0; b < NB; b++) ones[b] = 1.f;
    {
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; b++) {
            ss[b] = 0.f;
#pragma unroll
            for (int e = 0; e < EM; e++) {
                const int k = e * kFusedThreads + tid;
                if (k < H) {
                    const float x = bf16_to_f32(ex[b][e]);
                    ss[b] += x * x;
                    xs[b * H + k] = x * bf16_to_f32(eg[e]);
                }
            }
            const float s = sum64(ss[b]);
            if (lane == 0) red[wv * NB + b] = s;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NB; b++)
            rinv[b] = rsqrtf((red[b] + red[NB + b] + red[2 * NB + b] + red[3 * NB + b]) / (float)H + a.eps);
    }

    // rotary (cos, sin) of this block's attention row, computed once per step
    const int dl = (lane % TPR) * 8, sub = lane / TPR;
    const bool upper = dl >= D / 2;
    const int items = NB * a.nkv * a.nchunks;
    float2 cs[8];
    int cs_row = -1;
    // The block's first attention item is the same in every layer, and where its tiles sit in a
    // layer's slab of the pool does not depend on the layer: the block-table entries are looked
    // up once, so that a layer's tile requests (and the q|k|v polls queued behind them) do not
    // wait for a table load first.
    int first_phys[kFusedWaveTiles], first_phys_new = 0;
#pragma unroll
    for (int u = 0; u < kFusedWaveTiles; u++) first_phys[u] = 0;
    if (blk < items) {
        const int c = blk % a.nchunks, j = (blk / a.nchunks) % a.nkv, b = blk / (a.nchunks * a.nkv);
        const int *table = a.block_tables + (long long)b * a.max_blocks;
#pragma unroll
        for (int u = 0; u < kFusedWaveTiles; u++)
            first_phys[u] = min(max(table[min(c * kFusedChunk / BS + wv + u * kFusedWaves, a.max_blocks - 1)], 0), a.num_blocks - 1);
        first_phys_new = min(max(table[T[b] / BS], 0), a.num_blocks - 1);
        (void)j;
    }

    // The MLP's weights are requested a first time while attention runs - most blocks have nothing to do then
    // and HBM is idle - so that the requests in front of the MLP's hand-overs find them in the die's L2: those
    // hand-overs are then as long as the hand-over takes, not as long as the burst of weight requests in front of
    // the polls.  (The narrow classes only: the wide ones stream more per block than the L2 can hold for them.)
    constexpr bool WARM = KSH <= 2 && KSF <= 8;
    uint32_t sink = 0;
    WarmWords<1> wg{}, wu{}, wd{}, wg2{}, wu2{}, wd2{};
    for (int l = 0; l < a.L; l++) {
        const FusedLayer &Lw = a.layers[l];
        if constexpr (STAMPS) stamp_on = stamp_to != nullptr && l == a.stamp_layer && tid == 0;
        if (l == 0) stamp_step(13);
        stamp(0);    // layer begins (input staged, q|k|v rows requested)
        float *base = a.set + lay.per_layer * l;
        float *b_qkv = base + lay.qkv, *b_part = base + lay.part, *b_attn = base + lay.attn, *b_xmid = base + lay.xmid;
        float *b_act = base + lay.act, *b_xout = base + lay.xout;
        // this block's copy of the replicated vectors
        const float *my_attn = b_attn + (long long)copy * NB * QD, *my_xmid = b_xmid + (long long)copy * NB * H;
        const float *my_act = b_act + (long long)copy * NB * F, *my_xout = b_xout + (long long)copy * NB * H;
        const float *x_in = l ? a.set + lay.per_layer * (l - 1) + lay.xout + (long long)copy * NB * H : nullptr;   // layer 0: embedding

        // ---- q|k|v = W_qkv rmsnorm(x) ------------------------------------------------
        gemv_rows<NB, RW_H, KSH, Q4>(pre_h, Lw.w_qkv, QKV, H, r0, r1, qkv_b0, xs, rinv, sm_y, lane);
        publish_rows<NB, 1>(b_qkv, QKV, qkv_b0, qkv_n, sm_y, 0.f);
        stamp(1);    // q|k|v rows handed over
        // ---- attention: request the K/V tiles, then wait for q|k|v --------------------
        RowRegs<RW_Q, KSQ, Q4> pre_q;
        int q0, q1;
        wave_rows(H, wv, q0, q1);
        load_rows<RW_Q, KSQ, Q4>(pre_q, Lw.w_o, H, QD, q0, q1, lane);
        // the residual of the element this thread will publish: the layer's input, which is
        // the embedding row (layer 0) or the previous x_out (complete: the block consumed it)
        float rv_o = 0.f;
        if (tid < h_n * NB) {
            const int b = tid / h_n, r = tid - b * h_n;
            if (l == 0) {
                const int tok = min(max(a.tokens[b], 0), V - 1);
                rv_o = bf16_to_f32(a.embed[(long long)tok * H + h_b0 + r]);
            } else {
                rv_o = __uint_as_float(ldc_u32(x_in + (long long)b * H + h_b0 + r));
            }
        }
        if constexpr (WARM) {
            // Only blocks without work in this layer's attention warm, and not at once: the attention blocks' K/V
            // tiles and the q|k|v hand-over come first.  A block with an attention item has a partner among the
            // idle blocks of its die - `pair` blocks further on, a multiple of 8 - that warms its rows for it.
            auto attends = [&](int who) {
                const int c = who % a.nchunks, b = who / (a.nchunks * a.nkv);
                return who < items && c < nact[min(b, NB - 1)];
            };
            auto warm_rows_of = [&](int who, WarmWords<1> &g, WarmWords<1> &u, WarmWords<1> &d) {
                const int fb = (int)((long long)F * who / nblk), fn = (int)((long long)F * (who + 1) / nblk) - fb;
                const int hb = (int)((long long)H * who / nblk), hn = (int)((long long)H * (who + 1) / nblk) - hb;
                if constexpr (Q4) {   // the rows' 4-bit codes (half a byte per column; the scales, an eighth of that, are left)
                    g = warm_l2<1>(reinterpret_cast<const uint8_t *>(Lw.w_gate) + (long long)fb * (H >> 1), fn * (H >> 1));
                    u = warm_l2<1>(reinterpret_cast<const uint8_t *>(Lw.w_up) + (long long)fb * (H >> 1), fn * (H >> 1));
                    d = warm_l2<1>(reinterpret_cast<const uint8_t *>(Lw.w_down) + (long long)hb * (F >> 1), hn * (F >> 1));
                } else {
                    g = warm_l2<1>(Lw.w_gate + (long long)fb * H, fn * H * 2);
                    u = warm_l2<1>(Lw.w_up + (long long)fb * H, fn * H * 2);
                    d = warm_l2<1>(Lw.w_down + (long long)hb * F, hn * F * 2);
                }
            };
            if (!attends(blk)) {
                const int pair = (min(items, nblk) + 7) & ~7;
                __builtin_amdgcn_s_sleep(kFusedWarmDelay);
                warm_rows_of(blk, wg, wu, wd);
                if (blk >= pair && attends(blk - pair)) warm_rows_of(blk - pair, wg2, wu2, wd2);
            }
        }
        for (int item = blk; item < items; item += nblk) {
            const int c = item % a.nchunks, j = (item / a.nchunks) % a.nkv, b = item / (a.nchunks * a.nkv);
            if (c >= nact[b]) continue;
            const int *table = a.block_tables + (long long)b * a.max_blocks;
            const int t0 = c * kFusedChunk, t1 = min(T[b], t0 + kFusedChunk);
            const bool owns_new = (c == nact[b] - 1);
            const bool norm = Lw.g_q != nullptr;
            // the head-norm gains are only requested here and unpacked once q has arrived (used on
            // the spot they would hold up the tile requests below for a round trip)
            const uint4 gq_raw = ld16((norm ? Lw.g_q : Lw.g_attn) + dl), gk_raw = ld16((norm ? Lw.g_k : Lw.g_attn) + dl);
            const bool first_item = item == blk;
            // this wave's tiles: t0/16 + wv (+ 4, + 8 ... when a chunk has more tiles than waves)
            uint4 kw[kFusedWaveTiles][NI], vw[kFusedWaveTiles][NI];
#pragma unroll
            for (int u = 0; u < kFusedWaveTiles; u++) {
                int phys = first_phys[u];
                if (!first_item) {
                    const int tb = min(t0 / BS + wv + u * kFusedWaves, a.max_blocks - 1);
                    phys = min(max(table[tb], 0), a.num_blocks - 1);
                }
                const uint16_t *kt = a.pool + kv_tile_offset(l, a.num_blocks, phys, 0, a.nkv, j, BS, D);
                const uint16_t *vt = kt + (long long)a.nkv * BS * D;
#pragma unroll
                for (int i = 0; i < NI; i++) {
                    kw[u][i] = ld16(kt + i * 512 + lane * 8);
                    vw[u][i] = ld16(vt + i * 512 + lane * 8);
                }
            }
            if (cs_row != b) {
                cs_row = b;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const int i = (upper ? dl - D / 2 : dl) + e;
                    double s_, c_;
                    sincos((double)T[b] * a.inv_freq[i], &s_, &c_);
                    cs[e] = make_float2((float)c_, (float)s_);
                }
            }
            // wait for this (row, kv head)'s q heads and new k, v: each word is fetched once per block
            {
                constexpr int NW = (G + 2) * D, PE = (NW + kFusedThreads - 1) / kFusedThreads;
                const float *rowp = b_qkv + (long long)b * QKV;
                const float *src[PE];
                uint32_t got[PE];
#pragma unroll
                for (int e = 0; e < PE; e++) {
                    const int idx = e * kFusedThreads + tid;
                    const int part = idx / D, dim = idx - part * D;   // part: G query heads, then k, then v
                    const int head = part < G ? j * G + part : (part == G ? a.nq + j : a.nq + a.nkv + j);
                    src[e] = rowp + (long long)head * D + dim;     // threads past the last word repeat a word of v
                }
                w.spins = 0;
                for (;;) {
                    bool ready = true;
#pragma unroll
                    for (int e = 0; e < PE; e++) {
                        got[e] = ldc_u32(src[e]);
                        ready = ready && got[e] != kNotYet;
                    }
                    if (w.done(ready)) break;
                }
                stamp(2);    // q|k|v of the block's attention item arrived
#pragma unroll
                for (int e = 0; e < PE; e++)
                    if (e * kFusedThreads + tid < NW) sm_qkv[e * kFusedThreads + tid] = __uint_as_float(got[e]);
                __syncthreads();
            }
            float gq[8], gk[8];
            unpack8(gq_raw, gq);
            unpack8(gk_raw, gk);
            if (!norm) {
#pragma unroll
                for (int e = 0; e < 8; e++) gq[e] = gk[e] = 1.f;
            }
            float q[G][8], kn[8], vn[8];
#pragma unroll
            for (int e = 0; e < 8; e++) {
#pragma unroll
                for (int g = 0; g < G; g++) q[g][e] = sm_qkv[g * D + dl + e];
                kn[e] = sm_qkv[G * D + dl + e];
                vn[e] = sm_qkv[(G + 1) * D + dl + e];
            }
#pragma unroll
            for (int g = 0; g < G; g++) {
                head_norm_rope<D>(q[g], norm, gq, a.eps, cs, upper);
#pragma unroll
                for (int e = 0; e < 8; e++) q[g][e] *= a.scale;
            }
            float m[G], lsum[G], o[G][8];
#pragma unroll
            for (int g = 0; g < G; g++) {
                m[g] = -1e30f;
                lsum[g] = 0.f;
#pragma unroll
                for (int e = 0; e < 8; e++) o[g][e] = 0.f;
            }
            if (owns_new && wv == 0) {
                head_norm_rope<D>(kn, norm, gk, a.eps, cs, upper);
                uint32_t kb[4], vb[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const uint32_t k0 = f32_to_bf16_rne(kn[2 * e]), k1 = f32_to_bf16_rne(kn[2 * e + 1]);
                    const uint32_t v0 = f32_to_bf16_rne(vn[2 * e]), v1 = f32_to_bf16_rne(vn[2 * e + 1]);
                    kb[e] = k0 | (k1 << 16);
                    vb[e] = v0 | (v1 << 16);
                    kn[2 * e] = __uint_as_float(k0 << 16); kn[2 * e + 1] = __uint_as_float(k1 << 16);
                    vn[2 * e] = __uint_as_float(v0 << 16); vn[2 * e + 1] = __uint_as_float(v1 << 16);
                }
                if (sub == 0) {
                    int phys = first_phys_new;
                    if (!first_item) phys = min(max(table[T[b] / BS], 0), a.num_blocks - 1);
                    uint16_t *kt = a.pool + kv_tile_offset(l, a.num_blocks, phys, 0, a.nkv, j, BS, D) +
                                   (T[b] % BS) * D + dl;
                    uint16_t *vt = kt + (long long)a.nkv * BS * D;
                    *reinterpret_cast<uint4 *>(kt) = make_uint4(kb[0], kb[1], kb[2], kb[3]);
                    *reinterpret_cast<uint4 *>(vt) = make_uint4(vb[0], vb[1], vb[2], vb[3]);
                }
#pragma unroll
                for (int g = 0; g < G; g++) {
                    float p = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; e++) p += q[g][e] * kn[e];
                    p = (TPR == 16) ? sum16(p) : sum8(p);
                    if (sub == 0) {
                        m[g] = p;
                        lsum[g] = 1.f;
#pragma unroll
                        for (int e = 0; e < 8; e++) o[g][e] = vn[e];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kFusedWaveTiles; u++) {
                const int tile = t0 / BS + wv + u * kFusedWaves;
                float s[NI][G];
                bool valid[NI];
#pragma unroll
                for (int i = 0; i < NI; i++) {
                    valid[i] = (tile * BS + i * TPW + sub) < t1;
                    float kf[8];
                    unpack8(kw[u][i], kf);
#pragma unroll
                    for (int g = 0; g < G; g++) {
                        float p = 0.f;
#pragma unroll
                        for (int e = 0; e < 8; e++) p += q[g][e] * kf[e];
                        p = (TPR == 16) ? sum16(p) : sum8(p);
                        s[i][g] = valid[i] ? p : -1e30f;
                    }
                }
#pragma unroll
                for (int g = 0; g < G; g++) {
                    float mn = m[g];
#pragma unroll
                    for (int i = 0; i < NI; i++) mn = fmaxf(mn, s[i][g]);
                    const float alpha = __expf(m[g] - mn);
                    m[g] = mn;
                    lsum[g] *= alpha;
#pragma unroll
                    for (int e = 0; e < 8; e++) o[g][e] *= alpha;
                }
#pragma unroll
                for (int i = 0; i < NI; i++) {
                    float vf[8];
                    unpack8(vw[u][i], vf);
#pragma unroll
                    for (int g = 0; g < G; g++) {
                        const float p = valid[i] ? __expf(s[i][g] - m[g]) : 0.f;
                        lsum[g] += p;
#pragma unroll
                        for (int e = 0; e < 8; e++) o[g][e] += valid[i] ? p * vf[e] : 0.f;
                    }
                }
            }
            // merge the token groups of the wave, then the waves
#pragma unroll
            for (int off = TPR; off < 64; off <<= 1) {
#pragma unroll
                for (int g = 0; g < G; g++) {
                    const float om = __shfl_xor(m[g], off), ol = __shfl_xor(lsum[g], off);
                    const float mn = fmaxf(m[g], om);
                    const float sa = __expf(m[g] - mn), sb = __expf(om - mn);
                    lsum[g] = lsum[g] * sa + ol * sb;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const float oo = __shfl_xor(o[g][e], off);
                        o[g][e] = o[g][e] * sa + oo * sb;
                    }
                    m[g] = mn;
                }
            }
            if (lane < TPR) {
#pragma unroll
                for (int g = 0; g < G; g++) {
#pragma unroll
                    for (int e = 0; e < 8; e++) sm_o[wv][g][dl + e] = o[g][e];
                    if (lane == 0) { sm_ml[wv][g][0] = m[g]; sm_ml[wv][g][1] = lsum[g]; }
                }
            }
            __syncthreads();
            stamp(3);    // the chunk's scores, softmax and weighted values done
            // thread tid owns the elements tid, tid + 256, ... (g, dim) of the chunk's result
            bool has[EP];
            int g_[EP], dim[EP];
            float mn[EP], ls[EP], os[EP];
            const float *pg[EP];
#pragma unroll
            for (int x = 0; x < EP; x++) {
                const int idx = x * kFusedThreads + tid;
                has[x] = idx < G * D;
                g_[x] = has[x] ? idx / D : 0;
                dim[x] = has[x] ? idx - g_[x] * D : 0;
                mn[x] = sm_ml[0][g_[x]][0];
#pragma unroll
                for (int ww = 1; ww < kFusedWaves; ww++) mn[x] = fmaxf(mn[x], sm_ml[ww][g_[x]][0]);
                ls[x] = 0.f;
                os[x] = 0.f;
#pragma unroll
                for (int ww = 0; ww < kFusedWaves; ww++) {
                    const float sc = __expf(sm_ml[ww][g_[x]][0] - mn[x]);
                    ls[x] += sm_ml[ww][g_[x]][1] * sc;
                    os[x] += sm_o[ww][g_[x]][dim[x]] * sc;
                }
                pg[x] = b_part + (((long long)b * a.nkv + j) * a.nchunks) * (G * (D + 2)) + g_[x] * (D + 2);
            }
            if (c != 0) {
                // a later chunk: hand the partial to the block of chunk 0
#pragma unroll
                for (int x = 0; x < EP; x++)
                    if (has[x]) {
                        float *pp = const_cast<float *>(pg[x]) + (long long)c * (G * (D + 2));
                        stc_f32(pp + dim[x], os[x]);
                        if (dim[x] == 0) { stc_f32(pp + D, mn[x]); stc_f32(pp + D + 1, ls[x]); }
                    }
            } else {
                // chunk 0 collects the other chunks of its (row, kv head) in order and
                // publishes the finished attention output
                // a round awaits ROUND chunks at once; its size follows the number of chunks, so that a short
                // context does not poll (and wait for) repeats of its last chunk
                auto merge_rounds = [&](auto round_tag) {
                    constexpr int ROUND = decltype(round_tag)::value;
                    for (int c0 = 1; c0 < nact[b]; c0 += ROUND) {
                        uint32_t uml[EP][ROUND], uo[EP][ROUND];
                        w.spins = 0;
                        for (;;) {
                            bool ready = true;
                            // every request is unconditional (chunks past the last repeat it, threads
                            // without an element read element 0): a load inside a condition is waited
                            // for on the spot, and a round of polls would be a chain of round trips
#pragma unroll
                            for (int x = 0; x < EP; x++)
#pragma unroll
                                for (int u = 0; u < ROUND; u++) {
                                    const float *pp = pg[x] + (long long)min(c0 + u, nact[b] - 1) * (G * (D + 2));
                                    // (maximum, sum) of the chunk: even lanes fetch the one, odd lanes the other -
                                    // a query head's elements fill whole waves, so one request serves a wave
                                    uml[x][u] = ldc_u32(pp + D + (lane & 1));
                                    uo[x][u] = ldc_u32(pp + dim[x]);
                                    ready = ready && uml[x][u] != kNotYet && uo[x][u] != kNotYet;
                                }
                            if (w.done(ready)) break;
                        }
#pragma unroll
                        for (int x = 0; x < EP; x++)
#pragma unroll
                            for (int u = 0; u < ROUND; u++)
                                if (c0 + u < nact[b]) {
                                    const float mc = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)uml[x][u], 0));
                                    const float lc = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)uml[x][u], 1));
                                    const float oc = __uint_as_float(uo[x][u]);
                                    const float m2 = fmaxf(mn[x], mc);
                                    const float sa = __expf(mn[x] - m2), sb = __expf(mc - m2);
                                    ls[x] = ls[x] * sa + lc * sb;
                                    os[x] = os[x] * sa + oc * sb;
                                    mn[x] = m2;
                                }
                    }
                };
                // the smallest of the instantiated round sizes (multiples of ROUND_STEP) that takes all chunks at once
                constexpr int ROUND_STEP = MERGE_ROUND >= 6 ? MERGE_ROUND / 6 : 1;
                auto pick_round = [&](auto self, auto round_tag) -> void {
                    constexpr int ROUND = decltype(round_tag)::value;
                    if constexpr (ROUND + ROUND_STEP > MERGE_ROUND) {
                        merge_rounds(std::integral_constant<int, MERGE_ROUND>{});
                    } else {
                        if (nact[b] - 1 <= ROUND) merge_rounds(round_tag);
                        else self(self, std::integral_constant<int, ROUND + ROUND_STEP>{});
                    }
                };
                pick_round(pick_round, std::integral_constant<int, ROUND_STEP>{});
#pragma unroll
                for (int x = 0; x < EP; x++)
                    if (has[x]) {
                        const float y = os[x] / ls[x];
#pragma unroll
                        for (int cp = 0; cp < kFusedReplicas; cp++)
                            stc_f32(b_attn + ((long long)cp * NB + b) * QD + (long long)(j * G + g_[x]) * D + dim[x], y);
                    }
                stamp(4);    // (collecting blocks) merged attention output handed over
            }
            __syncthreads();   // sm_o / sm_ml / sm_qkv are rewritten by the block's next item
        }
        // ---- x_mid = x + W_o attn -------------------------------------------------------------
        {
            float dummy[NB];
            stage_input<NB, false, 2 * KSQ>(my_attn, QD, nullptr, a.eps, xs, dummy, red, w);
            stamp(5);    // attention output arrived
            gemv_rows<NB, RW_Q, KSQ, Q4>(pre_q, Lw.w_o, H, QD, q0, q1, h_b0, xs, ones, sm_y, lane);
            publish_rows<NB>(b_xmid, H, h_b0, h_n, sm_y, rv_o);
            stamp(6);    // x_mid rows handed over
        }
        // ---- act = silu(W_g h) * (W_u h), h = rmsnorm(x_mid) ----------------------------
        {
            int f0, f1;
            wave_rows(F, wv, f0, f1);
            RowRegs<RW_GU, KSH, Q4> pg, pu;
            load_rows<RW_GU, KSH, Q4>(pg, Lw.w_gate, F, H, f0, f1, lane);
            load_rows<RW_GU, KSH, Q4>(pu, Lw.w_up, F, H, f0, f1, lane);
            __syncthreads();   // xs is about to be overwritten
            stage_input<NB, true, 2 * KSH>(my_xmid, H, Lw.g_mlp, a.eps, xs, rinv, red, w);
            stamp(7);    // x_mid arrived
            if constexpr (WARM) sink ^= wg.w[0] ^ wu.w[0] ^ wd.w[0] ^ wg2.w[0] ^ wu2.w[0] ^ wd2.w[0];
            for (int rb = f0; rb < f1; rb += RW_GU) {
                if (rb != f0) {
                    load_rows<RW_GU, KSH, Q4>(pg, Lw.w_gate, F, H, rb, f1, lane);
                    load_rows<RW_GU, KSH, Q4>(pu, Lw.w_up, F, H, rb, f1, lane);
                }
                float ag[RW_GU][NB], au[RW_GU][NB];
                dot_rows<NB, RW_GU, KSH, Q4>(pg, xs, H, lane, ag);
                dot_rows<NB, RW_GU, KSH, Q4>(pu, xs, H, lane, au);
                float v = 0.f;
#pragma unroll
                for (int i = 0; i < RW_GU; i++)
#pragma unroll
                    for (int b = 0; b < NB; b++)
                        if (lane == i * NB + b) {
                            const float z = ag[i][b] * rinv[b];
                            v = z / (1.0f + __expf(-z)) * (au[i][b] * rinv[b]);
                        }
                const int li = lane / NB, lb = lane - li * NB;
                if (lane < RW_GU * NB && rb + li < f1) sm_y[lb * kFusedMaxBlockRows + rb + li - f_b0] = v;
            }
            publish_rows<NB>(b_act, F, f_b0, f_n, sm_y, 0.f);
            stamp(8);    // activations handed over
        }
        // ---- x_out = x_mid + W_d act ------------------------------------------------------
        {
            int d0, d1;
            wave_rows(H, wv, d0, d1);
            // (a row of more than 8192 columns and the polled activations do not fit the registers
            // together: such a row is requested after the wait instead of before it)
            constexpr bool ROW_AHEAD = KSF <= 16;
            RowRegs<RW_F, KSF, Q4> pd;
            if (ROW_AHEAD) load_rows<RW_F, KSF, Q4>(pd, Lw.w_down, H, F, d0, d1, lane);
            float rv_d = 0.f;
            if (tid < h_n * NB) {
                const int b = tid / h_n, r = tid - b * h_n;
                rv_d = __uint_as_float(ldc_u32(my_xmid + (long long)b * H + h_b0 + r));
            }
            __syncthreads();
            float dummy[NB];
            stage_input<NB, false, 2 * KSF>(my_act, F, nullptr, a.eps, xs, dummy, red, w);
            stamp(9);    // activations arrived
            if (!ROW_AHEAD) load_rows<RW_F, KSF, Q4>(pd, Lw.w_down, H, F, d0, d1, lane);
            gemv_rows<NB, RW_F, KSF, Q4>(pd, Lw.w_down, H, F, d0, d1, h_b0, xs, ones, sm_y, lane);
            publish_rows<NB>(b_xout, H, h_b0, h_n, sm_y, rv_d);
            stamp(10);   // x_out rows handed over
        }
        // ---- next layer's q|k|v weights ahead, then its input --------------------------------
        if (l + 1 < a.L) {
            load_rows<RW_H, KSH, Q4>(pre_h, a.layers[l + 1].w_qkv, QKV, H, r0, r1, lane);
            __syncthreads();
            stage_input<NB, true, 2 * KSH>(my_xout, H, a.layers[l + 1].g_attn, a.eps, xs, rinv, red, w);
            stamp(11);   // next layer's input arrived
        }
    }

    // ---- logits = W_lm rmsnorm(x); per-block maxima; block 0 picks the tokens ------------------
    stamp_step(14);
    {
        int v0, v1;
        wave_rows(V, wv, v0, v1);
        // a ring of PF batches of RW_H rows stays requested: one batch ahead leaves the wave
        // waiting a full HBM round trip per batch (a third of the bandwidth)
        constexpr int PF = 4;
        RowRegs<RW_H, KSH, Q4> ring[PF];
#pragma unroll
        for (int p = 0; p < PF; p++) load_rows<RW_H, KSH, Q4>(ring[p], a.lm_head, V, H, v0 + p * RW_H, v1, lane);
        __syncthreads();
        // (the warmed words have to end somewhere: a store that never happens - the wait limit is positive)
        if (WARM && a.spin_limit < 0 && sink == 0x5bd1e995u) a.status[1] = sink;
        const float *x_last = a.set + lay.per_layer * (a.L - 1) + lay.xout + (long long)copy * NB * H;
        stage_input<NB, true, 2 * KSH>(x_last, H, a.g_final, a.eps, xs, rinv, red, w);
        float best[NB];
        int best_i[NB];
#pragma unroll
        for (int b = 0; b < NB; b++) { best[b] = -INFINITY; best_i[b] = 0x7fffffff; }
        for (int rb0 = v0; rb0 < v1; rb0 += RW_H * PF) {
#pragma unroll
            for (int p = 0; p < PF; p++) {
                const int rb = rb0 + p * RW_H;
                float acc[RW_H][NB];
                dot_rows<NB, RW_H, KSH, Q4>(ring[p], xs, H, lane, acc);
                // refill the slot (rows past the end re-read the last row and are not used)
                load_rows<RW_H, KSH, Q4>(ring[p], a.lm_head, V, H, rb + RW_H * PF, v1, lane);
#pragma unroll
                for (int i = 0; i < RW_H; i++)
#pragma unroll
                    for (int b = 0; b < NB; b++) {
                        const float v = acc[i][b] * rinv[b];
                        if (rb + i < v1) {
                            if (v > best[b]) { best[b] = v; best_i[b] = rb + i; }   // rows ascend: ties keep the lower
                            if (a.logits != nullptr && lane == i * NB + b) a.logits[(long long)b * V + rb + i] = v;
                        }
                    }
            }
        }
        stamp_step(15);
        // block maximum per row of the batch: waves own ascending row ranges
        __syncthreads();
        float *sv = xs;                       // reuse LDS: [wave][b] values and indices
        int *si = reinterpret_cast<int *>(xs + kFusedWaves * NB);
        if (lane == 0) {
#pragma unroll
            for (int b = 0; b < NB; b++) { sv[wv * NB + b] = best[b]; si[wv * NB + b] = best_i[b]; }
        }
        __syncthreads();
        float *amax = a.set + lay.amax;
        if (tid < NB) {
            float bv = sv[tid];
            int bi = si[tid];
            for (int ww = 1; ww < kFusedWaves; ww++)
                if (sv[ww * NB + tid] > bv) { bv = sv[ww * NB + tid]; bi = si[ww * NB + tid]; }
            stc_f32(amax + 2 * ((long long)blk * NB + tid), bv);
            // a block without rows reports index -1 (0x7fffffff would read as "not yet"); a block
            // that gave up a wait (or saw another give up) reports -2: the verdict travels with the
            // data block 0 waits for, so no ordering between this store and the abort word is needed
            stc_f32(amax + 2 * ((long long)blk * NB + tid) + 1,
                    __int_as_float(w.aborted ? -2 : (bi == 0x7fffffff ? -1 : bi)));
        }
        if (blk != 0) return;
        // block 0: all per-block maxima (blocks own ascending row ranges)
        for (int b = 0; b < NB; b++) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
            bool some_gave_up = false;
            w.spins = 0;
            for (;;) {
                bool ready = true;
                bv = -INFINITY;
                bi = 0x7fffffff;
                some_gave_up = false;
                for (int i = tid; i < nblk; i += kFusedThreads) {
                    const uint32_t uv = ldc_u32(amax + 2 * ((long long)i * NB + b));
                    const uint32_t ui = ldc_u32(amax + 2 * ((long long)i * NB + b) + 1);
                    ready = ready && uv != kNotYet && ui != kNotYet;
                    const float v = __uint_as_float(uv);
                    const int ix = (int)ui;
                    some_gave_up = some_gave_up || ix == -2;
                    if (ix >= 0 && (v > bv || (v == bv && ix < bi))) { bv = v; bi = ix; }
                }
                if (w.done(ready)) break;
            }
            some_gave_up = __syncthreads_or(some_gave_up);
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oi = __shfl_xor(bi, off);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            __syncthreads();
            if (lane == 0) { sv[wv] = bv; si[wv] = bi; }
            __syncthreads();
            if (tid == 0) {
                for (int ww = 1; ww < kFusedWaves; ww++)
                    if (sv[ww] > bv || (sv[ww] == bv && si[ww] < bi)) { bv = sv[ww]; bi = si[ww]; }
                if (bi == 0x7fffffff) bi = 0;
                // a step in which some block gave up a wait has no valid result: it says so
                // with the token -1 and does not advance the sequence
                const bool gave_up = w.aborted || some_gave_up || ldc_u32(a.status) == a.serial;
                a.next[b] = gave_up ? -1 : bi;
                if (a.advance && !gave_up) {
                    a.tokens[b] = bi;
                    a.seq_lens[b] += 1;
                }
            }
        }
    }
}

// Fills both buffer sets with the "not written yet" pattern (first use of a workspace).
__global__ __launch_bounds__(256) void fused_fill_kernel(uint32_t *p, long long n, unsigned *status)
{
    const long long i0 = (long long)blockIdx.x * 256 + threadIdx.x, stride = (long long)gridDim.x * 256;
    for (long long i = i0; i < n; i += stride) p[i] = kNotYet;
    if (i0 == 0) { status[0] = 0; status[1] = 0; }
}

}  // namespace dk
