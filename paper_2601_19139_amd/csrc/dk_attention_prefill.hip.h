// Attention for a chunk of consecutive prompt positions of ONE sequence
// (chunked prefill) on the matrix cores.
//
// The rows of such a chunk share the block table and all but the last few
// positions of their context, so the 16 MFMA columns that the decode kernel
// fills with the G query heads of one row are filled here with the G heads of
// RPB = 16 / G consecutive rows: a K/V tile is read (and multiplied) once for
// RPB rows instead of once per row.  Column col = (row in group) * G + head.
//
// Every row's own k and v are already in the pool (prefill_append_kernel runs
// first), so there is no "new token" special case: column col attends to the
// positions 0..T(col) of the pool, and the causal mask inside the group is the
// per-column limit.  The inner loop is the decode kernel's (mfma_attend_tile_pair:
// scores = K q with q as three bf16 terms, online softmax per column, output = P V
// with V staged in LDS and fetched with the LDS transpose read), given that limit.  A tile past a column's limit contributes exactly nothing to it, and an
// empty chunk partial merges as exactly nothing, so a row's result depends on
// the chunk length only, not on which rows share its group.
//
// K/V come from the L2 here (every tile is read by all row groups), and the kernel
// is bound by its instructions, not by the stream: a wave requests its tile pair
// and uses it in the same iteration, three blocks per compute unit cover the
// latency (holding the next pair in registers as the decode kernel does costs the
// third block: measured slower from 2 k tokens of context on).
//
// grid = (kv heads, chunks, row groups); chunk partials of a (group, kv head)
// are merged, in chunk order, by the block that takes its last ticket.  The kv
// head is the fastest block index: consecutive blocks go to consecutive compute
// dies, so a die's L2 sees the K/V of its own heads only (each tile is read by
// all groups), and a short context, with one active chunk, still spreads over
// all dies.
#pragma once
#include "dk_attention_mfma.hip.h"

namespace dk {

template <int D, int G>
__global__ __launch_bounds__(256, 3) void prefill_attention_kernel(AttnArgs a)
{
    constexpr int BS = 16;            // tokens per block tile
    constexpr int TPR = D / 8;        // lanes per head vector in the row-major prologue
    constexpr int TPW = 64 / TPR;     // head vectors per wave in the prologue / tokens per wave load
    constexpr int NI = BS / TPW;      // wave loads per V tile
    constexpr int NS = D / 32;        // MFMAs (per hi / lo) for the scores of one tile
    constexpr int NT = D / 16;        // 16-dim column tiles of the output
    constexpr int NWV = 4;
    constexpr int VROW = D + 16;      // LDS row stride of a staged V tile, in bf16
    constexpr int RPB = 16 / G;       // rows per group
    constexpr int NCOL = RPB * G;     // MFMA columns in use
    static_assert(G >= 1 && G <= 8, "a group holds at least two rows");
    constexpr int V_BYTES = NWV * 2 * BS * VROW * 2;
    constexpr int QROW = D + 4;       // LDS row stride of q and of the waves' outputs, in floats: rows 4 banks apart
    constexpr int O_BYTES = NWV * 16 * QROW * 4;
    constexpr int RAW_BYTES = V_BYTES > O_BYTES ? V_BYTES : O_BYTES;

    __shared__ __attribute__((aligned(16))) float sm_q[16][QROW];   // prepared q of every column (unused: 0)
    // the staged V tiles during the main loop, the waves' outputs after it
    __shared__ __attribute__((aligned(16))) unsigned char sm_raw[RAW_BYTES];
    __shared__ float sm_ml[NWV][16][2];
    __shared__ int sm_ticket;
    typedef uint16_t (*VTiles)[2][BS][VROW];
    typedef float (*OTiles)[16][QROW];
    VTiles sm_v = reinterpret_cast<VTiles>(sm_raw);
    OTiles sm_o = reinterpret_cast<OTiles>(sm_raw);

    const int j = blockIdx.x, c = blockIdx.y, grp = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int dl = (lane % TPR) * 8;   // prologue layout: this lane's 8 dims
    const int sub = lane / TPR;        // prologue layout: head vector within the wave
    const int ln = lane & 15, lg = lane >> 4;   // MFMA layout
    const int q_stride = (a.nq + 2 * a.nkv) * D;
    const int *table = a.block_tables;           // one table for all rows
    const int row0 = grp * RPB;

    // ---- limits: column ln attends to positions < t1c ---------------------------
    const int row_c = row0 + ln / G;
    const bool valid_c = ln < NCOL && row_c < a.n_rows;
    int t1c = 0;
    if (valid_c) t1c = min(max(a.seq_lens[row_c], 0), a.max_blocks * BS - 1) + 1;
    int tmax = t1c;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) tmax = max(tmax, __shfl_xor(tmax, off));
    const int nact = (tmax + a.chunk_tokens - 1) / a.chunk_tokens;
    if (c >= nact) return;             // (also a group without rows: tmax = 0)
    const int t0 = c * a.chunk_tokens;
    const int t1 = min(tmax, t0 + a.chunk_tokens);
    const int blk_first = c * (a.chunk_tokens / BS) + 2 * wv;
    const int blk_end = (t1 + BS - 1) / BS;

    auto request = [&](int blk0, uint4 (&kw)[2][NS], uint4 (&vw)[2][NI]) {
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int phys = min(max(table[min(blk0 + u, a.max_blocks - 1)], 0), a.num_blocks - 1);
            const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
            const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
#pragma unroll
            for (int s = 0; s < NS; s++) kw[u][s] = ld16(kt + ln * D + s * 32 + lg * 8);
#pragma unroll
            for (int i = 0; i < NI; i++) vw[u][i] = ld16(vt + i * 512 + lane * 8);
        }
    };
    uint4 kw[2][NS], vw[2][NI];

    // ---- prologue: head norm, rotation and scale of q, one column per lane group --
    {
        const int col = wv * TPW + sub;
        const int rq = row0 + col / G;
        const bool valid_q = col < NCOL && rq < a.n_rows;
        const int rr = min(rq, a.n_rows - 1);
        const float *qp = a.qkv + (int64_t)rr * q_stride + (int64_t)(j * G + col % G) * D + dl;
        const float4 qa = ldf4(qp), qb = ldf4(qp + 4);
        float q[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
        const bool upper = dl >= D / 2;
        float2 cs[8];
        {
            const float4 *cp = reinterpret_cast<const float4 *>(a.cs + (int64_t)rr * (D / 2) +
                                                                (upper ? dl - D / 2 : dl));
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float4 t = cp[e];
                cs[2 * e] = make_float2(t.x, t.y);
                cs[2 * e + 1] = make_float2(t.z, t.w);
            }
        }
        const bool norm = a.g_q != nullptr;
        float gq[8];
        if (norm) {
            unpack8(ld16(a.g_q + dl), gq);
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) gq[e] = 1.f;
        }
        head_norm_rope<D>(q, norm, gq, a.eps, cs, upper);
        if (col < 16) {
#pragma unroll
            for (int e = 0; e < 8; e++) sm_q[col][dl + e] = valid_q ? q[e] * a.scale : 0.f;
        }
    }
    __syncthreads();

    uint4 qt[3][NS];   // q as the B operand
    mfma_q_operand<D>(sm_q[ln], true, lg, qt);

    // ---- main loop: a pair of block tiles (32 tokens) per iteration -----------
    MfmaAttnRun<D> run;
    run.init();
    for (int blk0 = blk_first; blk0 < blk_end; blk0 += 2 * NWV) {
        request(blk0, kw, vw);
        mfma_attend_tile_pair<D, VROW>(kw, vw, qt, sm_v[wv], blk0, t1, t1c, lane, run);
    }
    float l_run = run.l_run;
    const float m_run = run.m_run;
    const f32x4_t (&o)[NT] = run.o;

    // ---- per-wave state to LDS (over the V tiles: every wave is done with them) ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();
    if (lg == 0) { sm_ml[wv][ln][0] = m_run; sm_ml[wv][ln][1] = l_run; }
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
#pragma unroll
        for (int i = 0; i < 4; i++) sm_o[wv][4 * lg + i][nt * 16 + ln] = o[nt][i];
    __syncthreads();

    // ---- merge the waves; then the chunks ---------------------------------------
    constexpr int PSTRIDE = 16 * (D + 2);
    float *part = a.part + (((int64_t)grp * a.nkv + j) * a.max_chunks) * PSTRIDE;
    for (int idx = tid; idx < 16 * D; idx += 256) {
        const int col = idx / D, dim = idx % D;
        float mn = sm_ml[0][col][0];
#pragma unroll
        for (int w = 1; w < NWV; w++) mn = fmaxf(mn, sm_ml[w][col][0]);
        float ls = 0.f, os = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; w++) {
            const float scl = __expf(sm_ml[w][col][0] - mn);
            ls += sm_ml[w][col][1] * scl;
            os += sm_o[w][col][dim] * scl;
        }
        if (nact == 1) {
            const int r = row0 + col / G;
            if (col < NCOL && r < a.n_rows) store_attn_out(a, r, (j * G + col % G) * D + dim, a.nq * D, os / ls);
        } else {
            float *pp = part + (int64_t)c * PSTRIDE + col * (D + 2);
            st_coherent(pp + dim, os);
            if (dim == 0) { st_coherent(pp + D, mn); st_coherent(pp + D + 1, ls); }
        }
    }
    if (nact == 1) return;
    drain_stores();    // every thread's partials are complete ...
    __syncthreads();   // ... before one thread takes the ticket
    if (tid == 0)
        sm_ticket = __hip_atomic_fetch_add(&a.tickets[grp * a.nkv + j], 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sm_ticket != nact - 1) return;
    // eight columns at a time (the merge keeps eight chunks of every element in flight)
    constexpr int NE = (8 * D + 255) / 256;
#pragma unroll
    for (int half = 0; half < 2; half++) {
        float mv[NE];
        merge_chunk_partials<8, D, 16>(part + half * 8 * (D + 2), nact, tid, mv);
#pragma unroll
        for (int i = 0; i < NE; i++) {
            const int idx = tid + 256 * i;
            const int col = half * 8 + idx / D, dim = idx % D;
            const int r = row0 + col / G;
            if (idx < 8 * D && col < NCOL && r < a.n_rows)
                store_attn_out(a, r, (j * G + col % G) * D + dim, a.nq * D, mv[i]);
        }
    }
    if (tid == 0)
        __hip_atomic_store(&a.tickets[grp * a.nkv + j], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace dk
