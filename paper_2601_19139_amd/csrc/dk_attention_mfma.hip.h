// Ragged grouped-query decode attention on the matrix cores, for the batched
// path (many rows and/or long contexts), where the vector-ALU kernel would be
// bound by its multiply-adds rather than by the KV stream.
//
// Same contract, grid and prologue as attention_kernel (head norm + rotation of
// q, KV append of the new token by the block that owns its position, chunks
// merged by the last block of a (row, kv head)); only the inner loop differs.
// A wave takes two 16-token block tiles at a time:
//
//   scores  S[token][g] = sum_dim K[token][dim] * q[g][dim]
//           16x16x32 bf16 MFMAs with A = the K tile straight from the pool (lane
//           = token row, 16-byte loads) and B = q as three bf16 terms (three MFMAs
//           per 32 dims, so q keeps 24 significant bits: an error in a score is an
//           equal relative error in its probability); the G query heads of the
//           group are the first G of the 16 columns.
//   softmax online per column: the lane (column g, lane group lg) holds tokens
//           4*lg..4*lg+3 of each tile; running max / sum as usual.
//   output  O[g][dim] += sum_token P[g][token] * V[token][dim]
//           MFMAs with A = P as bf16 hi + lo - the lane's 8 probabilities are
//           already the 8 k-values the A operand wants, in the token order
//           (tile0: 4lg..4lg+3, tile1: 4lg..4lg+3) - and B = V with tokens along
//           k, i.e. V transposed: the wave stages its two V tiles in LDS (rows
//           of masked-out tokens zeroed) and fetches the B operand from there
//           with the LDS transpose read (ds_read_b64_tr_b16).
#pragma once
#include "dk_attention.hip.h"
#include "dk_gemm.hip.h"

namespace dk {

// One iteration of the matrix-core inner loop, shared by the decode kernel below and the
// chunked-prefill kernel (dk_attention_prefill.hip.h): a wave's pair of 16-token block tiles
// starting at block blk0, already in registers (kw: K tiles as the A operand, vw: V tiles row
// major), against the 16 query columns in qt.  Column ln attends to positions < t1_col;
// V rows of positions >= t1_stage (>= every column's limit) are zeroed while staged, since
// they may hold anything.  Running maximum, sum and output of the wave are updated in place.
// q as the B operand of the score MFMAs: lane (column ln, lane group lg) holds dims s*32 + lg*8 .. +8
// of its column, as THREE bf16 terms whose sum has 24 significant bits.  K is exact bf16, so the
// scores then carry float32 accuracy; with two terms (16 bits) a score of magnitude 30 was off by
// 2e-4 absolute, which a row with a handful of cached tokens shows undiminished in its output.
template <int D>
__device__ __forceinline__ void mfma_q_operand(const float *qrow, bool valid, int lg, uint4 (&qt)[3][D / 32])
{
#pragma unroll
    for (int s = 0; s < D / 32; s++) {
        const float4 *src = reinterpret_cast<const float4 *>(qrow + s * 32 + lg * 8);
        const float4 f0 = src[0], f1 = src[1];
        const float f[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
        uint32_t w[3][4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const float a = valid ? f[2 * e] : 0.f, b = valid ? f[2 * e + 1] : 0.f;
            w[0][e] = f32x2_to_bf16x2_rne(a, b);
            const float ra = a - bf16lo(w[0][e]), rb = b - bf16hi(w[0][e]);
            w[1][e] = f32x2_to_bf16x2_rne(ra, rb);
            w[2][e] = f32x2_to_bf16x2_rne(ra - bf16lo(w[1][e]), rb - bf16hi(w[1][e]));
        }
#pragma unroll
        for (int t = 0; t < 3; t++) qt[t][s] = make_uint4(w[t][0], w[t][1], w[t][2], w[t][3]);
    }
}

template <int D>
struct MfmaAttnRun {
    float m_run, l_run;          // column ln, over this lane group's tokens
    f32x4_t o[D / 16];           // O[column 4*lg + i][dim 16*nt + ln]
    __device__ __forceinline__ void init()
    {
        m_run = -1e30f;
        l_run = 0.f;
#pragma unroll
        for (int nt = 0; nt < D / 16; nt++) o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
};

template <int D, int VROW>
__device__ __forceinline__ void mfma_attend_tile_pair(const uint4 (&kw)[2][D / 32], const uint4 (&vw)[2][16 / (512 / D)],
                                                      const uint4 (&qt)[3][D / 32],
                                                      uint16_t (*sm_vw)[16][VROW], int blk0, int t1_stage,
                                                      int t1_col, int lane, MfmaAttnRun<D> &r)
{
    constexpr int BS = 16, TPR = D / 8, TPW = 64 / TPR, NI = BS / TPW, NS = D / 32, NT = D / 16;
    const int dl = (lane % TPR) * 8, sub = lane / TPR;
    const int ln = lane & 15, lg = lane >> 4;
    // scores
    f32x4_t sc[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
        sc[u] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; s++) {
#pragma unroll
            for (int t = 0; t < 3; t++)
                sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kw[u][s]), as_bf16x8(qt[t][s]), sc[u], 0, 0, 0);
        }
    }
    // stage V while the scores are computed
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < NI; i++) {
            const int row = i * TPW + sub;
            const bool ok = (blk0 + u) * BS + row < t1_stage;
            const uint4 w = ok ? vw[u][i] : make_uint4(0, 0, 0, 0);
            uint2 *dst = reinterpret_cast<uint2 *>(&sm_vw[u][row][dl]);
            dst[0] = make_uint2(w.x, w.y);
            dst[1] = make_uint2(w.z, w.w);
        }
    // online softmax of column ln over the 8 tokens of this lane
    float p[2][4];
    float mx = r.m_run;
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const bool ok = (blk0 + u) * BS + 4 * lg + i < t1_col;
            p[u][i] = ok ? sc[u][i] : -1e30f;
            mx = fmaxf(mx, p[u][i]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));      // the column's max over all 32 tokens and the past
    const float alpha = __expf(r.m_run - mx);
    r.m_run = mx;
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const bool ok = (blk0 + u) * BS + 4 * lg + i < t1_col;
            p[u][i] = ok ? __expf(p[u][i] - mx) : 0.f;
            psum += p[u][i];
        }
    r.l_run = r.l_run * alpha + psum;
    // P as the A operand (bf16 hi / lo): k-slot e <-> (tile e/4, token 4*lg + e%4)
    uint4 ph, pl;
    {
        uint32_t hw[4], lw[4];
#pragma unroll
        for (int e = 0; e < 4; e++) split_bf16x2(p[e / 2][(2 * e) % 4], p[e / 2][(2 * e) % 4 + 1], hw[e], lw[e]);
        ph = make_uint4(hw[0], hw[1], hw[2], hw[3]);
        pl = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    }
    // rescale the running output: row i of this lane is column 4*lg + i, whose alpha lives in
    // the lanes of that column.  Once the running maxima have settled every alpha is exactly 1
    // and the pass is skipped.
    if (__any(alpha != 1.f)) {
        float al[4];
#pragma unroll
        for (int i = 0; i < 4; i++) al[i] = __shfl(alpha, 4 * lg + i);
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
#pragma unroll
            for (int i = 0; i < 4; i++) r.o[nt][i] *= al[i];
    }
    // O += P V : the B operand is V with tokens along k.  The LDS transpose read hands lane
    // (column ln, lane group lg) the four tokens 4*lg..4*lg+3 of column nt*16 + ln when lane i
    // of the group points at the 4 consecutive dims nt*16 + 4*(i%4) of token 4*lg + i/4 (layout
    // checked on the device: lane 4g+c, element e <- address of lane 4e+g, element c).
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        uint32_t vwd[4];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            typedef short v4s __attribute__((ext_vector_type(4)));
            const uint16_t *src = &sm_vw[u][4 * lg + (ln >> 2)][nt * 16 + 4 * (ln & 3)];
            const v4s rr = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4s *)(src));
            __builtin_memcpy(&vwd[2 * u], &rr, 8);   // elements 0, 1 | 2, 3 as two words
        }
        const uint4 vb = make_uint4(vwd[0], vwd[1], vwd[2], vwd[3]);
        r.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ph), as_bf16x8(vb), r.o[nt], 0, 0, 0);
        r.o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(pl), as_bf16x8(vb), r.o[nt], 0, 0, 0);
    }
}

template <int D, int G, bool PREFETCH>
__global__ __launch_bounds__(256, PREFETCH ? 2 : 3) void attention_mfma_kernel(AttnArgs a)
{
    constexpr int BS = 16;            // tokens per block tile
    constexpr int TPR = D / 8;        // lanes per token in the row-major tile loads
    constexpr int TPW = 64 / TPR;     // tokens per wave load
    constexpr int NI = BS / TPW;      // wave loads per tile
    constexpr int NS = D / 32;        // MFMAs (per hi / lo) for the scores of one tile
    constexpr int NT = D / 16;        // 16-dim column tiles of the output
    constexpr int NWV = 4;
    constexpr int VROW = D + 16;      // LDS row stride of a staged V tile, in bf16: 4 consecutive rows start 8 banks apart
    static_assert(G <= 8, "the query group occupies the first G of 16 MFMA columns");

    __shared__ __attribute__((aligned(16))) float sm_q[G][D];   // prepared q (norm, rotation, scale)
    __shared__ __attribute__((aligned(16))) uint16_t sm_v[NWV][2][BS][VROW];   // per wave: two V tiles
    __shared__ float sm_o[NWV + 1][G][D];              // per wave + the new token
    __shared__ float sm_ml[NWV + 1][G][2];
    __shared__ int sm_ticket;

    const int c = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int dl = (lane % TPR) * 8;   // row-major layout: this lane's 8 dims
    const int sub = lane / TPR;        // row-major layout: token within a wave load
    const int ln = lane & 15, lg = lane >> 4;   // MFMA layout
    const int q_stride = (a.nq + 2 * a.nkv) * D;
    const float *row = a.qkv + (int64_t)b * q_stride;
    const float2 *cs_row = a.cs + (int64_t)b * (D / 2);
    const int *table = a.block_tables + (int64_t)b * a.table_stride;

    // ---- requests first, arithmetic later -------------------------------------
    // The q | k | v row, the rotation table and the gains do not depend on the
    // sequence state: they are requested before anything else so that they are
    // back while the first K/V tiles (requested right after, once the block table
    // has been read) are still on their way.  Loads return in order, so the other
    // way round the prologue would wait for the K/V tiles.
    float4 q_raw[G][2], k_raw[2], v_raw[2], cs_raw[4];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const float *qp = row + (int64_t)(j * G + g) * D + dl;
        q_raw[g][0] = ldf4(qp);
        q_raw[g][1] = ldf4(qp + 4);
    }
    const bool upper = dl >= D / 2;
    {
        const float4 *cp = reinterpret_cast<const float4 *>(cs_row + (upper ? dl - D / 2 : dl));
#pragma unroll
        for (int e = 0; e < 4; e++) cs_raw[e] = cp[e];
    }
    const bool norm = a.g_q != nullptr;
    uint4 gq_raw = make_uint4(0, 0, 0, 0), gk_raw = make_uint4(0, 0, 0, 0);
    if (norm) {
        gq_raw = ld16(a.g_q + dl);
        gk_raw = ld16(a.g_k + dl);
    }
    {
        const float *kp = row + (int64_t)(a.nq + j) * D + dl;
        const float *vp = row + (int64_t)(a.nq + a.nkv + j) * D + dl;
        k_raw[0] = ldf4(kp); k_raw[1] = ldf4(kp + 4);
        v_raw[0] = ldf4(vp); v_raw[1] = ldf4(vp + 4);
    }
    // block-table entries of the wave's first tile pair: they depend on the chunk
    // index only, so they are read together with the sequence length
    const int blk_first = c * (a.chunk_tokens / BS) + 2 * wv;
    const int phys_a = table[min(blk_first, a.max_blocks - 1)];
    const int phys_b = table[min(blk_first + 1, a.max_blocks - 1)];
    const int T = min(max(a.seq_lens[b], 0), a.max_blocks * BS - 1);
    const int nact = (T + 1 + a.chunk_tokens - 1) / a.chunk_tokens;
    if (c >= nact) return;
    const int t0 = c * a.chunk_tokens;
    const int t1 = min(T, t0 + a.chunk_tokens);   // cached positions [t0, t1) come from the pool
    const bool owns_new = (c == nact - 1);        // position T itself
    const int blk_end = (t1 + BS - 1) / BS;
    // The K and V tiles of the next iteration are requested before this one is
    // computed (the last iteration re-requests its own tiles: a cache hit, and
    // every request is unconditional so the loads stay counted in order).
    auto request_phys = [&](int pa, int pb, uint4 (&kw)[2][NS], uint4 (&vw)[2][NI]) {
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int phys = min(max(u ? pb : pa, 0), a.num_blocks - 1);
            const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
            const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
#pragma unroll
            for (int s = 0; s < NS; s++) kw[u][s] = ld16(kt + ln * D + s * 32 + lg * 8);
#pragma unroll
            for (int i = 0; i < NI; i++) vw[u][i] = ld16(vt + i * 512 + lane * 8);
        }
    };
    auto request = [&](int blk0, uint4 (&kw)[2][NS], uint4 (&vw)[2][NI]) {
        request_phys(table[min(blk0, a.max_blocks - 1)], table[min(blk0 + 1, a.max_blocks - 1)], kw, vw);
    };
    uint4 kw[2][NS], vw[2][NI];
    request_phys(phys_a, phys_b, kw, vw);

    // ---- prologue (row-major head layout, as in attention_kernel) ------------
    float q[G][8], kn[8], vn[8], gq[8], gk[8];
    float2 cs[8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        q[g][0] = q_raw[g][0].x; q[g][1] = q_raw[g][0].y; q[g][2] = q_raw[g][0].z; q[g][3] = q_raw[g][0].w;
        q[g][4] = q_raw[g][1].x; q[g][5] = q_raw[g][1].y; q[g][6] = q_raw[g][1].z; q[g][7] = q_raw[g][1].w;
    }
#pragma unroll
    for (int e = 0; e < 4; e++) {
        cs[2 * e] = make_float2(cs_raw[e].x, cs_raw[e].y);
        cs[2 * e + 1] = make_float2(cs_raw[e].z, cs_raw[e].w);
    }
    if (norm) {
        unpack8(gq_raw, gq);
        unpack8(gk_raw, gk);
    } else {
#pragma unroll
        for (int e = 0; e < 8; e++) gq[e] = gk[e] = 1.f;
    }
    kn[0] = k_raw[0].x; kn[1] = k_raw[0].y; kn[2] = k_raw[0].z; kn[3] = k_raw[0].w;
    kn[4] = k_raw[1].x; kn[5] = k_raw[1].y; kn[6] = k_raw[1].z; kn[7] = k_raw[1].w;
    vn[0] = v_raw[0].x; vn[1] = v_raw[0].y; vn[2] = v_raw[0].z; vn[3] = v_raw[0].w;
    vn[4] = v_raw[1].x; vn[5] = v_raw[1].y; vn[6] = v_raw[1].z; vn[7] = v_raw[1].w;

#pragma unroll
    for (int g = 0; g < G; g++) {
        head_norm_rope<D>(q[g], norm, gq, a.eps, cs, upper);
#pragma unroll
        for (int e = 0; e < 8; e++) q[g][e] *= a.scale;
    }
    if (wv == 0 && sub == 0) {
#pragma unroll
        for (int g = 0; g < G; g++)
#pragma unroll
            for (int e = 0; e < 8; e++) sm_q[g][dl + e] = q[g][e];
    }
    __syncthreads();
    // (after the barrier, so that the other waves do not wait for it: wave 0's own
    // first tiles are still on their way at this point)
    if (wv == 0) {
        if (owns_new) {
            // the new token: stored (bf16) at position T and kept as one more
            // partial (score, 1, v) that the final merge adds
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
            if (sub == 0 && !a.no_append) {
                const int phys = min(max(table[T / BS], 0), a.num_blocks - 1);
                uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D) +
                               (T % BS) * D + dl;
                uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
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
#pragma unroll
                    for (int e = 0; e < 8; e++) sm_o[NWV][g][dl + e] = vn[e];
                    if (lane == 0) { sm_ml[NWV][g][0] = p; sm_ml[NWV][g][1] = 1.f; }
                }
            }
        } else if (sub == 0) {
#pragma unroll
            for (int g = 0; g < G; g++) {
#pragma unroll
                for (int e = 0; e < 8; e++) sm_o[NWV][g][dl + e] = 0.f;
                if (lane == 0) { sm_ml[NWV][g][0] = -1e30f; sm_ml[NWV][g][1] = 0.f; }
            }
        }
    }

    // q as the B operand (columns >= G are zero)
    uint4 qt[3][NS];
    mfma_q_operand<D>(sm_q[min(ln, G - 1)], ln < G, lg, qt);

    // ---- main loop: a pair of block tiles (32 tokens) per iteration -----------
    MfmaAttnRun<D> run;
    run.init();
    if constexpr (PREFETCH) {
        // long chunks: the next tile pair is requested before this one is used (two blocks per
        // compute unit; the stream is what matters)
        uint4 kw_n[2][NS], vw_n[2][NI];
        for (int blk0 = blk_first; blk0 < blk_end; blk0 += 2 * NWV) {
            const int blk_next = blk0 + 2 * NWV;
            request(blk_next < blk_end ? blk_next : blk0, kw_n, vw_n);
            mfma_attend_tile_pair<D, VROW>(kw, vw, qt, sm_v[wv], blk0, t1, t1, lane, run);
#pragma unroll
            for (int u = 0; u < 2; u++) {
#pragma unroll
                for (int s = 0; s < NS; s++) kw[u][s] = kw_n[u][s];
#pragma unroll
                for (int i = 0; i < NI; i++) vw[u][i] = vw_n[u][i];
            }
        }
    } else {
        // short chunks (a few iterations per wave): no second set of tile registers, three
        // blocks per compute unit cover the latency instead
        for (int blk0 = blk_first; blk0 < blk_end; blk0 += 2 * NWV) {
            if (blk0 != blk_first) request(blk0, kw, vw);
            mfma_attend_tile_pair<D, VROW>(kw, vw, qt, sm_v[wv], blk0, t1, t1, lane, run);
        }
    }
    float l_run = run.l_run;
    const float m_run = run.m_run;
    const f32x4_t (&o)[NT] = run.o;

    // ---- per-wave state to LDS -------------------------------------------------
    // the column sum is spread over the four lane groups
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (lg == 0 && ln < G) { sm_ml[wv][ln][0] = m_run; sm_ml[wv][ln][1] = l_run; }
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
#pragma unroll
        for (int i = 0; i < 4; i++)
            if (4 * lg + i < G) sm_o[wv][4 * lg + i][nt * 16 + ln] = o[nt][i];
    __syncthreads();

    // ---- merge the waves and the new token; chunks as in attention_kernel ------
    float *part = a.part + (((int64_t)b * a.nkv + j) * a.max_chunks) * (G * (D + 2));
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, dim = idx % D;
        float mn = sm_ml[0][g][0];
#pragma unroll
        for (int w = 1; w <= NWV; w++) mn = fmaxf(mn, sm_ml[w][g][0]);
        float ls = 0.f, os = 0.f;
#pragma unroll
        for (int w = 0; w <= NWV; w++) {
            const float scl = __expf(sm_ml[w][g][0] - mn);
            ls += sm_ml[w][g][1] * scl;
            os += sm_o[w][g][dim] * scl;
        }
        float *pp = part + (int64_t)c * (G * (D + 2)) + g * (D + 2);
        if (nact == 1) {
            store_attn_out(a, b, (j * G + g) * D + dim, a.nq * D, os / ls);
        } else {
            st_coherent(pp + dim, os);
            if (dim == 0) { st_coherent(pp + D, mn); st_coherent(pp + D + 1, ls); }
        }
    }
    if (nact == 1) return;
    drain_stores();   // the partials are complete before the ticket is taken (see attention_kernel)
    __syncthreads();
    if (tid == 0)
        sm_ticket = __hip_atomic_fetch_add(&a.tickets[b * a.nkv + j], 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sm_ticket != nact - 1) return;
    float mv[(G * D + 255) / 256];
    merge_chunk_partials<G, D>(part, nact, tid, mv);
#pragma unroll
    for (int i = 0; i < (G * D + 255) / 256; i++) {
        const int idx = tid + 256 * i;
        if (idx < G * D) store_attn_out(a, b, j * G * D + idx, a.nq * D, mv[i]);
    }
    if (tid == 0)
        __hip_atomic_store(&a.tickets[b * a.nkv + j], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace dk
