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
//           = token row, 16-byte loads) and B = q as bf16 hi + lo (two MFMAs per
//           32 dims, so q keeps ~16 significant bits); the G query heads of the
//           group are the first G of the 16 columns.
//   softmax online per column: the lane (column g, lane group lg) holds tokens
//           4*lg..4*lg+3 of each tile; running max / sum as usual.
//   output  O[g][dim] += sum_token P[g][token] * V[token][dim]
//           MFMAs with A = P as bf16 hi + lo - the lane's 8 probabilities are
//           already the 8 k-values the A operand wants, in the token order
//           (tile0: 4lg..4lg+3, tile1: 4lg..4lg+3) - and B = V with tokens along
//           k, i.e. V transposed: the wave stages its two V tiles in LDS (rows
//           of masked-out tokens zeroed) and gathers the B operand from there.
#pragma once
#include "dk_attention.hip.h"
#include "dk_gemm.hip.h"

namespace dk {

template <int D, int G>
__global__ __launch_bounds__(256) void attention_mfma_kernel(AttnArgs a)
{
    constexpr int BS = 16;            // tokens per block tile
    constexpr int TPR = D / 8;        // lanes per token in the row-major tile loads
    constexpr int TPW = 64 / TPR;     // tokens per wave load
    constexpr int NI = BS / TPW;      // wave loads per tile
    constexpr int NS = D / 32;        // MFMAs (per hi / lo) for the scores of one tile
    constexpr int NT = D / 16;        // 16-dim column tiles of the output
    constexpr int NWV = 4;
    constexpr int VROW = D + 4;       // LDS row stride of a staged V tile, in bf16 (8 bytes of padding)
    static_assert(G <= 8, "the query group occupies the first G of 16 MFMA columns");

    __shared__ float sm_q[G][D];                       // prepared q (norm, rotation, scale)
    __shared__ uint16_t sm_v[NWV][2][BS][VROW];        // per wave: two V tiles
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
    const int *table = a.block_tables + (int64_t)b * a.max_blocks;

    // ---- prologue (row-major head layout, as in attention_kernel) ------------
    float q[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const float *qp = row + (int64_t)(j * G + g) * D + dl;
        const float4 lo = ldf4(qp), hi = ldf4(qp + 4);
        q[g][0] = lo.x; q[g][1] = lo.y; q[g][2] = lo.z; q[g][3] = lo.w;
        q[g][4] = hi.x; q[g][5] = hi.y; q[g][6] = hi.z; q[g][7] = hi.w;
    }
    const bool upper = dl >= D / 2;
    float2 cs[8];
    {
        const float4 *cp = reinterpret_cast<const float4 *>(cs_row + (upper ? dl - D / 2 : dl));
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const float4 t = cp[e];
            cs[2 * e] = make_float2(t.x, t.y);
            cs[2 * e + 1] = make_float2(t.z, t.w);
        }
    }
    const bool norm = a.g_q != nullptr;
    float gq[8], gk[8];
    if (norm) {
        unpack8(ld16(a.g_q + dl), gq);
        unpack8(ld16(a.g_k + dl), gk);
    } else {
#pragma unroll
        for (int e = 0; e < 8; e++) gq[e] = gk[e] = 1.f;
    }
    float kn[8], vn[8];
    {
        const float *kp = row + (int64_t)(a.nq + j) * D + dl;
        const float *vp = row + (int64_t)(a.nq + a.nkv + j) * D + dl;
        const float4 klo = ldf4(kp), khi = ldf4(kp + 4), vlo = ldf4(vp), vhi = ldf4(vp + 4);
        kn[0] = klo.x; kn[1] = klo.y; kn[2] = klo.z; kn[3] = klo.w;
        kn[4] = khi.x; kn[5] = khi.y; kn[6] = khi.z; kn[7] = khi.w;
        vn[0] = vlo.x; vn[1] = vlo.y; vn[2] = vlo.z; vn[3] = vlo.w;
        vn[4] = vhi.x; vn[5] = vhi.y; vn[6] = vhi.z; vn[7] = vhi.w;
    }
    const int T = min(max(a.seq_lens[b], 0), a.max_blocks * BS - 1);
    const int nact = (T + 1 + a.chunk_tokens - 1) / a.chunk_tokens;
    if (c >= nact) return;
    const int t0 = c * a.chunk_tokens;
    const int t1 = min(T, t0 + a.chunk_tokens);   // cached positions [t0, t1) come from the pool
    const bool owns_new = (c == nact - 1);        // position T itself

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
            if (sub == 0) {
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
    __syncthreads();

    // q as the B operand: lane (column g = ln, lane group lg) holds dims
    // s*32 + lg*8 .. +8 of head g, as bf16 hi and lo; columns >= G are zero
    uint4 qh[NS], ql[NS];
#pragma unroll
    for (int s = 0; s < NS; s++) {
        uint32_t hw[4], lw[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const float v0 = ln < G ? sm_q[min(ln, G - 1)][s * 32 + lg * 8 + 2 * e] : 0.f;
            const float v1 = ln < G ? sm_q[min(ln, G - 1)][s * 32 + lg * 8 + 2 * e + 1] : 0.f;
            uint16_t h0, l0, h1, l1;
            split_bf16(v0, h0, l0);
            split_bf16(v1, h1, l1);
            hw[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            lw[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
        }
        qh[s] = make_uint4(hw[0], hw[1], hw[2], hw[3]);
        ql[s] = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    }

    // ---- main loop: a pair of block tiles (32 tokens) per iteration -----------
    float m_run = -1e30f, l_run = 0.f;     // column ln, over this lane group's tokens
    f32x4_t o[NT];                          // O[head 4*lg + i][dim 16*nt + ln]
#pragma unroll
    for (int nt = 0; nt < NT; nt++) o[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int blk_end = (t1 + BS - 1) / BS;
    for (int blk0 = t0 / BS + 2 * wv; blk0 < blk_end; blk0 += 2 * NWV) {
        uint4 kw[2][NS], vw[2][NI];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int blk = min(blk0 + u, a.max_blocks - 1);
            const int phys = min(max(table[blk], 0), a.num_blocks - 1);
            const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
            const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
#pragma unroll
            for (int s = 0; s < NS; s++) kw[u][s] = ld16(kt + ln * D + s * 32 + lg * 8);
#pragma unroll
            for (int i = 0; i < NI; i++) vw[u][i] = ld16(vt + i * 512 + lane * 8);
        }
        // scores
        f32x4_t sc[2];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            sc[u] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; s++) {
                sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kw[u][s]), as_bf16x8(qh[s]), sc[u], 0, 0, 0);
                sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kw[u][s]), as_bf16x8(ql[s]), sc[u], 0, 0, 0);
            }
        }
        // stage V (rows of positions >= t1 zeroed) while the scores are computed
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int i = 0; i < NI; i++) {
                const int r = i * TPW + sub;
                const bool ok = (blk0 + u) * BS + r < t1;
                const uint4 w = ok ? vw[u][i] : make_uint4(0, 0, 0, 0);
                uint2 *dst = reinterpret_cast<uint2 *>(&sm_v[wv][u][r][dl]);
                dst[0] = make_uint2(w.x, w.y);
                dst[1] = make_uint2(w.z, w.w);
            }
        // online softmax of column ln over the 8 tokens of this lane
        float p[2][4];
        float mx = m_run;
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const bool ok = (blk0 + u) * BS + 4 * lg + i < t1;
                p[u][i] = ok ? sc[u][i] : -1e30f;
                mx = fmaxf(mx, p[u][i]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));      // the column's max over all 32 tokens and the past
        const float alpha = __expf(m_run - mx);
        m_run = mx;
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const bool ok = (blk0 + u) * BS + 4 * lg + i < t1;
                p[u][i] = ok ? __expf(p[u][i] - mx) : 0.f;
                psum += p[u][i];
            }
        l_run = l_run * alpha + psum;
        // P as the A operand (bf16 hi / lo): k-slot e <-> (tile e/4, token 4*lg + e%4)
        uint4 ph, pl;
        {
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                uint16_t h0, l0, h1, l1;
                split_bf16(p[e / 2][(2 * e) % 4], h0, l0);
                split_bf16(p[e / 2][(2 * e) % 4 + 1], h1, l1);
                hw[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                lw[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            ph = make_uint4(hw[0], hw[1], hw[2], hw[3]);
            pl = make_uint4(lw[0], lw[1], lw[2], lw[3]);
        }
        // rescale the running output: row i of this lane is head 4*lg + i, whose
        // alpha lives in the lanes of column 4*lg + i
        float al[4];
#pragma unroll
        for (int i = 0; i < 4; i++) al[i] = __shfl(alpha, 4 * lg + i);
#pragma unroll
        for (int nt = 0; nt < NT; nt++)
#pragma unroll
            for (int i = 0; i < 4; i++) o[nt][i] *= al[i];
        // O += P V : B operand gathered from the staged tiles (V transposed)
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            uint32_t vwd[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int u = e / 2, r = 4 * lg + (2 * e) % 4;
                const uint32_t v0 = sm_v[wv][u][r][nt * 16 + ln];
                const uint32_t v1 = sm_v[wv][u][r + 1][nt * 16 + ln];
                vwd[e] = v0 | (v1 << 16);
            }
            const uint4 vb = make_uint4(vwd[0], vwd[1], vwd[2], vwd[3]);
            o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ph), as_bf16x8(vb), o[nt], 0, 0, 0);
            o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(pl), as_bf16x8(vb), o[nt], 0, 0, 0);
        }
    }

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
    __syncthreads();
    if (tid == 0)
        sm_ticket = __hip_atomic_fetch_add(&a.tickets[b * a.nkv + j], 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sm_ticket != nact - 1) return;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, dim = idx % D;
        const float *pg = part + g * (D + 2);
        float mn = -1e30f, ls = 0.f, os = 0.f;
        for (int cc = 0; cc < nact; cc++) {
            const float *pp = pg + (int64_t)cc * (G * (D + 2));
            const float mc = ld_coherent(pp + D), lc = ld_coherent(pp + D + 1), oc = ld_coherent(pp + dim);
            const float m2 = fmaxf(mn, mc);
            const float sa = __expf(mn - m2), sb = __expf(mc - m2);
            ls = ls * sa + lc * sb;
            os = os * sa + oc * sb;
            mn = m2;
        }
        store_attn_out(a, b, (j * G + g) * D + dim, a.nq * D, os / ls);
    }
    if (tid == 0)
        __hip_atomic_store(&a.tickets[b * a.nkv + j], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace dk
