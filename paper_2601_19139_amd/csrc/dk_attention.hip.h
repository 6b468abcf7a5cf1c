// Embedding gather, q/k head norm + rotary embedding + KV append, and ragged
// grouped-query decode attention over the block-table KV pool.
#pragma once
#include "dk_common.hip.h"

namespace dk {

// ---------------------------------------------------------------------------
// Step prologue: x[b][:] = float(E[tokens[b]][:]); the (cos, sin) table of the
// rotary embedding at position seq_lens[b]; attention tickets cleared.
struct EmbedArgs {
    const uint16_t *embed;  // [V][H]
    const int *tokens;      // [B]
    const int *seq_lens;    // [B]
    float *x;               // [B][H]
    float2 *cs;             // [B][d/2]
    int *tickets;           // [n_tickets]
    int n_tickets;
    int H, half, V;
    double inv_freq[64];    // theta^(-2i/d), i < d/2
};

__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a)
{
    const int b = blockIdx.x, tid = threadIdx.x;
    // an out-of-range token id is clamped (reads a valid row) rather than faulting
    const int tok = min(max(a.tokens[b], 0), a.V - 1);
    const uint16_t *row = a.embed + (int64_t)tok * a.H;
    for (int k = tid * 8; k < a.H; k += 256 * 8) {
        float f[8];
        unpack8(ld16(row + k), f);
        float *o = a.x + (int64_t)b * a.H + k;
        *reinterpret_cast<float4 *>(o) = make_float4(f[0], f[1], f[2], f[3]);
        *reinterpret_cast<float4 *>(o + 4) = make_float4(f[4], f[5], f[6], f[7]);
    }
    if (tid < a.half) {
        double ang = (double)a.seq_lens[b] * a.inv_freq[tid];
        double s, c;
        sincos(ang, &s, &c);
        a.cs[b * a.half + tid] = make_float2((float)c, (float)s);
    }
    if (b == 0)
        for (int i = tid; i < a.n_tickets; i += 256) a.tickets[i] = 0;
}

// ---------------------------------------------------------------------------
// Per head of the fused qkv vector: (q, k) optional RMSNorm over the head,
// half-split rotation by the step's angle; q is written back in place (f32),
// k and v are rounded to bf16 and stored at position seq_lens[b] of the
// sequence through its block table.  One wave per (row, head); lane i owns the
// rotation pair (i, i + d/2).
struct RopeAppendArgs {
    float *qkv;             // [B][(nq+2nkv)*d]
    const float2 *cs;       // [B][d/2]
    const uint16_t *g_q, *g_k;  // [d] or null
    uint16_t *pool;
    const int *block_tables;
    const int *seq_lens;
    int max_blocks, num_blocks, block_size;
    int layer, nq, nkv, d;
    float eps;
};

__global__ __launch_bounds__(64) void rope_append_kernel(RopeAppendArgs a)
{
    const int head = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int d = a.d, half = d >> 1;
    const bool act = lane < half;
    float *v = a.qkv + (int64_t)b * (a.nq + 2 * a.nkv) * d + (int64_t)head * d;
    float lo = act ? v[lane] : 0.f, hi = act ? v[lane + half] : 0.f;
    const bool is_q = head < a.nq, is_k = !is_q && head < a.nq + a.nkv;
    if (is_q || is_k) {
        const uint16_t *g = is_q ? a.g_q : a.g_k;
        if (g != nullptr) {
            float ss = sum64(lo * lo + hi * hi);
            float inv = rsqrtf(ss / (float)d + a.eps);
            if (act) {
                lo = lo * inv * bf16_to_f32(g[lane]);
                hi = hi * inv * bf16_to_f32(g[lane + half]);
            }
        }
        if (act) {
            float2 cs = a.cs[b * half + lane];
            float nlo = lo * cs.x - hi * cs.y;
            float nhi = hi * cs.x + lo * cs.y;
            lo = nlo;
            hi = nhi;
        }
    }
    if (!act) return;
    if (is_q) {
        v[lane] = lo;
        v[lane + half] = hi;
        return;
    }
    // positions / block ids outside the table or pool are clamped: the result
    // is then meaningless but no access leaves the caller's buffers
    const int pos = min(max(a.seq_lens[b], 0), a.max_blocks * a.block_size - 1);
    const int block = min(max(a.block_tables[(int64_t)b * a.max_blocks + pos / a.block_size], 0),
                          a.num_blocks - 1);
    const int slot = pos % a.block_size;
    const int kvh = is_k ? head - a.nq : head - a.nq - a.nkv;
    uint16_t *dst = a.pool + kv_tile_offset(a.layer, a.num_blocks, block, is_k ? 0 : 1, a.nkv, kvh,
                                            a.block_size, d) + (int64_t)slot * d;
    dst[lane] = f32_to_bf16_rne(lo);
    dst[lane + half] = f32_to_bf16_rne(hi);
}

// Stand-alone append of caller-provided bf16 K/V rows (bit for bit).
struct AppendArgs {
    const uint16_t *k, *v;  // [B][nkv][d]
    uint16_t *pool;
    const int *block_tables;
    const int *seq_lens;
    int max_blocks, num_blocks, block_size, layer, nkv, d;
};

__global__ __launch_bounds__(128) void append_kv_kernel(AppendArgs a)
{
    const int head = blockIdx.x, b = blockIdx.y, kv = blockIdx.z, i = threadIdx.x;
    if (i >= a.d) return;
    const int pos = min(max(a.seq_lens[b], 0), a.max_blocks * a.block_size - 1);
    const int block = min(max(a.block_tables[(int64_t)b * a.max_blocks + pos / a.block_size], 0),
                          a.num_blocks - 1);
    const int slot = pos % a.block_size;
    const uint16_t *src = (kv ? a.v : a.k) + ((int64_t)b * a.nkv + head) * a.d;
    uint16_t *dst = a.pool + kv_tile_offset(a.layer, a.num_blocks, block, kv, a.nkv, head,
                                            a.block_size, a.d) + (int64_t)slot * a.d;
    dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// Ragged grouped-query decode attention, split over the context.
//
// grid = (chunks, kv heads, rows); a block handles `chunk_tokens` consecutive
// positions of one sequence for one kv head and the G query heads that share
// it, so every K/V byte is read once for all G heads.  A wave reads a 16-token
// block tile (contiguous 16*d bf16) with 16-byte lane loads: D/8 lanes span a
// token, so one load covers 512/D tokens.  Each aligned group of D/8 lanes
// keeps its own running (max, sum, output) over the tokens it sees; the groups
// of a wave, the waves of a block and finally the chunks of a sequence are
// merged with the usual rescaling by exp(max differences).  The last block to
// finish for a (row, kv head) merges the chunk partials, in chunk order, so
// results do not depend on timing.
struct AttnArgs {
    const float *q;          // [B][(nq+2nkv)*d]: q heads first (already rotated)
    const uint16_t *pool;
    const int *block_tables;
    const int *seq_lens;
    float *out;              // [B][nq*d]
    float *part;             // [B][nkv][max_chunks][G][d+2]
    int *tickets;            // [B*nkv]
    int max_blocks, num_blocks, layer, nq, nkv;
    int chunk_tokens;        // multiple of 64
    int max_chunks;
    int q_stride;            // (nq+2nkv)*d
    float scale;
};

template <int D, int G>
__global__ __launch_bounds__(256) void attention_kernel(AttnArgs a)
{
    constexpr int BS = 16;            // tokens per block
    constexpr int TPR = D / 8;        // lanes per token
    constexpr int TPW = 64 / TPR;     // tokens per wave load
    constexpr int NI = BS / TPW;      // wave loads per block tile
    constexpr int NWV = 4;
    __shared__ float sm_o[NWV][G][D];
    __shared__ float sm_ml[NWV][G][2];
    __shared__ int sm_ticket;

    const int c = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // keys to attend to, incl. the new token (clamped to what the table can name)
    const int T1 = min(max(a.seq_lens[b], 0) + 1, a.max_blocks * BS);
    const int nact = (T1 + a.chunk_tokens - 1) / a.chunk_tokens;
    if (c >= nact) return;
    const int t0 = c * a.chunk_tokens;
    const int t1 = min(T1, t0 + a.chunk_tokens);
    const int dl = (lane % TPR) * 8;   // this lane's 8 dims
    const int sub = lane / TPR;        // token within a wave load

    float q[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const float *qp = a.q + (int64_t)b * a.q_stride + (int64_t)(j * G + g) * D + dl;
        float4 lo = ldf4(qp), hi = ldf4(qp + 4);
        q[g][0] = lo.x * a.scale; q[g][1] = lo.y * a.scale; q[g][2] = lo.z * a.scale; q[g][3] = lo.w * a.scale;
        q[g][4] = hi.x * a.scale; q[g][5] = hi.y * a.scale; q[g][6] = hi.z * a.scale; q[g][7] = hi.w * a.scale;
    }
    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -1e30f;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) o[g][e] = 0.f;
    }

    const int *table = a.block_tables + (int64_t)b * a.max_blocks;
    const int blk_end = (t1 + BS - 1) / BS;
    for (int blk = t0 / BS + wv; blk < blk_end; blk += NWV) {
        const int phys = min(max(table[blk], 0), a.num_blocks - 1);
        const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
        const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
        uint4 kw[NI], vw[NI];
#pragma unroll
        for (int i = 0; i < NI; i++) {
            kw[i] = ld16(kt + i * 512 + lane * 8);
            vw[i] = ld16(vt + i * 512 + lane * 8);
        }
        float s[NI][G];
        bool valid[NI];
#pragma unroll
        for (int i = 0; i < NI; i++) {
            valid[i] = (blk * BS + i * TPW + sub) < t1;
            float kf[8];
            unpack8(kw[i], kf);
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
            l[g] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; e++) o[g][e] *= alpha;
        }
#pragma unroll
        for (int i = 0; i < NI; i++) {
            float vf[8];
            unpack8(vw[i], vf);
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float p = valid[i] ? __expf(s[i][g] - m[g]) : 0.f;
                l[g] += p;
#pragma unroll
                for (int e = 0; e < 8; e++) o[g][e] += valid[i] ? p * vf[e] : 0.f;
            }
        }
    }

    // merge the token groups of the wave (lanes differing in bits >= log2(TPR))
#pragma unroll
    for (int off = TPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            const float om = __shfl_xor(m[g], off), ol = __shfl_xor(l[g], off);
            const float mn = fmaxf(m[g], om);
            const float sa = __expf(m[g] - mn), sb = __expf(om - mn);
            l[g] = l[g] * sa + ol * sb;
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
            if (lane == 0) { sm_ml[wv][g][0] = m[g]; sm_ml[wv][g][1] = l[g]; }
        }
    }
    __syncthreads();

    // merge the waves; thread (g, dim) for g*D + dim = tid, tid + 256, ...
    float *part = a.part + (((int64_t)b * a.nkv + j) * a.max_chunks) * (G * (D + 2));
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, dim = idx % D;
        float mn = sm_ml[0][g][0];
#pragma unroll
        for (int w = 1; w < NWV; w++) mn = fmaxf(mn, sm_ml[w][g][0]);
        float ls = 0.f, os = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; w++) {
            const float sc = __expf(sm_ml[w][g][0] - mn);
            ls += sm_ml[w][g][1] * sc;
            os += sm_o[w][g][dim] * sc;
        }
        if (nact == 1) {
            a.out[(int64_t)b * a.nq * D + (int64_t)(j * G + g) * D + dim] = os / ls;
        } else {
            float *pp = part + (int64_t)c * (G * (D + 2)) + g * (D + 2);
            pp[dim] = os;
            if (dim == 0) { pp[D] = mn; pp[D + 1] = ls; }
        }
    }
    if (nact == 1) return;

    // last block of this (row, kv head) merges the chunk partials
    __threadfence();
    __syncthreads();
    if (tid == 0) sm_ticket = atomicAdd(&a.tickets[b * a.nkv + j], 1);
    __syncthreads();
    if (sm_ticket != nact - 1) return;
    __threadfence();
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, dim = idx % D;
        float mn = -1e30f;
        for (int cc = 0; cc < nact; cc++)
            mn = fmaxf(mn, part[(int64_t)cc * (G * (D + 2)) + g * (D + 2) + D]);
        float ls = 0.f, os = 0.f;
        for (int cc = 0; cc < nact; cc++) {
            const float *pp = part + (int64_t)cc * (G * (D + 2)) + g * (D + 2);
            const float sc = __expf(pp[D] - mn);
            ls += pp[D + 1] * sc;
            os += pp[dim] * sc;
        }
        a.out[(int64_t)b * a.nq * D + (int64_t)(j * G + g) * D + dim] = os / ls;
    }
    if (tid == 0) a.tickets[b * a.nkv + j] = 0;
}

}  // namespace dk
