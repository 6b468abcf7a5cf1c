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
    // batched path (null otherwise): (x * gain) as bf16 hi/lo in act_offset() order and the
    // row's sum of x^2 in ssq_out[b], for the first matrix-core GEMM
    const uint16_t *gain;
    uint16_t *xhi, *xlo;
    float *ssq_out;
    double inv_freq[64];    // theta^(-2i/d), i < d/2
};

__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a)
{
    const int b = blockIdx.x, tid = threadIdx.x;
    // an out-of-range token id is clamped (reads a valid row) rather than faulting
    const int tok = min(max(a.tokens[b], 0), a.V - 1);
    const uint16_t *row = a.embed + (int64_t)tok * a.H;
    float ss = 0.f;
    for (int k = tid * 8; k < a.H; k += 256 * 8) {
        float f[8];
        unpack8(ld16(row + k), f);
        float *o = a.x + (int64_t)b * a.H + k;
        *reinterpret_cast<float4 *>(o) = make_float4(f[0], f[1], f[2], f[3]);
        *reinterpret_cast<float4 *>(o + 4) = make_float4(f[4], f[5], f[6], f[7]);
        if (a.xhi != nullptr) {
            float g[8];
            unpack8(ld16(a.gain + k), g);
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                ss += f[2 * e] * f[2 * e] + f[2 * e + 1] * f[2 * e + 1];
                const float v0 = f[2 * e] * g[2 * e], v1 = f[2 * e + 1] * g[2 * e + 1];
                const uint32_t h0 = f32_to_bf16_rne(v0), h1 = f32_to_bf16_rne(v1);
                const uint32_t l0 = f32_to_bf16_rne(v0 - __uint_as_float(h0 << 16));
                const uint32_t l1 = f32_to_bf16_rne(v1 - __uint_as_float(h1 << 16));
                hw[e] = h0 | (h1 << 16);
                lw[e] = l0 | (l1 << 16);
            }
            const int64_t oo = act_offset(b, k, (a.H + 127) >> 7);
            *reinterpret_cast<uint4 *>(a.xhi + oo) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
            *reinterpret_cast<uint4 *>(a.xlo + oo) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
        }
    }
    if (a.xhi != nullptr) {
        __shared__ float ssw[4];
        ss = sum64(ss);
        if ((tid & 63) == 0) ssw[tid >> 6] = ss;
        __syncthreads();
        if (tid == 0) a.ssq_out[b] = ssw[0] + ssw[1] + ssw[2] + ssw[3];
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

// Chunked prefill: the rows of a step are consecutive positions of ONE sequence
// (row b sits at position seq_lens[b]; one shared block table).  Row b's
// attention reads the positions of rows < b from the pool, so every row's new k
// (head norm, rotation) and v are stored by prefill_append_kernel before
// attention starts, with exactly the arithmetic the attention kernel applies to
// its own new token.  grid = (rows), 256 threads: aligned groups of D/8 lanes
// take the kv heads in turn.
struct PrefillAppendArgs {
    const float *qkv;        // [B][(nq+2nkv)*d]
    const float2 *cs;        // [B][d/2]
    const uint16_t *g_k;     // [d] or null
    uint16_t *pool;
    const int *block_table;  // [max_blocks], shared by all rows
    const int *seq_lens;     // [B]
    int max_blocks, num_blocks, layer, nq, nkv;
    float eps;
};

// ---------------------------------------------------------------------------
// Fused q/k head norm + rotary embedding + KV append + ragged grouped-query
// decode attention, split over the context.
//
// grid = (chunks, kv heads, rows); a block handles `chunk_tokens` consecutive
// positions of one sequence for one kv head and the G query heads that share
// it, so every K/V byte is read once for all G heads.
//
// Prologue: each aligned group of D/8 lanes holds a whole head (8 dims per
// lane), so the head RMSNorm is a reduction inside the group and the rotation
// partner (dim +- D/2) sits D/16 lanes away.  Every block prepares its G query
// heads this way.  The block that owns the chunk containing the new position T
// also prepares the new k and v, rounds them to bf16, stores them at position T
// through the block table, and feeds the rounded values to its own softmax as
// one more token (so cached positions < T come from the pool, T from registers).
//
// Main loop: a wave reads a 16-token block tile (contiguous 16*D bf16) with
// 16-byte lane loads; one load covers 512/D tokens.  Each lane group keeps its
// own running (max, sum, output) over the tokens it sees; groups, waves and
// finally chunks are merged with the usual exp(max difference) rescaling.  The
// last block to finish for a (row, kv head) merges the chunk partials in chunk
// order, so results do not depend on timing.  Partials cross compute dies
// through device-coherent stores and loads (no cache flush is needed then).
struct AttnArgs {
    const float *qkv;        // [B][(nq+2nkv)*d]: raw projections q | k | v
    const float2 *cs;        // [B][d/2] (cos, sin) at the row's position
    const uint16_t *g_q, *g_k;  // [d] head-norm gains or null
    uint16_t *pool;
    const int *block_tables;
    const int *seq_lens;
    float *out;              // [B][nq*d] float32 result, or
    uint16_t *out_hi, *out_lo;  // (batched path) the result as bf16 hi/lo in act_offset() order
    float *part;             // [B][nkv][max_chunks][G][d+2]
    int *tickets;            // [B*nkv], zero before the launch, zero after
    int max_blocks, num_blocks, layer, nq, nkv;
    int chunk_tokens;        // multiple of 64
    int max_chunks;
    int defer_merge;         // 1: leave the chunk partials for the consumer to merge
    int table_stride;        // ints between the rows' block tables (0: all rows share one table)
    int no_append;           // 1: the new tokens' K/V are already in the pool (chunked prefill)
    int n_rows;              // batch rows (the kernel that groups rows checks against it)
    float scale, eps;
};

__device__ __forceinline__ void st_coherent(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_coherent(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Online merge, in chunk order, of the chunk partials of one (row, kv head): [chunk][G][d+2] with the
// running max and sum behind the d outputs.  Thread tid produces elements idx = tid, tid + 256, ... of
// the G*d outputs (v[i] for idx = tid + 256*i; entries past G*d are not meaningful).  The device-coherent
// loads of eight chunks for ALL of a thread's elements are issued together: one round trip per eight
// chunks for the whole block instead of one per element and eight chunks.
template <int G, int D, int SG = G>
__device__ __forceinline__ void merge_chunk_partials(const float *part, int nact, int tid,
                                                     float (&v)[(G * D + 255) / 256])
{
    constexpr int NE = (G * D + 255) / 256, MR = 8;
    constexpr int64_t stride = (int64_t)SG * (D + 2);   // a chunk's record holds SG >= G heads
    float mn[NE], ls[NE], os[NE];
    const float *pe[NE];
    int dim[NE];
#pragma unroll
    for (int i = 0; i < NE; i++) {
        const int idx = min(tid + 256 * i, G * D - 1);   // clamped: a valid address, result unused
        mn[i] = -1e30f; ls[i] = 0.f; os[i] = 0.f;
        dim[i] = idx % D;
        pe[i] = part + (idx / D) * (D + 2);
    }
    for (int c0 = 0; c0 < nact; c0 += MR) {
        float mc[NE][MR], lc[NE][MR], oc[NE][MR];
#pragma unroll
        for (int i = 0; i < NE; i++)
#pragma unroll
            for (int u = 0; u < MR; u++) {
                const float *pp = pe[i] + (int64_t)min(c0 + u, nact - 1) * stride;
                mc[i][u] = ld_coherent(pp + D);
                lc[i][u] = ld_coherent(pp + D + 1);
                oc[i][u] = ld_coherent(pp + dim[i]);
            }
#pragma unroll
        for (int i = 0; i < NE; i++)
#pragma unroll
            for (int u = 0; u < MR; u++)
                if (c0 + u < nact) {
                    const float m2 = fmaxf(mn[i], mc[i][u]);
                    const float sa = __expf(mn[i] - m2), sb = __expf(mc[i][u] - m2);
                    ls[i] = ls[i] * sa + lc[i][u] * sb;
                    os[i] = os[i] * sa + oc[i][u] * sb;
                    mn[i] = m2;
                }
    }
#pragma unroll
    for (int i = 0; i < NE; i++) v[i] = os[i] / ls[i];
}

// element k of batch row b of the attention output (k = head*d + dim)
__device__ __forceinline__ void store_attn_out(const AttnArgs &a, int b, int k, int width, float v)
{
    if (a.out_hi != nullptr) {
        const uint16_t hi = f32_to_bf16_rne(v);
        const int64_t oo = act_offset(b, k, (width + 127) >> 7);
        a.out_hi[oo] = hi;
        a.out_lo[oo] = f32_to_bf16_rne(v - bf16_to_f32(hi));
    } else {
        a.out[(int64_t)b * width + k] = v;
    }
}

// One head held as 8 dims per lane by an aligned group of TPR = D/8 lanes:
// optional RMSNorm over the head (gain g, already loaded), then the half-split
// rotation by the angles whose (cos, sin) are in cs (already loaded; cs[e]
// belongs to dim (dl + e) mod D/2).
template <int D>
__device__ __forceinline__ void head_norm_rope(float (&h)[8], bool norm, const float (&g)[8],
                                               float eps, const float2 (&cs)[8], bool upper)
{
    constexpr int TPR = D / 8;
    if (norm) {
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) ss += h[e] * h[e];
        ss = (TPR == 16) ? sum16(ss) : sum8(ss);
        const float inv = rsqrtf(ss / (float)D + eps);
#pragma unroll
        for (int e = 0; e < 8; e++) h[e] = h[e] * inv * g[e];
    }
#pragma unroll
    for (int e = 0; e < 8; e++) {
        // element dl+e +- D/2 sits TPR/2 lanes away: with 16 lanes per head that is a rotation of
        // the 16-lane row by 8 (DPP row_ror:8), otherwise a shuffle
        const float other = (TPR == 16) ? dpp_f<0x128>(h[e]) : __shfl_xor(h[e], TPR / 2);
        h[e] = upper ? h[e] * cs[e].x + other * cs[e].y : h[e] * cs[e].x - other * cs[e].y;
    }
}

template <int D>
__global__ __launch_bounds__(256) void prefill_append_kernel(PrefillAppendArgs a)
{
    constexpr int BS = 16, TPR = D / 8;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int dl = (tid % TPR) * 8;
    const bool upper = dl >= D / 2;
    const float *row = a.qkv + (int64_t)b * (a.nq + 2 * a.nkv) * D;
    const float2 *cs_row = a.cs + (int64_t)b * (D / 2);
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
    const bool norm = a.g_k != nullptr;
    float gk[8];
    if (norm) {
        unpack8(ld16(a.g_k + dl), gk);
    } else {
#pragma unroll
        for (int e = 0; e < 8; e++) gk[e] = 1.f;
    }
    const int T = min(max(a.seq_lens[b], 0), a.max_blocks * BS - 1);
    const int phys = min(max(a.block_table[T / BS], 0), a.num_blocks - 1);
    // whole groups of TPR lanes stay together (the head norm reduces inside a group)
    const int heads_per_pass = 256 / TPR;
    for (int j0 = 0; j0 < a.nkv; j0 += heads_per_pass) {
        const int j = j0 + tid / TPR;
        const int jc = min(j, a.nkv - 1);
        const float *kp = row + (int64_t)(a.nq + jc) * D + dl;
        const float *vp = row + (int64_t)(a.nq + a.nkv + jc) * D + dl;
        const float4 klo = ldf4(kp), khi = ldf4(kp + 4), vlo = ldf4(vp), vhi = ldf4(vp + 4);
        float kn[8] = {klo.x, klo.y, klo.z, klo.w, khi.x, khi.y, khi.z, khi.w};
        const float vn[8] = {vlo.x, vlo.y, vlo.z, vlo.w, vhi.x, vhi.y, vhi.z, vhi.w};
        head_norm_rope<D>(kn, norm, gk, a.eps, cs, upper);
        uint32_t kb[4], vb[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            kb[e] = (uint32_t)f32_to_bf16_rne(kn[2 * e]) | ((uint32_t)f32_to_bf16_rne(kn[2 * e + 1]) << 16);
            vb[e] = (uint32_t)f32_to_bf16_rne(vn[2 * e]) | ((uint32_t)f32_to_bf16_rne(vn[2 * e + 1]) << 16);
        }
        if (j < a.nkv) {
            uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D) +
                           (T % BS) * D + dl;
            uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
            *reinterpret_cast<uint4 *>(kt) = make_uint4(kb[0], kb[1], kb[2], kb[3]);
            *reinterpret_cast<uint4 *>(vt) = make_uint4(vb[0], vb[1], vb[2], vb[3]);
        }
    }
}

// seq[i] = start + i: the positions of a prefill chunk's rows
__global__ void iota_kernel(int *seq, int start, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) seq[i] = start + i;
}

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
    const int dl = (lane % TPR) * 8;   // this lane's 8 dims
    const int sub = lane / TPR;        // token within a wave load
    const int q_stride = (a.nq + 2 * a.nkv) * D;
    const float *row = a.qkv + (int64_t)b * q_stride;
    const float2 *cs_row = a.cs + (int64_t)b * (D / 2);
    const int *table = a.block_tables + (int64_t)b * a.table_stride;

    // Everything that does not depend on the sequence length is requested
    // before the length is looked at, so the loads overlap: the raw q heads and
    // the first block-table entry this wave will need (always inside the table).
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
    // raw k and v of the new token (only the block owning position T uses them)
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
    const int first_blk = c * (a.chunk_tokens / BS) + wv;
    int phys_next = table[min(first_blk, a.max_blocks - 1)];
    // T = cached tokens = position of the new token (clamped to what the table can name)
    const int T = min(max(a.seq_lens[b], 0), a.max_blocks * BS - 1);
    const int T1 = T + 1;
    const int nact = (T1 + a.chunk_tokens - 1) / a.chunk_tokens;
    if (c >= nact) return;
    const int t0 = c * a.chunk_tokens;
    const int t1 = min(T, t0 + a.chunk_tokens);   // cached positions [t0, t1) come from the pool
    const bool owns_new = (c == nact - 1);        // position T itself

    const int blk_end = (t1 + BS - 1) / BS;
    // the tile after the current one is already in flight while the current is used
    uint4 kw[NI], vw[NI], kw_n[NI], vw_n[NI];
    if (first_blk < blk_end) {
        const int phys = min(max(phys_next, 0), a.num_blocks - 1);
        const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
        const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
#pragma unroll
        for (int i = 0; i < NI; i++) {
            kw_n[i] = ld16(kt + i * 512 + lane * 8);
            vw_n[i] = ld16(vt + i * 512 + lane * 8);
        }
        phys_next = table[min(first_blk + NWV, a.max_blocks - 1)];
    }

#pragma unroll
    for (int g = 0; g < G; g++) {
        head_norm_rope<D>(q[g], norm, gq, a.eps, cs, upper);
#pragma unroll
        for (int e = 0; e < 8; e++) q[g][e] *= a.scale;
    }
    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -1e30f;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) o[g][e] = 0.f;
    }

    if (owns_new && wv == 0) {
        // the new token: k (norm, rotation) and v, rounded to bf16, stored, and used
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
        // lane group 0 takes the new token into its running softmax
#pragma unroll
        for (int g = 0; g < G; g++) {
            float p = 0.f;
#pragma unroll
            for (int e = 0; e < 8; e++) p += q[g][e] * kn[e];
            p = (TPR == 16) ? sum16(p) : sum8(p);
            if (sub == 0) {
                m[g] = p;
                l[g] = 1.f;
#pragma unroll
                for (int e = 0; e < 8; e++) o[g][e] = vn[e];
            }
        }
    }

    for (int blk = first_blk; blk < blk_end; blk += NWV) {
#pragma unroll
        for (int i = 0; i < NI; i++) { kw[i] = kw_n[i]; vw[i] = vw_n[i]; }
        if (blk + NWV < blk_end) {
            const int phys = min(max(phys_next, 0), a.num_blocks - 1);
            const uint16_t *kt = a.pool + kv_tile_offset(a.layer, a.num_blocks, phys, 0, a.nkv, j, BS, D);
            const uint16_t *vt = kt + (int64_t)a.nkv * BS * D;
#pragma unroll
            for (int i = 0; i < NI; i++) {
                kw_n[i] = ld16(kt + i * 512 + lane * 8);
                vw_n[i] = ld16(vt + i * 512 + lane * 8);
            }
            phys_next = table[min(blk + 2 * NWV, a.max_blocks - 1)];
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
        float *pp = part + (int64_t)c * (G * (D + 2)) + g * (D + 2);
        if (a.defer_merge) {
            // the next kernel merges the partials while it loads its input
            pp[dim] = os;
            if (dim == 0) { pp[D] = mn; pp[D + 1] = ls; }
        } else if (nact == 1) {
            store_attn_out(a, b, (j * G + g) * D + dim, a.nq * D, os / ls);
        } else {
            st_coherent(pp + dim, os);
            if (dim == 0) { st_coherent(pp + D, mn); st_coherent(pp + D + 1, ls); }
        }
    }
    if (a.defer_merge || nact == 1) return;

    // Last block of this (row, kv head) merges the chunk partials.  The partial
    // stores above are device-coherent; every thread waits for its own to complete,
    // then the barrier, then one thread takes the ticket: whoever draws the last
    // ticket reads finished partials (with device-coherent loads).
    drain_stores();
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
