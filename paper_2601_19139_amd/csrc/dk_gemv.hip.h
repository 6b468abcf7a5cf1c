// Weight-streaming GEMV for small batches (vector ALU, fp32 accumulation).
//
//   y[b][r] = epilogue( scale_b * sum_k W[r][k] * (x[b][k] * gain[k]) )
//
// Every weight byte is read from HBM exactly once, 16 bytes per lane per load;
// the activations (a few KB) are re-read from cache.  With NORM the RMSNorm of
// the input is fused: the gain is multiplied into x on the fly, each block sums
// x^2 over the K positions it visits anyway, and the scalar 1/rms is applied in
// the epilogue (it commutes with the matrix product).
#pragma once
#include "dk_common.hip.h"

namespace dk {

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

struct GemvArgs {
    const uint16_t *W;     // [N][K] bf16
    const uint16_t *W2;    // EPI_SWIGLU: the "up" matrix [N][K]
    const float *x;        // [NB][K]
    const uint16_t *gain;  // NORM: [K] bf16
    float eps;
    float *y;              // [NB][N]
    const float *resid;    // EPI_RESID: [NB][N] (may alias y)
    int N, K;
    float *pmax_val;       // optional per-block running maximum [NB][gridDim.x]
    int *pmax_idx;
    int tiles;             // row tiles (of RB rows) a block walks through
    // XATTN: x is the attention output, given as per-chunk softmax partials
    // part[b][kv head][chunk][g][d+2] = (unnormalised output[d], max, sum) that
    // are merged while loading (k = head*d + dim)
    const float *part;
    const int *seq_lens;
    int chunk_tokens, max_chunks, max_blocks, group, d, nkv;
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// BT threads stride over K in 8-element pieces; a block owns `tiles` consecutive
// tiles of RB rows (EPI_SWIGLU: RB rows of each of the two matrices).
template <int NB, int BT, int RB, int EPI, bool NORM, bool XATTN = false>
__global__ __launch_bounds__(BT) void gemv_kernel(GemvArgs a)
{
    constexpr int NW = BT / kWave;
    constexpr int NM = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int NV = NM * RB * NB + (NORM ? NB : 0);
    __shared__ float red[NW][NV];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int K = a.K, N = a.N;
    float best = -INFINITY;
    int best_i = 0x7fffffff;

  for (int tile = 0; tile < a.tiles; tile++) {
    const int row0 = (blockIdx.x * a.tiles + tile) * RB;
    if (row0 >= N) break;
    float acc[NM][RB][NB];
    float ssq[NB];
#pragma unroll
    for (int m = 0; m < NM; m++)
#pragma unroll
        for (int r = 0; r < RB; r++)
#pragma unroll
            for (int b = 0; b < NB; b++) acc[m][r][b] = 0.f;
#pragma unroll
    for (int b = 0; b < NB; b++) ssq[b] = 0.f;

    const uint16_t *wrow[NM][RB];
#pragma unroll
    for (int r = 0; r < RB; r++) {
        int row = min(row0 + r, N - 1);  // clamped rows are computed and dropped
        wrow[0][r] = a.W + (int64_t)row * K;
        if (NM == 2) wrow[NM - 1][r] = a.W2 + (int64_t)row * K;
    }

    for (int k = tid * 8; k < K; k += BT * 8) {
        uint4 w[NM][RB];
#pragma unroll
        for (int m = 0; m < NM; m++)
#pragma unroll
            for (int r = 0; r < RB; r++) w[m][r] = ld16(wrow[m][r] + k);
        float xv[NB][8];
#pragma unroll
        for (int b = 0; b < NB; b++) {
            if (XATTN) {
                // merge the chunk partials of head k/d (in chunk order) for dims k%d .. +8
                const int d = a.d, h = k / d, dim = k - h * d, stride = a.group * (d + 2);
                const int T1 = min(max(a.seq_lens[b], 0), a.max_blocks * 16 - 1) + 1;
                const int nact = (T1 + a.chunk_tokens - 1) / a.chunk_tokens;
                const float *pg = a.part + ((int64_t)(b * a.nkv + h / a.group) * a.max_chunks) * stride +
                                  (h % a.group) * (d + 2);
                float mn = -1e30f, ls = 0.f, os[8];
#pragma unroll
                for (int e = 0; e < 8; e++) os[e] = 0.f;
                // eight chunks per round: their loads are issued together
                constexpr int MR = 8;
                for (int c0 = 0; c0 < nact; c0 += MR) {
                    float2 ml[MR];
                    float4 lo[MR], hi[MR];
#pragma unroll
                    for (int u = 0; u < MR; u++) {
                        const float *pp = pg + (int64_t)min(c0 + u, nact - 1) * stride;
                        ml[u] = *reinterpret_cast<const float2 *>(pp + d);
                        lo[u] = ldf4(pp + dim);
                        hi[u] = ldf4(pp + dim + 4);
                    }
#pragma unroll
                    for (int u = 0; u < MR; u++) {
                        if (c0 + u < nact) {
                            const float m2 = fmaxf(mn, ml[u].x);
                            const float sa = __expf(mn - m2), sb = __expf(ml[u].x - m2);
                            ls = ls * sa + ml[u].y * sb;
                            os[0] = os[0] * sa + lo[u].x * sb; os[1] = os[1] * sa + lo[u].y * sb;
                            os[2] = os[2] * sa + lo[u].z * sb; os[3] = os[3] * sa + lo[u].w * sb;
                            os[4] = os[4] * sa + hi[u].x * sb; os[5] = os[5] * sa + hi[u].y * sb;
                            os[6] = os[6] * sa + hi[u].z * sb; os[7] = os[7] * sa + hi[u].w * sb;
                            mn = m2;
                        }
                    }
                }
                const float inv = 1.0f / ls;
#pragma unroll
                for (int e = 0; e < 8; e++) xv[b][e] = os[e] * inv;
            } else {
                float4 lo = ldf4(a.x + (int64_t)b * K + k), hi = ldf4(a.x + (int64_t)b * K + k + 4);
                xv[b][0] = lo.x; xv[b][1] = lo.y; xv[b][2] = lo.z; xv[b][3] = lo.w;
                xv[b][4] = hi.x; xv[b][5] = hi.y; xv[b][6] = hi.z; xv[b][7] = hi.w;
            }
        }
        if (NORM) {
            float g[8];
            unpack8(ld16(a.gain + k), g);
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    ssq[b] += xv[b][e] * xv[b][e];
                    xv[b][e] *= g[e];
                }
        }
#pragma unroll
        for (int m = 0; m < NM; m++)
#pragma unroll
            for (int r = 0; r < RB; r++) {
                float wf[8];
                unpack8(w[m][r], wf);
#pragma unroll
                for (int b = 0; b < NB; b++)
#pragma unroll
                    for (int e = 0; e < 8; e++) acc[m][r][b] += wf[e] * xv[b][e];
            }
    }

    // block reduction: wave sums (every lane gets them), then across waves in
    // a fixed order so that the result does not depend on timing
#pragma unroll
    for (int m = 0; m < NM; m++)
#pragma unroll
        for (int r = 0; r < RB; r++)
#pragma unroll
            for (int b = 0; b < NB; b++) {
                float s = sum64(acc[m][r][b]);
                if (lane == 0) red[wv][(m * RB + r) * NB + b] = s;
            }
    if (NORM) {
#pragma unroll
        for (int b = 0; b < NB; b++) {
            float s = sum64(ssq[b]);
            if (lane == 0) red[wv][NM * RB * NB + b] = s;
        }
    }
    __syncthreads();

    if (tid < RB * NB) {
        const int r = tid % RB, b = tid / RB;
        const int row = row0 + r;
        float v[NM];
#pragma unroll
        for (int m = 0; m < NM; m++) {
            float s = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; w2++) s += red[w2][(m * RB + r) * NB + b];
            v[m] = s;
        }
        if (NORM) {
            float s = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < NW; w2++) s += red[w2][NM * RB * NB + b];
            float inv = rsqrtf(s / (float)K + a.eps);
#pragma unroll
            for (int m = 0; m < NM; m++) v[m] *= inv;
        }
        if (row < N) {
            float out;
            if (EPI == EPI_SWIGLU) out = silu_f(v[0]) * v[NM - 1];
            else if (EPI == EPI_RESID) out = a.resid[(int64_t)b * N + row] + v[0];
            else out = v[0];
            if (a.y != nullptr) a.y[(int64_t)b * N + row] = out;
            if (out > best) { best = out; best_i = row; }   // rows ascend: ties keep the lower
        }
    }
    if (tile + 1 < a.tiles) __syncthreads();   // `red` is reused by the next tile
  }
    if (a.pmax_val != nullptr && tid < 64) {
        // lanes b*RB .. b*RB+RB-1 hold the RB rows of batch row b: RB <= 16 and a
        // power of two, so a row-of-16 butterfly restricted to RB lanes reduces them
        static_assert(RB * NB <= 64 && (RB & (RB - 1)) == 0, "argmax epilogue needs RB*NB <= 64, RB a power of two");
#pragma unroll
        for (int off = 1; off < RB; off <<= 1) {
            float ov = __shfl_xor(best, off);
            int oi = __shfl_xor(best_i, off);
            if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
        }
        if (tid < RB * NB && (tid % RB) == 0) {
            const int b = tid / RB;
            a.pmax_val[(int64_t)b * gridDim.x + blockIdx.x] = best;
            a.pmax_idx[(int64_t)b * gridDim.x + blockIdx.x] = best_i;
        }
    }
}

// Final argmax over the per-block maxima of the lm_head GEMV (lowest index
// among equal values).  One block per batch row.
struct ArgmaxArgs {
    const float *pmax_val;  // [B][nblk]
    const int *pmax_idx;
    int nblk;
    int *next;       // [B]
    int *tokens;     // advance: tokens[b] = next[b]
    int *seq_lens;   // advance: seq_lens[b] += 1
    int advance;
};

__global__ __launch_bounds__(1024) void argmax_final_kernel(ArgmaxArgs a)
{
    __shared__ float sv[16];
    __shared__ int si[16];
    const int b = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    const float *pv = a.pmax_val + (int64_t)b * a.nblk;
    const int *pi = a.pmax_idx + (int64_t)b * a.nblk;
    for (int i0 = tid; i0 < a.nblk; i0 += 1024 * 8) {
        float v[8];
        int ix[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {       // independent loads first
            const int i = i0 + u * 1024;
            v[u] = i < a.nblk ? pv[i] : -INFINITY;
            ix[u] = i < a.nblk ? pi[i] : 0x7fffffff;
        }
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (v[u] > best || (v[u] == best && ix[u] < best_i)) { best = v[u]; best_i = ix[u]; }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        float ov = __shfl_xor(best, off);
        int oi = __shfl_xor(best_i, off);
        if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
    }
    if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = best_i; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; w++)
            if (sv[w] > best || (sv[w] == best && si[w] < best_i)) { best = sv[w]; best_i = si[w]; }
        if (best_i == 0x7fffffff) best_i = 0;   // only if every logit is NaN
        a.next[b] = best_i;
        if (a.advance) {
            a.tokens[b] = best_i;
            a.seq_lens[b] += 1;
        }
    }
}

}  // namespace dk
