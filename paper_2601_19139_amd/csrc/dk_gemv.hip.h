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
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// BT threads stride over K in 8-element pieces; a block owns RB consecutive rows
// (EPI_SWIGLU: RB rows of each of the two matrices).
template <int NB, int BT, int RB, int EPI, bool NORM>
__global__ __launch_bounds__(BT) void gemv_kernel(GemvArgs a)
{
    constexpr int NW = BT / kWave;
    constexpr int NM = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int NV = NM * RB * NB + (NORM ? NB : 0);
    __shared__ float red[NW][NV];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int row0 = blockIdx.x * RB;
    const int K = a.K, N = a.N;

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
            float4 lo = ldf4(a.x + (int64_t)b * K + k), hi = ldf4(a.x + (int64_t)b * K + k + 4);
            xv[b][0] = lo.x; xv[b][1] = lo.y; xv[b][2] = lo.z; xv[b][3] = lo.w;
            xv[b][4] = hi.x; xv[b][5] = hi.y; xv[b][6] = hi.z; xv[b][7] = hi.w;
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

    float best = -INFINITY;
    int best_i = 0x7fffffff;
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
            best = out;
            best_i = row;
        }
    }
    if (a.pmax_val != nullptr && tid < 64) {
        // lanes b*RB .. b*RB+RB-1 hold the RB rows of batch row b: RB <= 16 and a
        // power of two, so a row-of-16 butterfly restricted to RB lanes reduces them
        static_assert(RB * NB <= 64, "argmax epilogue needs RB*NB <= 64");
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

__global__ __launch_bounds__(256) void argmax_final_kernel(ArgmaxArgs a)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    for (int i = tid; i < a.nblk; i += 256) {
        float v = a.pmax_val[(int64_t)b * a.nblk + i];
        int ix = a.pmax_idx[(int64_t)b * a.nblk + i];
        if (v > best || (v == best && ix < best_i)) { best = v; best_i = ix; }
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
        for (int w = 1; w < 4; w++)
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
