// Weight-streaming skinny GEMM on the matrix cores for batches of 5..64 rows.
//
//   D[r][n] = sum_k W[r][k] * X[n][k]          r: weight row, n: batch row
//
// One 16x16x32 bf16 MFMA takes a 16-row x 32-k weight tile as its A operand
// and 32 k x 16 batch rows as its B operand, so the weights go from the global
// load straight into the MFMA with no vector-ALU work at all, and each weight
// byte is still read from HBM exactly once.  The activations stay accurate:
// they are kept as two bf16 numbers hi + lo (hi = bf16(x), lo = bf16(x - hi),
// about 16 significant bits) and each weight tile is multiplied by both - the
// matrix cores have an order of magnitude more throughput than the HBM stream
// needs, so the second product is free.
//
// A block owns 16 weight rows (SWIGLU: 16 rows of each of the two matrices);
// its KS waves split K in interleaved 128-element steps (a lane loads 64
// contiguous bytes of one row per step, the wave 16 rows x 256 bytes) and add
// their accumulators through LDS in a fixed order.  With NORM the RMSNorm of
// the input is fused: the producer stored (x * gain) as hi/lo plus per-tile
// sums of x^2; the scalar 1/rms per batch row is applied in the epilogue.
#pragma once
#include "dk_common.hip.h"

namespace dk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

enum { GEPI_STORE = 0, GEPI_RESID = 1, GEPI_SWIGLU = 2 };

constexpr int kSsqStride = 64;  // floats per row of the sum-of-squares partial table

struct GemmArgs {
    const uint16_t *W;       // [N][K]
    const uint16_t *W2;      // GEPI_SWIGLU: the "up" matrix [N][K]
    int N, K, B;             // B valid batch rows (<= 16*MT)
    const uint16_t *xhi;     // [16*MT][K] bf16, hi part of the input
    const uint16_t *xlo;     // [16*MT][K] bf16, lo part
    // NORM: sum over p < n_part of ssq_in[p][n] = sum_k x[n][k]^2
    const float *ssq_in;
    int n_part;
    float eps;
    // GEPI_STORE: y[B][N] (may be null), optional running maxima [B][gridDim.x]
    float *y;
    float *pmax_val;
    int *pmax_idx;
    // GEPI_SWIGLU and GEPI_RESID: result as hi/lo bf16 [16*MT][N] for the next GEMM
    uint16_t *ohi, *olo;
    // GEPI_RESID: xres[B][N] += D; the hi/lo output is (xres * gain_next); the
    // block's sum of xres^2 per batch row goes to ssq_out[blockIdx.x][n]
    float *xres;
    const uint16_t *gain_next;  // [N]
    float *ssq_out;
};

__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16_rne(x);
    lo = f32_to_bf16_rne(x - bf16_to_f32(hi));
}

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4 &u)
{
    union { uint4 u; bf16x8_t v; } c;
    c.u = u;
    return c.v;
}

template <int MT, int KS, int EPI, bool NORM>
__global__ __launch_bounds__(KS * 64) void skinny_gemm_kernel(GemmArgs a)
{
    constexpr int NM = (EPI == GEPI_SWIGLU) ? 2 : 1;
    static_assert(KS * NM * MT <= 32, "LDS reduction buffer is limited to 32 KB");
    __shared__ float red[KS][NM][MT][4][64];
    __shared__ float ssq_s[KS][64];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int r0 = blockIdx.x * 16;
    const int K = a.K, N = a.N;

    // sum-of-squares partials of the input rows (independent of the main loop)
    if (NORM) {
        float s = 0.f;
        for (int p = wv; p < a.n_part; p += KS) s += a.ssq_in[(int64_t)p * kSsqStride + lane];
        ssq_s[wv][lane] = s;
    }

    f32x4_t acc[NM][MT];
#pragma unroll
    for (int m = 0; m < NM; m++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[m][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int wrow = min(r0 + ln, N - 1);   // clamped rows are computed and dropped
    const uint16_t *wp0 = a.W + (int64_t)wrow * K;
    const uint16_t *wp1 = (NM == 2) ? a.W2 + (int64_t)wrow * K : nullptr;
    const int nks = (K + 127) >> 7;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    for (int ks = wv; ks < nks; ks += KS) {
        const int kb = ks * 128 + lg * 32;
        uint4 wa[NM][4], bh[MT][4], bl[MT][4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int k = kb + s * 8;
            const bool in = k < K;
            wa[0][s] = in ? ld16(wp0 + k) : zero4;
            if (NM == 2) wa[NM - 1][s] = in ? ld16(wp1 + k) : zero4;
#pragma unroll
            for (int t = 0; t < MT; t++) {
                const int64_t xo = (int64_t)(t * 16 + ln) * K + k;
                bh[t][s] = in ? ld16(a.xhi + xo) : zero4;
                bl[t][s] = in ? ld16(a.xlo + xo) : zero4;
            }
        }
#pragma unroll
        for (int s = 0; s < 4; s++)
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[m][s]), as_bf16x8(bh[t][s]),
                                                                        acc[m][t], 0, 0, 0);
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wa[m][s]), as_bf16x8(bl[t][s]),
                                                                        acc[m][t], 0, 0, 0);
                }
    }

#pragma unroll
    for (int m = 0; m < NM; m++)
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int i = 0; i < 4; i++) red[wv][m][t][i][lane] = acc[m][t][i];
    __syncthreads();
    if (wv != 0) return;

    // wave 0: add the K-splits in wave order, then the epilogue.  The lane holds
    // D[r0 + 4*lg + i][n = 16*t + ln], i = 0..3.
    float best = -INFINITY;
    int best_i = 0x7fffffff;
#pragma unroll
    for (int t = 0; t < MT; t++) {
        const int n = t * 16 + ln;
        float v[NM][4];
#pragma unroll
        for (int m = 0; m < NM; m++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < KS; w++) s += red[w][m][t][i][lane];
                v[m][i] = s;
            }
        if (NORM) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < KS; w++) s += ssq_s[w][n];
            const float inv = rsqrtf(s / (float)K + a.eps);
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) v[m][i] *= inv;
        }
        const bool nvalid = n < a.B;
        const int rr = r0 + 4 * lg;
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int r = rr + i;
            if (!nvalid || r >= N) continue;
            if (EPI == GEPI_STORE) {
                const float out = v[0][i];
                if (a.y != nullptr) a.y[(int64_t)n * N + r] = out;
                if (out > best) { best = out; best_i = r; }
            } else if (EPI == GEPI_SWIGLU) {
                const float z = v[0][i];
                const float out = z / (1.0f + __expf(-z)) * v[NM - 1][i];
                uint16_t hi, lo;
                split_bf16(out, hi, lo);
                a.ohi[(int64_t)n * N + r] = hi;
                a.olo[(int64_t)n * N + r] = lo;
            } else {
                const float xn = a.xres[(int64_t)n * N + r] + v[0][i];
                a.xres[(int64_t)n * N + r] = xn;
                sq += xn * xn;
                uint16_t hi, lo;
                split_bf16(xn * bf16_to_f32(a.gain_next[r]), hi, lo);
                a.ohi[(int64_t)n * N + r] = hi;
                a.olo[(int64_t)n * N + r] = lo;
            }
        }
        if (EPI == GEPI_RESID) {
            // the block's 16 rows of batch row n are spread over the 4 lane groups
            sq += __shfl_xor(sq, 16);
            sq += __shfl_xor(sq, 32);
            if (lg == 0) a.ssq_out[(int64_t)blockIdx.x * kSsqStride + n] = nvalid ? sq : 0.f;
        }
        if (EPI == GEPI_STORE && a.pmax_val != nullptr) {
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float ov = __shfl_xor(best, off);
                const int oi = __shfl_xor(best_i, off);
                if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
            }
            if (lg == 0 && nvalid) {
                a.pmax_val[(int64_t)n * gridDim.x + blockIdx.x] = best;
                a.pmax_idx[(int64_t)n * gridDim.x + blockIdx.x] = best_i;
            }
            best = -INFINITY;
            best_i = 0x7fffffff;
        }
    }
}

}  // namespace dk
