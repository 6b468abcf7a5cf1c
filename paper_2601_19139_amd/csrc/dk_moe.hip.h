// Mixture-of-experts MLP: softmax router with top-k selection, expert SwiGLU
// GEMMs over only the experts that some row selected, and the weighted
// combination.  Every byte of a selected expert is streamed once per step; the
// blocks of an expert nobody selected read one counter and exit.
#pragma once
#include "dk_common.hip.h"
#include "dk_gemm.hip.h"

namespace dk {

// ---------------------------------------------------------------------------
// Router, in two small kernels.
//   logits: grid (ceil(E/8), B), 256 threads.  Each block normalises its row
//           (h = rmsnorm(x) * gain, recomputed per block: the row is a few KB)
//           and computes 8 router logits, two per wave.
//   select: grid (B), one wave.  Softmax over all experts, the top_k largest
//           probabilities (ties to the lower expert index) renormalised to sum
//           to one.  Each (row, slot) pair is appended to the list of the expert
//           it chose, so that the expert kernels need no search.
struct RouterArgs {
    const float *x;          // [B][H] residual stream
    const uint16_t *gain;    // [H]
    const uint16_t *w_router;  // [E][H]
    float eps;
    int H, E, top_k;
    float *logits;           // [B][E]
    int *topk_idx;           // [B][top_k] experts in order of decreasing probability
    float *topk_w;           // [B][top_k] renormalised weights
    float *rinv;             // [B] 1/rms of the row (the expert GEMMs apply it)
    int B;
    int *exp_cnt;            // [E] pairs that chose the expert
    int *exp_list;           // [E][B*top_k] their indices row*top_k + slot (any order)
};

__global__ __launch_bounds__(256) void moe_router_logits_kernel(RouterArgs a)
{
    __shared__ float xs[8192];           // x * gain for the row (H <= 8192)
    __shared__ float red[4];
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float *xr = a.x + (int64_t)b * a.H;
    float ss = 0.f;
    for (int k = tid * 4; k < a.H; k += 1024) {
        const float4 v = ldf4(xr + k);
        const uint2 gw = *reinterpret_cast<const uint2 *>(a.gain + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        xs[k] = v.x * bf16lo(gw.x);
        xs[k + 1] = v.y * bf16hi(gw.x);
        xs[k + 2] = v.z * bf16lo(gw.y);
        xs[k + 3] = v.w * bf16hi(gw.y);
    }
    ss = sum64(ss);
    if (lane == 0) red[wv] = ss;
    __syncthreads();
    const float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)a.H + a.eps);
    if (blockIdx.x == 0 && tid == 0) a.rinv[b] = inv;
    // the counters of this block's 8 experts start at zero for the select kernel
    if (b == 0 && tid < 8 && blockIdx.x * 8 + tid < a.E) a.exp_cnt[blockIdx.x * 8 + tid] = 0;
    // wave wv: experts 8*blockIdx.x + 2*wv, +1; lanes stride over H in 8-element pieces
    const int e0 = blockIdx.x * 8 + wv * 2;
    const uint16_t *w0 = a.w_router + (int64_t)min(e0, a.E - 1) * a.H;
    const uint16_t *w1 = a.w_router + (int64_t)min(e0 + 1, a.E - 1) * a.H;
    float acc0 = 0.f, acc1 = 0.f;
    for (int k = lane * 8; k < a.H; k += 512) {
        float f0[8], f1[8];
        unpack8(ld16(w0 + k), f0);
        unpack8(ld16(w1 + k), f1);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            acc0 += f0[i] * xs[k + i];
            acc1 += f1[i] * xs[k + i];
        }
    }
    acc0 = sum64(acc0);
    acc1 = sum64(acc1);
    if (lane == 0) {
        if (e0 < a.E) a.logits[(int64_t)b * a.E + e0] = acc0 * inv;
        if (e0 + 1 < a.E) a.logits[(int64_t)b * a.E + e0 + 1] = acc1 * inv;
    }
}

__global__ __launch_bounds__(64) void moe_router_select_kernel(RouterArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const float *logit = a.logits + (int64_t)b * a.E;
    // softmax over the E logits (lane holds experts lane, lane+64, ...; E <= 256)
    float p[4];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int e = lane + 64 * i;
        p[i] = e < a.E ? logit[e] : -INFINITY;
        mx = fmaxf(mx, p[i]);
    }
    mx = max64(mx);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        p[i] = (lane + 64 * i < a.E) ? expf(p[i] - mx) : -1.f;   // -1 marks "not an expert"
        sum += fmaxf(p[i], 0.f);
    }
    sum = sum64(sum);
#pragma unroll
    for (int i = 0; i < 4; i++)
        if (p[i] >= 0.f) p[i] /= sum;
    // top_k by repeated argmax (largest probability, lowest index among equals)
    float sel_sum = 0.f, my_w = 0.f;
    int my_e = 0;
    for (int k = 0; k < a.top_k; k++) {
        float bv = -1.f;
        int be = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < 4; i++)
            if (p[i] > bv) { bv = p[i]; be = lane + 64 * i; }   // ascending index: ties keep the lower
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oe = __shfl_xor(be, off);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        sel_sum += bv;
        if (lane == k) { my_w = bv; my_e = be; }
#pragma unroll
        for (int i = 0; i < 4; i++)
            if (lane + 64 * i == be) p[i] = -1.f;   // taken
    }
    if (lane < a.top_k) {
        const int pair = b * a.top_k + lane;
        a.topk_idx[pair] = my_e;
        a.topk_w[pair] = my_w / sel_sum;
        // the pair joins its expert's list (the counters were cleared by the logits kernel).
        // The order of a list depends on timing; the expert kernels compute every pair's
        // column independently, so their results do not.
        const int pos = atomicAdd(a.exp_cnt + my_e, 1);
        a.exp_list[(int64_t)my_e * (a.B * a.top_k) + pos] = pair;
    }
}

// ---------------------------------------------------------------------------
// Expert GEMMs.  grid = (row tiles, experts).  A block looks up how many (row,
// slot) pairs selected its expert (none -> it exits) and their ordered list.  The
// pairs become the batch columns of 16x16x32 bf16 MFMAs exactly as in the dense
// skinny GEMM (activations as bf16 hi + lo in act_offset() order, KS waves
// splitting K, accumulators added through LDS in wave order).
//
// UP:   in  = (x * gain) of batch row `row`            (activation row = row)
//       out = silu(rinv*Wg x) * (rinv*Wu x) as hi/lo   (activation row = row*top_k + slot)
// DOWN: in  = the UP output of (row, slot)
//       out = y[row*top_k + slot][:] = Wd act   (float32; weighted and summed later)
struct ExpertArgs {
    const uint16_t *w_a;     // UP: gate [E][Fe][H];  DOWN: down [E][H][Fe]
    const uint16_t *w_b;     // UP: up   [E][Fe][H]
    int N, K;                // rows and columns of one expert matrix
    int n_experts;           // Q4: the packed matrices hold all experts stacked by rows (E*N rows)
    int B, top_k;
    const int *exp_cnt;      // [E] pairs that chose the expert
    const int *exp_list;     // [E][B*top_k] pair indices row*top_k + slot (any order)
    const uint16_t *xhi, *xlo;   // input activations (act_offset order)
    const float *rinv;       // UP: [B]
    uint16_t *ohi, *olo;     // UP: output activations (act_offset order, K' = N)
    float *y;                // DOWN: [B*top_k][N]
};

template <bool UP, int KS>
__global__ __launch_bounds__(KS * 64) void moe_expert_kernel(ExpertArgs a)
{
    constexpr int NM = UP ? 2 : 1;
    __shared__ float red[KS][NM][4][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const int e = blockIdx.y;
    const int r0 = blockIdx.x * 16;
    const int K = a.K, N = a.N;

    const int ncol = a.exp_cnt[e];
    if (ncol == 0) return;
    const int *col_row = a.exp_list + (int64_t)e * (a.B * a.top_k);

    const int wrow = min(r0 + ln, N - 1);
    const uint16_t *wp0 = a.w_a + ((int64_t)e * N + wrow) * K;
    const uint16_t *wp1 = UP ? a.w_b + ((int64_t)e * N + wrow) * K : nullptr;
    const int nks = (K + 127) >> 7;
    const int onks = (N + 127) >> 7;

    for (int c0 = 0; c0 < ncol; c0 += 16) {   // 16 batch columns per pass
        // column ln of this pass: pair index, its batch row, its activation row
        const int pair = col_row[min(c0 + ln, ncol - 1)];
        const int in_row = UP ? pair / a.top_k : pair;
        const int64_t xbase = (((int64_t)(in_row >> 4) * nks) * 4 * 64 + lg * 16 + (in_row & 15)) * 8;

        f32x4_t acc[NM];
#pragma unroll
        for (int m = 0; m < NM; m++) acc[m] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int ks = wv; ks < nks; ks += KS) {
            const int kb = ks * 128 + lg * 8;
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const bool in = kb + s * 32 < K;
                const int kc = min(kb + s * 32, K - 8);
                const uint4 z = make_uint4(0, 0, 0, 0);
                const int64_t xo = xbase + ((int64_t)ks * 4 + s) * 512;
                const uint4 h4 = in ? ld16(a.xhi + xo) : z, l4 = in ? ld16(a.xlo + xo) : z;
                const uint4 w0 = in ? ld16(wp0 + kc) : z;
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w0), as_bf16x8(h4), acc[0], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w0), as_bf16x8(l4), acc[0], 0, 0, 0);
                if (UP) {
                    const uint4 w1 = in ? ld16(wp1 + kc) : z;
                    acc[NM - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w1), as_bf16x8(h4),
                                                                          acc[NM - 1], 0, 0, 0);
                    acc[NM - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w1), as_bf16x8(l4),
                                                                          acc[NM - 1], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int m = 0; m < NM; m++)
#pragma unroll
            for (int i = 0; i < 4; i++) red[wv][m][i][lane] = acc[m][i];
        __syncthreads();
        if (wv == 0 && c0 + ln < ncol) {
            // lane holds D[r0 + 4*lg + i][column ln]
            float v[NM][4];
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < KS; w++) s += red[w][m][i][lane];
                    v[m][i] = s;
                }
            const float inv = UP ? a.rinv[in_row] : 1.f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int r = r0 + 4 * lg + i;
                if (r >= N) continue;
                if (UP) {
                    const float z = v[0][i] * inv;
                    const float out = z / (1.0f + __expf(-z)) * (v[NM - 1][i] * inv);
                    uint16_t hi, lo;
                    split_bf16(out, hi, lo);
                    const int64_t oo = act_offset(pair, r, onks);
                    a.ohi[oo] = hi;
                    a.olo[oo] = lo;
                } else {
                    a.y[(int64_t)pair * N + r] = v[0][i];
                }
            }
        }
        __syncthreads();   // `red` is reused by the next pass
    }
}

// The same expert GEMMs for K a multiple of 128 (every request unconditional and
// inside the matrix), restructured like the dense skinny GEMM: a wave requests
// all the weight and activation pieces of a round (PD k-steps of 128 columns, RT
// row tiles) before the first MFMA, so a block pays one memory round trip per
// round instead of one per 32 columns.  A block covers 16*RT rows; the RT tiles
// share the activation registers.  Wave w < RT reduces and stores tile w.
//
// Q4: w_a / w_b are packed 4-bit matrices (layout of dk_create_model_q4) of E*N rows, expert e owning rows
// e*N..; N a multiple of 16.  Evaluated as in the dense 4-bit GEMM: codes through the matrix cores, the
// group sums of x from an all-ones operand, scale and bias applied to the fp32 tiles.
template <bool UP, int KS, int RT, int PD, bool Q4 = false>
__global__ __launch_bounds__(KS * 64) void moe_expert_fast_kernel(ExpertArgs a)
{
    constexpr int NM = UP ? 2 : 1;
    static_assert(RT <= KS, "one wave per row tile in the epilogue");
    __shared__ float red[KS][RT][NM][4][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const int e = blockIdx.y;
    const int r0 = blockIdx.x * 16 * RT;
    const int K = a.K, N = a.N;

    const int ncol = a.exp_cnt[e];
    if (ncol == 0) return;
    const int *col_row = a.exp_list + (int64_t)e * (a.B * a.top_k);

    const int nks = K >> 7;
    const int onks = (N + 127) >> 7;
    const uint16_t *wp0[RT], *wp1[RT];
    // Q4: byte offsets of the lane's codes (row of its tile) and of its tiles' (scale, bias) pieces
    int64_t qc[RT], qs[RT];
#pragma unroll
    for (int t = 0; t < RT; t++) {
        const int wrow = min(r0 + 16 * t + ln, N - 1);
        wp0[t] = a.w_a + ((int64_t)e * N + wrow) * K + lg * 8;
        wp1[t] = UP ? a.w_b + ((int64_t)e * N + wrow) * K + lg * 8 : nullptr;
        if (Q4) {
            const int tile = min((r0 >> 4) + t, (N >> 4) - 1);
            qc[t] = ((int64_t)e * N + min(tile * 16 + ln, N - 1)) * (K >> 1) + lg * 16;
            qs[t] = (int64_t)a.n_experts * N * (K >> 1) + (((int64_t)e * (N >> 4) + tile) * nks * 4 + lg) * 32;
        }
    }
    const uint8_t *qa = reinterpret_cast<const uint8_t *>(a.w_a), *qb = reinterpret_cast<const uint8_t *>(a.w_b);

    for (int c0 = 0; c0 < ncol; c0 += 16) {   // 16 batch columns per pass
        const int pair = col_row[min(c0 + ln, ncol - 1)];
        const int in_row = UP ? pair / a.top_k : pair;
        const int64_t xbase = (((int64_t)(in_row >> 4) * nks) * 4 * 64 + lg * 16 + (in_row & 15)) * 8;

        f32x4_t acc[RT][NM];
#pragma unroll
        for (int t = 0; t < RT; t++)
#pragma unroll
            for (int m = 0; m < NM; m++) acc[t][m] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int ks0 = wv; ks0 < nks; ks0 += PD * KS) {
            uint4 w0[PD][RT][4], w1[PD][RT][4], h4[PD][4], l4[PD][4];
#pragma unroll
            for (int p = 0; p < PD; p++) {
                const int ks = min(ks0 + p * KS, nks - 1);   // past the end: a valid re-read, zeroed below
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int64_t xo = xbase + ((int64_t)ks * 4 + s) * 512;
                    h4[p][s] = ld16(a.xhi + xo);
                    l4[p][s] = ld16(a.xlo + xo);
                    if (!Q4) {
#pragma unroll
                        for (int t = 0; t < RT; t++) {
                            w0[p][t][s] = ld16(wp0[t] + ks * 128 + s * 32);
                            if (UP) w1[p][t][s] = ld16(wp1[t] + ks * 128 + s * 32);
                        }
                    }
                }
                if (Q4) {
                    // [0]: the step's 32 codes of the lane's row; [1], [2]: (scale, bias) of its two groups
#pragma unroll
                    for (int t = 0; t < RT; t++) {
                        w0[p][t][0] = ld16(qa + qc[t] + ks * 64);
                        w0[p][t][1] = ld16(qa + qs[t] + (int64_t)ks * 128);
                        w0[p][t][2] = ld16(qa + qs[t] + (int64_t)ks * 128 + 16);
                        if (UP) {
                            w1[p][t][0] = ld16(qb + qc[t] + ks * 64);
                            w1[p][t][1] = ld16(qb + qs[t] + (int64_t)ks * 128);
                            w1[p][t][2] = ld16(qb + qs[t] + (int64_t)ks * 128 + 16);
                        }
                    }
                }
            }
            if constexpr (Q4) {
                const uint4 one4 = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
                const f32x4_t zero = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int p = 0; p < PD; p++) {
                    if (ks0 + p * KS >= nks) continue;   // past the end of K (the same for the whole wave)
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        const uint4 bh0 = h4[p][2 * h], bl0 = l4[p][2 * h], bh1 = h4[p][2 * h + 1], bl1 = l4[p][2 * h + 1];
                        f32x4_t S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bh0), zero, 0, 0, 0);
                        S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bl0), S, 0, 0, 0);
                        S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bh1), S, 0, 0, 0);
                        S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bl1), S, 0, 0, 0);
#pragma unroll
                        for (int t = 0; t < RT; t++)
#pragma unroll
                            for (int m = 0; m < NM; m++) {
                                const uint4 cw = m ? w1[p][t][0] : w0[p][t][0];
                                const uint4 sb = m ? w1[p][t][1 + h] : w0[p][t][1 + h];
                                const uint32_t sbw[4] = {sb.x, sb.y, sb.z, sb.w};
                                const uint4 cq0 = q4_codes_bf16(h ? cw.z : cw.x), cq1 = q4_codes_bf16(h ? cw.w : cw.y);
                                f32x4_t D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cq0), as_bf16x8(bh0), zero, 0, 0, 0);
                                D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cq0), as_bf16x8(bl0), D, 0, 0, 0);
                                D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cq1), as_bf16x8(bh1), D, 0, 0, 0);
                                D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cq1), as_bf16x8(bl1), D, 0, 0, 0);
#pragma unroll
                                for (int i = 0; i < 4; i++)
                                    acc[t][m][i] = fmaf(__uint_as_float(sbw[i] << 16), D[i],
                                                        fmaf(__uint_as_float(sbw[i] & 0xFFFF0000u), S[i], acc[t][m][i]));
                            }
                    }
                }
                continue;
            }
#pragma unroll
            for (int p = 0; p < PD; p++) {
                const bool ok = ks0 + p * KS < nks;
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const uint4 z = make_uint4(0, 0, 0, 0);
                    const uint4 hh = ok ? h4[p][s] : z, ll = ok ? l4[p][s] : z;
#pragma unroll
                    for (int t = 0; t < RT; t++) {
                        acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w0[p][t][s]), as_bf16x8(hh),
                                                                            acc[t][0], 0, 0, 0);
                        acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w0[p][t][s]), as_bf16x8(ll),
                                                                            acc[t][0], 0, 0, 0);
                        if (UP) {
                            acc[t][NM - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                as_bf16x8(w1[p][t][s]), as_bf16x8(hh), acc[t][NM - 1], 0, 0, 0);
                            acc[t][NM - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                as_bf16x8(w1[p][t][s]), as_bf16x8(ll), acc[t][NM - 1], 0, 0, 0);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < RT; t++)
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) red[wv][t][m][i][lane] = acc[t][m][i];
        __syncthreads();
        if (wv < RT && c0 + ln < ncol) {
            // lane holds D[r0 + 16*wv + 4*lg + i][column ln]
            float v[NM][4];
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < KS; w++) sum += red[w][wv][m][i][lane];
                    v[m][i] = sum;
                }
            const float inv = UP ? a.rinv[in_row] : 1.f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int r = r0 + 16 * wv + 4 * lg + i;
                if (r >= N) continue;
                if (UP) {
                    const float z = v[0][i] * inv;
                    const float out = z / (1.0f + __expf(-z)) * (v[NM - 1][i] * inv);
                    uint16_t hi, lo;
                    split_bf16(out, hi, lo);
                    const int64_t oo = act_offset(pair, r, onks);
                    a.ohi[oo] = hi;
                    a.olo[oo] = lo;
                } else {
                    a.y[(int64_t)pair * N + r] = v[0][i];
                }
            }
        }
        __syncthreads();   // `red` is reused by the next pass
    }
}

// ---------------------------------------------------------------------------
// x[b] += sum_k w[b][k] * y[b*top_k + k]   (k in the router's order), then the
// input of the next matrix-core GEMM: (x * next gain) as hi/lo and the sum of
// squares of the block's columns.  grid = (ceil(H/1024), B): a block covers
// 1024 columns of one row, four per thread.
struct MoeCombineArgs {
    float *x;                // [B][H]
    const float *y;          // [B*top_k][H]
    const float *topk_w;     // [B][top_k]
    const uint16_t *gain_next;  // [H]
    uint16_t *xhi, *xlo;
    float *ssq_out;          // [gridDim.x][kSsqStride]: entry [blockIdx.x][b]
    int H, top_k;
};

__global__ __launch_bounds__(256) void moe_combine_kernel(MoeCombineArgs a)
{
    __shared__ float red[4];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int nks = (a.H + 127) >> 7;
    const int k = blockIdx.x * 1024 + tid * 4;
    float ss = 0.f;
    if (k < a.H) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < a.top_k; j++) {
            const float w = a.topk_w[b * a.top_k + j];
            const float4 v = ldf4(a.y + ((int64_t)b * a.top_k + j) * a.H + k);
            acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
        }
        float4 xn = ldf4(a.x + (int64_t)b * a.H + k);
        xn.x += acc.x; xn.y += acc.y; xn.z += acc.z; xn.w += acc.w;
        *reinterpret_cast<float4 *>(a.x + (int64_t)b * a.H + k) = xn;
        ss = xn.x * xn.x + xn.y * xn.y + xn.z * xn.z + xn.w * xn.w;
        const uint2 gw = *reinterpret_cast<const uint2 *>(a.gain_next + k);
        uint16_t h[4], l[4];
        split_bf16(xn.x * bf16lo(gw.x), h[0], l[0]);
        split_bf16(xn.y * bf16hi(gw.x), h[1], l[1]);
        split_bf16(xn.z * bf16lo(gw.y), h[2], l[2]);
        split_bf16(xn.w * bf16hi(gw.y), h[3], l[3]);
        const int64_t oo = act_offset(b, k, nks);   // 4 consecutive k stay inside one 8-element piece
        *reinterpret_cast<uint2 *>(a.xhi + oo) = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16),
                                                            (uint32_t)h[2] | ((uint32_t)h[3] << 16));
        *reinterpret_cast<uint2 *>(a.xlo + oo) = make_uint2((uint32_t)l[0] | ((uint32_t)l[1] << 16),
                                                            (uint32_t)l[2] | ((uint32_t)l[3] << 16));
    }
    ss = sum64(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) a.ssq_out[(int64_t)blockIdx.x * kSsqStride + b] = red[0] + red[1] + red[2] + red[3];
}

}  // namespace dk
