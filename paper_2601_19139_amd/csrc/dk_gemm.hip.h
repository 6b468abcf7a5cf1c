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
// A block owns a group of 16*RT weight rows (SWIGLU: of each of the two
// matrices); its KS waves split K in interleaved 128-element steps (a lane loads 64
// contiguous bytes of one row per step, the wave 16 rows x 256 bytes) and add
// their accumulators through LDS in a fixed order.  The activations are stored
// in the order the B-operand loads consume them (act_offset), so each of those
// loads is one contiguous 1 KB run per wave.  With NORM the RMSNorm of
// the input is fused: the producer stored (x * gain) as hi/lo plus per-tile
// sums of x^2; the scalar 1/rms per batch row is applied in the epilogue.
//
// Q4: the weights are 4-bit codes with a bf16 scale and bias per group of 64
// columns (w = scale * q + bias).  A lane's 16-byte load then carries a whole
// K-step (32 codes) of its row.  The product is evaluated exactly as
//   sum_g ( scale_g * sum_{k in g} q_k x_k  +  bias_g * sum_{k in g} x_k ):
// the codes go to the matrix cores as the bf16 numbers 0..15, a second product
// with an all-ones operand gives the group sums of x, and fused multiply-adds
// apply scale and bias to the fp32 tiles.  (Feeding the codes as 128 + q, which
// is a two-instruction bit pattern, was measured to cost three decimal digits:
// the matrix cores do not keep the full fp32 sum while adding products, and the
// offset term, 17 times the useful one, has to cancel afterwards.)
#pragma once
#include "dk_common.hip.h"

namespace dk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

enum { GEPI_STORE = 0, GEPI_RESID = 1, GEPI_SWIGLU = 2 };

constexpr int kSsqStride = 64;  // floats per row of the sum-of-squares partial table

struct GemmArgs {
    const uint16_t *W;       // [N][K] bf16; Q4: the packed 4-bit matrix (codes, then scale/bias tiles)
    const uint16_t *W2;      // GEPI_SWIGLU: the "up" matrix, same format as W
    int N, K, B;             // B valid batch rows (<= 16*MT)
    int q4;                  // host side only: W / W2 are packed 4-bit matrices (selects the Q4 kernels)
    const uint16_t *xhi;     // hi part of the input, bf16 in act_offset() order
    const uint16_t *xlo;     // lo part
    // NORM: sum over p < n_part of ssq_in[p][n] = sum_k x[n][k]^2
    const float *ssq_in;
    int n_part;
    float eps;
    // GEPI_STORE: y[B][N] (may be null), optional running maxima [B][ceil(N/16)]
    float *y;
    float *pmax_val;
    int *pmax_idx;
    // GEPI_SWIGLU and GEPI_RESID: result as hi/lo bf16 in act_offset() order (K = N)
    // for the next GEMM
    uint16_t *ohi, *olo;
    // GEPI_RESID: xres[B][N] += D; the hi/lo output is (xres * gain_next); the
    // sum of xres^2 over each 16-row tile and batch row goes to ssq_out[tile][n]
    float *xres;
    const uint16_t *gain_next;  // [N]
    float *ssq_out;
    // shared_gemm_kernel with K cut into slices: partial tiles and one ticket per row block
    // (zero before the launch, zero after)
    float *kpart;
    int *ktickets;
};

__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16_rne(x);
    lo = f32_to_bf16_rne(x - bf16_to_f32(hi));
}

// the same for two values: a in the low half-words of hi / lo, b in the high ones
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t &hi, uint32_t &lo)
{
    hi = f32x2_to_bf16x2_rne(a, b);
    lo = f32x2_to_bf16x2_rne(a - bf16lo(hi), b - bf16hi(hi));
}

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4 &u)
{
    union { uint4 u; bf16x8_t v; } c;
    c.u = u;
    return c.v;
}

// The eight 4-bit codes of a word (code j in bits 4j..4j+3) as exact bf16 numbers, in matrix-core
// operand order: bytes of nibbles, byte -> float, then the upper halves of two floats side by side.
__device__ __forceinline__ uint4 q4_codes_bf16(uint32_t w)
{
    const uint32_t ev = w & 0x0F0F0F0Fu, od = (w >> 4) & 0x0F0F0F0Fu;
    uint4 r;
    r.x = __builtin_amdgcn_perm(__float_as_uint((float)(od & 0xFFu)), __float_as_uint((float)(ev & 0xFFu)), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint((float)((od >> 8) & 0xFFu)), __float_as_uint((float)((ev >> 8) & 0xFFu)), 0x07060302u);
    r.z = __builtin_amdgcn_perm(__float_as_uint((float)((od >> 16) & 0xFFu)), __float_as_uint((float)((ev >> 16) & 0xFFu)), 0x07060302u);
    r.w = __builtin_amdgcn_perm(__float_as_uint((float)(od >> 24)), __float_as_uint((float)(ev >> 24)), 0x07060302u);
    return r;
}

// Epilogue of one finished 16-row tile.  The lane holds D[row0 + 4*lg + i][n = 16*t + ln], i = 0..3, in
// v[t][matrix][i] (already scaled by 1/rms where the input norm is fused).  xr / gn: the residual rows and the
// next norm's gains of exactly those elements (GEPI_RESID; loaded by the caller ahead of the weight stream).
template <int MT, int EPI>
__device__ __forceinline__ void gemm_tile_epilogue(const GemmArgs &a, int out_tile, int lane,
                                                   const float (&v)[MT][(EPI == GEPI_SWIGLU) ? 2 : 1][4],
                                                   const float (&xr)[MT][4], const float (&gn)[4])
{
    constexpr int NM = (EPI == GEPI_SWIGLU) ? 2 : 1;
    const int ln = lane & 15, lg = lane >> 4;
    const int N = a.N;
    const int onks = (N + 127) >> 7;   // K-steps of the GEMM that consumes this output
    const int n_tiles = (N + 15) >> 4;
    const int row0 = out_tile * 16;
    float best = -INFINITY;
    int best_i = 0x7fffffff;
#pragma unroll
    for (int t = 0; t < MT; t++) {
        const int n = t * 16 + ln;
        const bool nvalid = n < a.B;
        const int rr = row0 + 4 * lg;
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int r = rr + i;
            if (!nvalid || r >= N) continue;
            if (EPI == GEPI_STORE) {
                const float out = v[t][0][i];
                if (a.y != nullptr) a.y[(int64_t)n * N + r] = out;
                if (out > best) { best = out; best_i = r; }
            } else if (EPI == GEPI_SWIGLU) {
                const float z = v[t][0][i];
                const float out = z / (1.0f + __expf(-z)) * v[t][NM - 1][i];
                uint16_t hi, lo;
                split_bf16(out, hi, lo);
                const int64_t oo = act_offset(n, r, onks);
                a.ohi[oo] = hi;
                a.olo[oo] = lo;
            } else {
                const float xn = xr[t][i] + v[t][0][i];
                a.xres[(int64_t)n * N + r] = xn;
                sq += xn * xn;
                uint16_t hi, lo;
                split_bf16(xn * gn[i], hi, lo);
                const int64_t oo = act_offset(n, r, onks);
                a.ohi[oo] = hi;
                a.olo[oo] = lo;
            }
        }
        if (EPI == GEPI_RESID) {
            // the tile's 16 rows of batch row n are spread over the 4 lane groups
            sq += __shfl_xor(sq, 16);
            sq += __shfl_xor(sq, 32);
            if (lg == 0) a.ssq_out[(int64_t)out_tile * kSsqStride + n] = nvalid ? sq : 0.f;
        }
        if (EPI == GEPI_STORE && a.pmax_val != nullptr) {
#pragma unroll
            for (int off = 16; off < 64; off <<= 1) {
                const float ov = __shfl_xor(best, off);
                const int oi = __shfl_xor(best_i, off);
                if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
            }
            if (lg == 0 && nvalid) {
                a.pmax_val[(int64_t)n * n_tiles + out_tile] = best;
                a.pmax_idx[(int64_t)n * n_tiles + out_tile] = best_i;
            }
            best = -INFINITY;
            best_i = 0x7fffffff;
        }
    }
}

// KALIGNED: K is a multiple of 128 (every real model shape); the K-steps are then
// whole and the loaded registers feed the MFMAs untouched.
// Q4 (needs KALIGNED): per row K/2 bytes of codes, a K-step of 128 columns being 16 words
// [lane group lg][sub-step s] whose nibble j (bits 4j..4j+3) is column s*32 + lg*8 + j;
// after the N rows, per 16-row tile and K-step 128 bytes [lg][group h of the step][row 4*lg+i]
// of (scale, bias) bf16 pairs - the order in which the accumulator lanes need them.
template <int MT, int KS, int RT, int PD, int EPI, bool NORM, bool KALIGNED, bool Q4 = false>
__global__ __launch_bounds__(KS * 64) void skinny_gemm_kernel(GemmArgs a)
{
    static_assert(!Q4 || KALIGNED, "4-bit weights need whole K-steps");
    constexpr int NM = (EPI == GEPI_SWIGLU) ? 2 : 1;
    constexpr int NA = NM * RT;   // weight tiles (accumulator sets) per wave
    static_assert(KS * NA * MT <= 32, "LDS reduction buffer is limited to 32 KB");
    extern __shared__ float dyn_lds[];
    typedef float RedBuf[KS][NA][MT][4][64];
    RedBuf *red = reinterpret_cast<RedBuf *>(dyn_lds);
    float (*ssq_s)[64] = reinterpret_cast<float (*)[64]>(dyn_lds + sizeof(RedBuf) / sizeof(float));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, known to be uniform
    const int ln = lane & 15, lg = lane >> 4;
    const int K = a.K, N = a.N;
    const int nks = (K + 127) >> 7;
    if (gridDim.y > 1) {
        // The batch rows are split across blockIdx.y in groups of 16*MT: a small matrix (few row
        // tiles) then still gives every compute unit a block, each with a quarter of the epilogue,
        // and the weights, read once per group, stay in the caches.  Every table is tile-major or
        // row-major in the batch row, so a group is the same problem behind shifted pointers.
        const int ct = (int)blockIdx.y * MT;   // first column tile of this block
        const int64_t onks = (N + 127) >> 7, n_tiles = (N + 15) >> 4;
        a.xhi += (int64_t)ct * nks * 2048;
        a.xlo += (int64_t)ct * nks * 2048;
        if (NORM) a.ssq_in += 16 * ct;
        if (EPI == GEPI_STORE) {
            if (a.y != nullptr) a.y += (int64_t)16 * ct * N;
            if (a.pmax_val != nullptr) {
                a.pmax_val += (int64_t)16 * ct * n_tiles;
                a.pmax_idx += (int64_t)16 * ct * n_tiles;
            }
        } else {
            a.ohi += (int64_t)ct * onks * 2048;
            a.olo += (int64_t)ct * onks * 2048;
        }
        if (EPI == GEPI_RESID) {
            a.xres += (int64_t)16 * ct * N;
            a.ssq_out += 16 * ct;
        }
        a.B = min(16 * MT, a.B - 16 * ct);
    }
    const int niter = (nks + KS - 1) / KS;   // K-steps per wave and row group
    const int niter2 = (niter + PD - 1) / PD * PD;   // padded to the pipeline depth

    f32x4_t acc[NA][MT];
#pragma unroll
    for (int m = 0; m < NA; m++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[m][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Software pipeline: PD K-steps are always in flight per wave.  The loop has
    // no conditional loads and no stores (the compiler can then wait for exactly
    // the stage it is about to use): every wave runs the same number of steps, a
    // multiple of PD; a step past the end of K reads clamped (valid, cached)
    // addresses and is not used.
    struct Stage {
        uint4 wa[NA][4], bh[MT][4], bl[MT][4];
    };
    int it_i = 0;   // step to issue next
    auto issue = [&](Stage &st) {
        const int g = (int)blockIdx.x;
        const int ks = min(it_i * KS + wv, nks - 1);
        const int kb = ks * 128 + lg * 8;
        if constexpr (Q4) {
            const int n_tiles16 = (N + 15) >> 4;
#pragma unroll
            for (int m = 0; m < NA; m++) {
                const uint8_t *base = reinterpret_cast<const uint8_t *>((m / RT) ? a.W2 : a.W);
                const int tile = min(g * RT + (m % RT), n_tiles16 - 1);
                const int wrow = min(tile * 16 + ln, N - 1);
                st.wa[m][0] = ld16(base + (int64_t)wrow * (K >> 1) + ks * 64 + lg * 16);
                const uint8_t *sb = base + (int64_t)N * (K >> 1) + (((int64_t)tile * nks + ks) * 4 + lg) * 32;
                st.wa[m][1] = ld16(sb);
                st.wa[m][2] = ld16(sb + 16);
            }
            const int64_t xb = ((int64_t)ks * 4 * 64 + lane) * 8;
#pragma unroll
            for (int s = 0; s < 4; s++)
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    const int64_t xo = xb + ((int64_t)t * nks * 4 + s) * 512;
                    st.bh[t][s] = ld16(a.xhi + xo);
                    st.bl[t][s] = ld16(a.xlo + xo);
                }
            it_i++;
            return;
        }
        const uint16_t *wq[NA];
#pragma unroll
        for (int m = 0; m < NA; m++) {
            // tile m: matrix m / RT, rows of group g; rows past the end are clamped
            const int wrow = min(g * (16 * RT) + 16 * (m % RT) + ln, N - 1);
            wq[m] = ((m / RT) ? a.W2 : a.W) + (int64_t)wrow * K + kb;
        }
        const int64_t xb = ((int64_t)ks * 4 * 64 + lane) * 8;
#pragma unroll
        for (int s = 0; s < 4; s++) {
            // aligned K: constant offsets; otherwise clamped into the row
            const int ko = KALIGNED ? s * 32 : min(kb + s * 32, K - 8) - kb;
#pragma unroll
            for (int m = 0; m < NA; m++) st.wa[m][s] = ld16(wq[m] + ko);
#pragma unroll
            for (int t = 0; t < MT; t++) {
                const int64_t xo = xb + ((int64_t)t * nks * 4 + s) * 512;
                st.bh[t][s] = ld16(a.xhi + xo);
                st.bl[t][s] = ld16(a.xlo + xo);
            }
        }
        it_i++;
    };
    auto consume = [&](Stage &st, int it) {
        const int ks = it * KS + wv;
        if (ks >= nks) return;   // a padding step of this wave (uniform branch)
        if constexpr (Q4) {
            const uint4 one4 = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
            const f32x4_t zero = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < 2; h++) {
                // group sums of x for this lane's batch row (the same in all four accumulator rows)
                f32x4_t S[MT];
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(st.bh[t][2 * h]), zero, 0, 0, 0);
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(st.bl[t][2 * h]), S[t], 0, 0, 0);
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(st.bh[t][2 * h + 1]), S[t], 0, 0, 0);
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(st.bl[t][2 * h + 1]), S[t], 0, 0, 0);
                }
#pragma unroll
                for (int m = 0; m < NA; m++) {
                    const uint4 sb = st.wa[m][1 + h];
                    const uint32_t sbw[4] = {sb.x, sb.y, sb.z, sb.w};
                    float sc[4], b2[4];
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        sc[i] = __uint_as_float(sbw[i] << 16);
                        b2[i] = __uint_as_float(sbw[i] & 0xFFFF0000u);
                    }
                    const uint4 a0 = q4_codes_bf16(h ? st.wa[m][0].z : st.wa[m][0].x);
                    const uint4 a1 = q4_codes_bf16(h ? st.wa[m][0].w : st.wa[m][0].y);
#pragma unroll
                    for (int t = 0; t < MT; t++) {
                        f32x4_t D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0), as_bf16x8(st.bh[t][2 * h]), zero, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0), as_bf16x8(st.bl[t][2 * h]), D, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a1), as_bf16x8(st.bh[t][2 * h + 1]), D, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a1), as_bf16x8(st.bl[t][2 * h + 1]), D, 0, 0, 0);
#pragma unroll
                        for (int i = 0; i < 4; i++)
                            acc[m][t][i] = fmaf(sc[i], D[i], fmaf(b2[i], S[t][i], acc[m][t][i]));
                    }
                }
            }
            return;
        }
        if (KALIGNED) {
#pragma unroll
            for (int s = 0; s < 4; s++)
#pragma unroll
                for (int t = 0; t < MT; t++)
#pragma unroll
                    for (int m = 0; m < NA; m++) {
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(st.wa[m][s]), as_bf16x8(st.bh[t][s]), acc[m][t], 0, 0, 0);
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(st.wa[m][s]), as_bf16x8(st.bl[t][s]), acc[m][t], 0, 0, 0);
                    }
        } else {
            const int kb = ks * 128 + lg * 8;
#pragma unroll
            for (int s = 0; s < 4; s++) {
                // past the end of K both operands are zeroed (the padding of the
                // activation buffer is not initialised)
                const bool in = kb + s * 32 < K;
                const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    const uint4 h4 = in ? st.bh[t][s] : z, l4 = in ? st.bl[t][s] : z;
#pragma unroll
                    for (int m = 0; m < NA; m++) {
                        const uint4 w4 = in ? st.wa[m][s] : z;
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w4), as_bf16x8(h4),
                                                                            acc[m][t], 0, 0, 0);
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w4), as_bf16x8(l4),
                                                                            acc[m][t], 0, 0, 0);
                    }
                }
            }
        }
    };

    // Sum-of-squares partials of the input rows: requested before the weight
    // stream starts and added up after it, so their latency is hidden and the
    // main loop never waits for them alone.  Wave wv takes partials wv, wv+KS, ...
    constexpr int SSQ_REGS = 32;
    float sv[SSQ_REGS];
    if (NORM) {
#pragma unroll
        for (int u = 0; u < SSQ_REGS; u++)
            sv[u] = a.ssq_in[(int64_t)min(wv + u * KS, a.n_part - 1) * kSsqStride + min(lane, 16 * MT - 1)];
    }

    // The residual rows and the next norm's gains that the epilogue of wave rt < RT will
    // need: requested ahead of the weight stream as well (clamped addresses; used only
    // where valid), so that the epilogue does not end on a memory round trip.
    float xr[MT][4], gn[4];
    if (EPI == GEPI_RESID) {
        const int rr = ((int)blockIdx.x * RT + min(wv, RT - 1)) * 16 + 4 * lg;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int r = min(rr + i, N - 1);
            gn[i] = bf16_to_f32(a.gain_next[r]);
#pragma unroll
            for (int t = 0; t < MT; t++)
                xr[t][i] = a.xres[(int64_t)min(t * 16 + ln, a.B - 1) * N + r];
        }
    }

    Stage st[PD];
#pragma unroll
    for (int p = 0; p < PD; p++) issue(st[p]);

    {
        for (int it = 0; it + PD < niter2; it += PD) {
#pragma unroll
            for (int p = 0; p < PD; p++) {
                consume(st[p], it + p);
                issue(st[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < PD; p++) consume(st[p], niter2 - PD + p);
        if (NORM) {
            float ss = 0.f;
#pragma unroll
            for (int u = 0; u < SSQ_REGS; u++) ss += (wv + u * KS < a.n_part) ? sv[u] : 0.f;
            for (int p = wv + SSQ_REGS * KS; p < a.n_part; p += KS)   // very wide models only
                ss += a.ssq_in[(int64_t)p * kSsqStride + min(lane, 16 * MT - 1)];
            ssq_s[wv][lane] = ss;
        }
        // K-splits meet in LDS
        RedBuf &rb = red[0];
#pragma unroll
        for (int m = 0; m < NA; m++)
#pragma unroll
            for (int t = 0; t < MT; t++)
#pragma unroll
                for (int i = 0; i < 4; i++) rb[wv][m][t][i][lane] = acc[m][t][i];
        __syncthreads();
        if (wv >= RT) return;

        // Wave rt < RT finishes row tile rt of the group: it adds the K-splits in
        // wave order, then the epilogue.  The lane holds
        // D[row0 + 4*lg + i][n = 16*t + ln], i = 0..3.
        const int rt = wv;
        const int out_tile = (int)blockIdx.x * RT + rt;
        if (out_tile * 16 >= N) return;
        float v[MT][NM][4];
#pragma unroll
        for (int t = 0; t < MT; t++) {
            const int n = t * 16 + ln;
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < KS; w++) s += rb[w][m * RT + rt][t][i][lane];
                    v[t][m][i] = s;
                }
            if (NORM) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < KS; w++) s += ssq_s[w][n];
                const float inv = rsqrtf(s / (float)K + a.eps);
#pragma unroll
                for (int m = 0; m < NM; m++)
#pragma unroll
                    for (int i = 0; i < 4; i++) v[t][m][i] *= inv;
            }
        }
        gemm_tile_epilogue<MT, EPI>(a, out_tile, lane, v, xr, gn);
    }
}

// Dynamic LDS bytes of a skinny_gemm_kernel instance.
template <int MT, int KS, int RT, int EPI>
constexpr size_t skinny_gemm_lds_bytes()
{
    return (size_t)KS * ((EPI == GEPI_SWIGLU) ? 2 : 1) * RT * MT * 4 * 64 * 4 + (size_t)KS * 64 * 4;
}

}  // namespace dk
