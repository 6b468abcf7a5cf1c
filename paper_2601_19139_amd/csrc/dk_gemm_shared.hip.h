// Skinny GEMM whose waves share one activation tile (batches of 17..64 rows).
//
// Same contract and epilogues as skinny_gemm_kernel (dk_gemm.hip.h).  There every wave of a block
// takes other K-steps, so every wave fetches its own activation operands: 8 KB of bf16 hi/lo
// per 128-column step and 16 batch rows, against 4 KB of weights per row tile.  At 16 batch rows
// that is affordable (and that kernel is the faster one); at 32..64 rows the activation traffic
// is 4..8 times the weight stream and bounds the kernel.  Here all W waves of a block walk the SAME
// K-steps and own different row tiles: the block fetches each step's activation tile once,
// 16 bytes per thread, puts it into LDS, and every wave reads its matrix-core operands from
// there.  A wave then carries only weights (and its 16-byte share of the activations) in
// flight, so the software pipeline can be deeper for the same registers, and a tile's sum over
// K is complete in one wave - no reduction across waves.
//
// The price is a barrier per K-step, which couples the waves of a block to its slowest load;
// measured on the 8B / 3B / 0.6B shapes this pays for the lm_head from 17 rows on (2-3.5x) and for
// the large layer matrices from 33 rows on (1.2-1.6x), and loses elsewhere - the host picks.
//
// A matrix with few row tiles would leave compute units idle, so K can be cut into gridDim.y
// slices.  Each block then stores its partial tiles (device-coherent stores: the dies' L2s
// are not coherent with each other), takes a ticket of its row block, and the block that
// arrives last adds the slices in slice order and runs the epilogue: the result does not
// depend on arrival order.
#pragma once
#include "dk_gemm.hip.h"

namespace dk {

// Floats of partial tiles a K-sliced GEMM needs: [slice][matrix][tile][column tile][4][64].
__host__ __device__ inline size_t shared_gemm_part_floats(int N, int slices, int n_mat, int MT)
{
    return (size_t)slices * n_mat * ((N + 15) / 16) * MT * 256;
}

// Dynamic LDS bytes of a shared_gemm_kernel instance.
constexpr size_t shared_gemm_lds_bytes(int MT) { return (size_t)2 * 512 * MT * 16; }

// W waves per block, RT row tiles per wave (GEPI_SWIGLU: of each of the two matrices), PD K-steps
// in flight per wave.  K must be a multiple of 128.  grid = (ceil(tiles / (W*RT)), slices).
// Q4: packed 4-bit weights, evaluated as in skinny_gemm_kernel's Q4 variant (codes through the matrix
// cores, group sums of x from an all-ones operand, scale and bias applied to the fp32 tiles).
template <int MT, int W, int RT, int PD, int EPI, bool NORM, bool Q4 = false>
__global__ __launch_bounds__(W * 64) void shared_gemm_kernel(GemmArgs a)
{
    constexpr int NM = (EPI == GEPI_SWIGLU) ? 2 : 1;
    constexpr int NA = NM * RT;
    constexpr int TPB = W * 64;
    constexpr int PIECES = 512 * MT;          // 16-byte pieces of one step's activation tile (hi and lo)
    static_assert(PIECES % TPB == 0, "every thread fetches the same number of pieces");
    constexpr int PPT = PIECES / TPB;
    extern __shared__ uint4 sm_act_dyn[];   // two slots of one step's activation tile (shared_gemm_lds_bytes)
    uint4 (*sm_act)[PIECES] = reinterpret_cast<uint4 (*)[PIECES]>(sm_act_dyn);
    __shared__ float sm_ssq[W][64];
    __shared__ int sm_last;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const int K = a.K, N = a.N;
    const int nks = K >> 7, n_tiles = (N + 15) >> 4;
    const int S = (int)gridDim.y, y = (int)blockIdx.y;
    const int ks0 = (int)((long long)nks * y / S), ks1 = (int)((long long)nks * (y + 1) / S);
    const int niter = ks1 - ks0;
    const int niter2 = (niter + PD - 1) / PD * PD;
    const int tile0 = ((int)blockIdx.x * W + wv) * RT;

    f32x4_t acc[NA][MT];
#pragma unroll
    for (int m = 0; m < NA; m++)
#pragma unroll
        for (int t = 0; t < MT; t++) acc[m][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Same pipeline discipline as skinny_gemm_kernel: no conditional loads, every wave runs a
    // multiple of PD steps, steps past the slice read clamped addresses and are not used.
    struct Stage {
        uint4 wa[NA][Q4 ? 3 : 4], act[PPT];   // Q4: codes of the whole step, (scale, bias) of its two groups
    };
    int it_i = 0;
    auto issue = [&](Stage &st) {
        const int ks = max(min(ks0 + it_i, ks1 - 1), 0);   // (an empty slice - more slices than steps - reads step 0, unused)
#pragma unroll
        for (int p = 0; p < PPT; p++) {
            const int piece = p * TPB + tid;
            const int t = piece >> 9, lo = (piece >> 8) & 1, idx = piece & 255;
            st.act[p] = ld16((lo ? a.xlo : a.xhi) + (((int64_t)t * nks + ks) * 256 + idx) * 8);
        }
#pragma unroll
        for (int m = 0; m < NA; m++) {
            if constexpr (Q4) {
                const uint8_t *base = reinterpret_cast<const uint8_t *>((m / RT) ? a.W2 : a.W);
                const int tile = min(tile0 + (m % RT), n_tiles - 1);
                const int wrow = min(tile * 16 + ln, N - 1);
                st.wa[m][0] = ld16(base + (int64_t)wrow * (K >> 1) + ks * 64 + lg * 16);
                const uint8_t *sb = base + (int64_t)N * (K >> 1) + (((int64_t)tile * nks + ks) * 4 + lg) * 32;
                st.wa[m][1] = ld16(sb);
                st.wa[m][2] = ld16(sb + 16);
            } else {
                const int wrow = min((tile0 + (m % RT)) * 16 + ln, N - 1);   // rows past the end are clamped
                const uint16_t *wq = ((m / RT) ? a.W2 : a.W) + (int64_t)wrow * K + ks * 128 + lg * 8;
#pragma unroll
                for (int s = 0; s < 4; s++) st.wa[m][s] = ld16(wq + s * 32);
            }
        }
        it_i++;
    };
    auto consume = [&](Stage &st, int it) {
        if (it < 0 || it >= niter) return;   // a padding step (the same for the whole block)
        uint4 *slot = sm_act[it & 1];
#pragma unroll
        for (int p = 0; p < PPT; p++) slot[p * TPB + tid] = st.act[p];
        // one barrier per step is enough with two slots: nobody can write this slot again
        // before every wave has passed the next step's barrier, i.e. has finished reading it
        __syncthreads();
        if constexpr (Q4) {
            const uint4 one4 = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
            const f32x4_t zero = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < 2; h++) {
                uint4 c0[NA], c1[NA];
                float sc[NA][4], bi[NA][4];
#pragma unroll
                for (int m = 0; m < NA; m++) {
                    c0[m] = q4_codes_bf16(h ? st.wa[m][0].z : st.wa[m][0].x);
                    c1[m] = q4_codes_bf16(h ? st.wa[m][0].w : st.wa[m][0].y);
                    const uint4 sb = st.wa[m][1 + h];
                    const uint32_t sbw[4] = {sb.x, sb.y, sb.z, sb.w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        sc[m][i] = __uint_as_float(sbw[i] << 16);
                        bi[m][i] = __uint_as_float(sbw[i] & 0xFFFF0000u);
                    }
                }
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    const uint4 bh0 = slot[t * 512 + (2 * h) * 64 + lane], bl0 = slot[t * 512 + 256 + (2 * h) * 64 + lane];
                    const uint4 bh1 = slot[t * 512 + (2 * h + 1) * 64 + lane], bl1 = slot[t * 512 + 256 + (2 * h + 1) * 64 + lane];
                    // group sums of x for this lane's batch row (the same in all four accumulator rows)
                    f32x4_t S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bh0), zero, 0, 0, 0);
                    S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bl0), S, 0, 0, 0);
                    S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bh1), S, 0, 0, 0);
                    S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(one4), as_bf16x8(bl1), S, 0, 0, 0);
#pragma unroll
                    for (int m = 0; m < NA; m++) {
                        f32x4_t D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(c0[m]), as_bf16x8(bh0), zero, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(c0[m]), as_bf16x8(bl0), D, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(c1[m]), as_bf16x8(bh1), D, 0, 0, 0);
                        D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(c1[m]), as_bf16x8(bl1), D, 0, 0, 0);
#pragma unroll
                        for (int i = 0; i < 4; i++)
                            acc[m][t][i] = fmaf(sc[m][i], D[i], fmaf(bi[m][i], S[i], acc[m][t][i]));
                    }
                }
            }
            return;
        }
#pragma unroll
        for (int s = 0; s < 4; s++)
#pragma unroll
            for (int t = 0; t < MT; t++) {
                const uint4 bh = slot[t * 512 + s * 64 + lane], bl = slot[t * 512 + 256 + s * 64 + lane];
#pragma unroll
                for (int m = 0; m < NA; m++) {
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(st.wa[m][s]), as_bf16x8(bh),
                                                                        acc[m][t], 0, 0, 0);
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(st.wa[m][s]), as_bf16x8(bl),
                                                                        acc[m][t], 0, 0, 0);
                }
            }
    };

    // sum-of-squares partials of the input rows (NORM), requested ahead of the stream:
    // wave wv takes partials wv, wv+W, ...; lane = batch row
    constexpr int SSQ_REGS = 32;
    float sv[SSQ_REGS];
    if (NORM) {
#pragma unroll
        for (int u = 0; u < SSQ_REGS; u++)
            sv[u] = a.ssq_in[(int64_t)min(wv + u * W, a.n_part - 1) * kSsqStride + lane];
    }
    // residual rows and next gains of this wave's tiles (GEPI_RESID)
    float xr[RT][MT][4], gn[RT][4];
    if (EPI == GEPI_RESID) {
#pragma unroll
        for (int r = 0; r < RT; r++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int row = min((tile0 + r) * 16 + 4 * lg + i, N - 1);
                gn[r][i] = bf16_to_f32(a.gain_next[row]);
#pragma unroll
                for (int t = 0; t < MT; t++)
                    xr[r][t][i] = a.xres[(int64_t)min(t * 16 + ln, a.B - 1) * N + row];
            }
    }

    Stage st[PD];
#pragma unroll
    for (int p = 0; p < PD; p++) issue(st[p]);
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
        for (int u = 0; u < SSQ_REGS; u++) ss += (wv + u * W < a.n_part) ? sv[u] : 0.f;
        for (int p = wv + SSQ_REGS * W; p < a.n_part; p += W) ss += a.ssq_in[(int64_t)p * kSsqStride + lane];
        sm_ssq[wv][lane] = ss;
    }

    if (S > 1) {
        // partial tiles out, ticket, and only the last block of this row block goes on
        const size_t slice_floats = (size_t)NM * n_tiles * MT * 256;
#pragma unroll
        for (int m = 0; m < NA; m++) {
            const int tile = tile0 + (m % RT);
            if (tile >= n_tiles) continue;
            float *pp = a.kpart + (size_t)y * slice_floats + ((size_t)(m / RT) * n_tiles + tile) * MT * 256;
#pragma unroll
            for (int t = 0; t < MT; t++)
#pragma unroll
                for (int i = 0; i < 4; i++)
                    __hip_atomic_store(pp + (t * 4 + i) * 64 + lane, acc[m][t][i], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        }
        drain_stores();    // every wave's partial tiles are complete ...
        __syncthreads();   // ... before one thread takes the ticket
        if (tid == 0)
            sm_last = __hip_atomic_fetch_add(&a.ktickets[blockIdx.x], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                      S - 1;
        __syncthreads();
        if (!sm_last) return;
        if (tid == 0) __hip_atomic_store(&a.ktickets[blockIdx.x], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Slices are added in slice order (the result does not depend on who arrived last).  The
        // device-coherent loads of a slice - one per accumulator element - are independent and
        // are all issued before the first is used; the next slice is requested before this one
        // is added, so a round trip is paid per slice, not per element.
        const float *pbase[NA];
#pragma unroll
        for (int m = 0; m < NA; m++) {
            const int tile = min(tile0 + (m % RT), n_tiles - 1);
            pbase[m] = a.kpart + ((size_t)(m / RT) * n_tiles + tile) * MT * 256 + lane;
        }
        auto fetch = [&](int q, f32x4_t (&v)[NA][MT]) {
            const size_t off = (size_t)min(q, S - 1) * slice_floats;
#pragma unroll
            for (int m = 0; m < NA; m++)
#pragma unroll
                for (int t = 0; t < MT; t++)
#pragma unroll
                    for (int i = 0; i < 4; i++)
                        v[m][t][i] = __hip_atomic_load(pbase[m] + off + (t * 4 + i) * 64, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
        };
        f32x4_t cur[NA][MT], nxt[NA][MT];
        fetch(0, cur);
#pragma unroll
        for (int m = 0; m < NA; m++)
#pragma unroll
            for (int t = 0; t < MT; t++) acc[m][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int q = 0; q < S; q++) {
            fetch(q + 1, nxt);       // (past the last slice: the last one again, unused)
#pragma unroll
            for (int m = 0; m < NA; m++)
#pragma unroll
                for (int t = 0; t < MT; t++) {
                    acc[m][t] += cur[m][t];
                    cur[m][t] = nxt[m][t];
                }
        }
    } else {
        __syncthreads();   // sm_ssq
    }

    float inv[MT];
#pragma unroll
    for (int t = 0; t < MT; t++) {
        inv[t] = 1.f;
        if (NORM) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < W; w++) s += sm_ssq[w][t * 16 + ln];
            inv[t] = rsqrtf(s / (float)K + a.eps);
        }
    }
#pragma unroll
    for (int r = 0; r < RT; r++) {
        const int tile = tile0 + r;
        if (tile >= n_tiles) continue;
        float v[MT][NM][4];
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
            for (int m = 0; m < NM; m++)
#pragma unroll
                for (int i = 0; i < 4; i++) v[t][m][i] = acc[m * RT + r][t][i] * inv[t];
        gemm_tile_epilogue<MT, EPI>(a, tile, lane, v, xr[r], gn[r]);
    }
}

}  // namespace dk
