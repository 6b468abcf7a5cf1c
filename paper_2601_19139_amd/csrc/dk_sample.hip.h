// Sampling beyond greedy: temperature, top-k and top-p (nucleus) on the device.
// The paper does not describe its sampler; the definition implemented here (and,
// independently, by the CPU oracle) is:
//
//   s_i = logit_i / T,  p_i = exp(s_i - max s)                    (float32)
//   top-k (0 < k < V):  candidates C = { i : p_i >= the k-th largest p }   (ties all stay)
//   top-p (p < 1):      t* = the largest value with  sum_{i in C, p_i >= t*} p_i >= p * sum_C p,
//                       kept set K = { i in C : p_i >= t* }
//   draw:               r = u * sum_K p;  the first i in K, in ascending index order, whose
//                       running sum exceeds r
//   u = (x0 >> 8) * 2^-24 with (x0,..) = Philox4x32-10(counter = (step_lo, step_hi, row, 0),
//                                                      key = (seed_lo, seed_hi))
//
// A vocabulary of 150 000 entries is too much for one compute unit per row, so a row is
// spread over kSampleBlocks blocks and the work is a short chain of launches of one
// kernel (its `stage` argument says which step).  Thresholds are found by a radix search
// on the bit pattern of the (non-negative) float threshold: count / mass above a
// threshold is monotone, so a pass tries the 15 next-digit candidates at once and settles
// four bits; eight passes settle all of them.  A pass leaves per-block partial totals;
// the next launch adds them in block order (every block does, redundantly) and decides
// the digit.  No atomics and a fixed summation order everywhere: a call is repeatable
// bit for bit.
#pragma once
#include "dk_common.hip.h"

namespace dk {

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3").
__device__ __forceinline__ uint32_t philox4x32_10_first(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                        uint32_t k0, uint32_t k1)
{
    for (int r = 0; r < 10; r++) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

constexpr int kSampleBlocks = 64;    // blocks per row
constexpr int kSampleThreads = 256;

// per-row search state handed from one launch to the next
struct SampleState {
    uint32_t prefix;      // threshold bits settled so far
    float need;           // total the threshold has to reach
    uint32_t floor_bits;  // only weights >= this (the top-k threshold) take part
    uint32_t pad;
};

enum {
    SAMPLE_MAX = 0,       // per-block maximum of logit / T
    SAMPLE_EXP,           // weights p, per-block total
    SAMPLE_PASS,          // settle the previous digit (unless first), partial totals of the next digit's candidates
    SAMPLE_MASS,          // settle the last digit of the top-k search; per-block candidate mass
    SAMPLE_KEEP,          // settle the last digit; per-block kept mass
    SAMPLE_DRAW           // one block per row: the draw
};

struct SampleArgs {
    const float *logits;   // [B][V]
    float *p;              // [B][V] weights
    float *pmax;           // [B][kSampleBlocks]
    float *part_in, *part_out;      // [B][kSampleBlocks][16] partial totals (ping-pong)
    SampleState *st_in, *st_out;    // [B] (ping-pong)
    int *out;              // [B]
    int V, stage;
    int shift;             // SAMPLE_PASS: bit position of the digit whose candidates are totalled
    int first;             // SAMPLE_PASS: no previous digit to settle; start a new search
    int count;             // SAMPLE_PASS: totals are counts (top-k) instead of masses (top-p)
    int settle;            // SAMPLE_MASS / SAMPLE_KEEP: a search precedes, its last digit is settled here
    int need_from_mass;    // SAMPLE_PASS with first: need = top_p * (sum of the blocks' masses in part_in)
    float temperature, top_p;
    int top_k;
    uint32_t seed_lo, seed_hi, step_lo, step_hi;
};

// The digit (0..15) of a finished pass: the largest candidate whose total over all blocks,
// added in block order, still reaches `need`.  Called by every thread of the block.
__device__ __forceinline__ uint32_t settle_digit(const float *part, float need, float *sm /*[16]*/)
{
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid < 15) {
        float t = 0.f;
        for (int g = 0; g < kSampleBlocks; g++) t += part[g * 16 + tid];
        sm[tid] = t;
    }
    __syncthreads();
    uint32_t digit = 0;
#pragma unroll
    for (int d = 0; d < 15; d++)
        if (sm[d] >= need) digit = (uint32_t)(d + 1);     // totals fall as d grows: the last hit is the largest
    return digit;
}

// Sum over the block in a fixed order; every thread gets it.
__device__ __forceinline__ float sample_block_sum(float v, float *sm /*[4]*/)
{
    v = sum64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    return sm[0] + sm[1] + sm[2] + sm[3];
}

__global__ __launch_bounds__(kSampleThreads) void sample_kernel(SampleArgs a)
{
    __shared__ float sm[16];
    __shared__ float red[4 * 15];
    __shared__ float scan[kSampleThreads];
    __shared__ int sm_i[2];
    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, V = a.V;
    const int slice = (V + kSampleBlocks - 1) / kSampleBlocks;
    const int i0 = min(g * slice, V), i1 = min(i0 + slice, V);
    const float *l = a.logits + (int64_t)b * V;
    float *p = a.p + (int64_t)b * V;
    float *part_out = a.part_out + ((int64_t)b * kSampleBlocks + g) * 16;
    const float *part_in = a.part_in + (int64_t)b * kSampleBlocks * 16;

    if (a.stage == SAMPLE_MAX) {
        float mx = -INFINITY;
        for (int i = i0 + tid; i < i1; i += kSampleThreads) mx = fmaxf(mx, l[i] / a.temperature);
        mx = max64(mx);
        if ((tid & 63) == 0) sm[tid >> 6] = mx;
        __syncthreads();
        if (tid == 0) a.pmax[b * kSampleBlocks + g] = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
        return;
    }
    if (a.stage == SAMPLE_EXP) {
        float mx = -INFINITY;
        for (int k = 0; k < kSampleBlocks; k++) mx = fmaxf(mx, a.pmax[b * kSampleBlocks + k]);
        float z = 0.f;
        for (int i = i0 + tid; i < i1; i += kSampleThreads) {
            const float v = expf(l[i] / a.temperature - mx);
            p[i] = v;
            z += v;
        }
        z = sample_block_sum(z, sm);
        if (tid == 0) part_out[0] = z;
        if (g == 0 && tid == 0) a.st_out[b] = SampleState{0u, 0.f, 0u, 0u};
        return;
    }
    if (a.stage == SAMPLE_DRAW) {
        // g == 0 only (grid.x = 1): the block that holds r, then the index inside its slice
        const SampleState st = a.st_in[b];
        const float tau = __uint_as_float(st.prefix);
        if (tid == 0) {
            float total = 0.f;
            for (int k = 0; k < kSampleBlocks; k++) total += part_in[k * 16];
            const uint32_t x0 = philox4x32_10_first(a.step_lo, a.step_hi, (uint32_t)b, 0u, a.seed_lo, a.seed_hi);
            const float r = (float)(x0 >> 8) * (1.0f / 16777216.0f) * total;
            float run = 0.f;
            int owner = -1, last = 0;
            for (int k = 0; k < kSampleBlocks; k++) {
                const float m = part_in[k * 16];
                if (m > 0.f) last = k;
                if (owner < 0 && run + m > r) owner = k;
                if (owner < 0) run += m;
            }
            if (owner < 0) { owner = last; run -= part_in[last * 16]; }   // rounding left r beyond the end
            sm_i[0] = owner;
            sm[0] = run;
            sm[1] = r;
        }
        __syncthreads();
        const int k0 = min(sm_i[0] * slice, V), k1 = min(k0 + slice, V);
        // thread t owns a contiguous piece of the slice; pieces in thread order = index order
        const int piece = (slice + kSampleThreads - 1) / kSampleThreads;
        const int j0 = min(k0 + tid * piece, k1), j1 = min(j0 + piece, k1);
        float mine = 0.f;
        for (int i = j0; i < j1; i++) mine += (p[i] >= tau) ? p[i] : 0.f;
        scan[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            float run = sm[0];
            int owner = -1, last = 0;
            for (int t = 0; t < kSampleThreads; t++) {
                if (scan[t] > 0.f) last = t;
                if (owner < 0 && run + scan[t] > sm[1]) owner = t;
                if (owner < 0) run += scan[t];
            }
            if (owner < 0) { owner = last; run -= scan[last]; }
            sm_i[1] = owner;
            sm[0] = run;
        }
        __syncthreads();
        if (tid == sm_i[1]) {
            float run = sm[0];
            int pick = -1, last = j0;
            for (int i = j0; i < j1; i++)
                if (p[i] >= tau) {
                    last = i;
                    run += p[i];
                    if (run > sm[1]) { pick = i; break; }
                }
            a.out[b] = pick >= 0 ? pick : last;
        }
        return;
    }

    // ---- the threshold searches ------------------------------------------------------------
    SampleState st = a.st_in[b];
    if (a.stage == SAMPLE_PASS && a.first) {
        // a new search: top-k counts every weight; top-p only the candidates of top-k (the
        // settled threshold of the search before, which SAMPLE_MASS left in floor_bits)
        st.prefix = 0;
        if (a.count) {
            st.need = (float)a.top_k;
            st.floor_bits = 0;
        }
        if (a.need_from_mass) {
            float z = 0.f;
            for (int k = 0; k < kSampleBlocks; k++) z += part_in[k * 16];
            st.need = a.top_p * z;
        }
    } else if (a.stage == SAMPLE_PASS || a.settle) {
        // the digit of the pass before (its position: 4 bits above this pass's, or bit 0)
        const int prev_shift = (a.stage == SAMPLE_PASS) ? a.shift + 4 : 0;
        st.prefix |= settle_digit(part_in, st.need, sm) << prev_shift;
    }
    const float floor_t = __uint_as_float(st.floor_bits);

    if (a.stage == SAMPLE_PASS) {
        float acc[15];
#pragma unroll
        for (int d = 0; d < 15; d++) acc[d] = 0.f;
        for (int i = i0 + tid; i < i1; i += kSampleThreads) {
            const float v = p[i];
            const float w = (v >= floor_t) ? (a.count ? 1.f : v) : 0.f;
            const uint32_t bits = __float_as_uint(v);
#pragma unroll
            for (int d = 0; d < 15; d++)
                acc[d] += (bits >= (st.prefix | ((uint32_t)(d + 1) << a.shift))) ? w : 0.f;
        }
#pragma unroll
        for (int d = 0; d < 15; d++) acc[d] = sum64(acc[d]);
        __syncthreads();
        if ((tid & 63) == 0) {
#pragma unroll
            for (int d = 0; d < 15; d++) red[(tid >> 6) * 15 + d] = acc[d];
        }
        __syncthreads();
        if (tid < 15) part_out[tid] = red[tid] + red[15 + tid] + red[30 + tid] + red[45 + tid];
        if (g == 0 && tid == 0) a.st_out[b] = st;
        return;
    }
    if (a.stage == SAMPLE_MASS) {
        // st.prefix is now the top-k threshold: it becomes the floor of what follows
        const float tau_k = __uint_as_float(st.prefix);
        float z = 0.f;
        for (int i = i0 + tid; i < i1; i += kSampleThreads) z += (p[i] >= tau_k) ? p[i] : 0.f;
        z = sample_block_sum(z, sm);
        if (tid == 0) part_out[0] = z;
        if (g == 0 && tid == 0) a.st_out[b] = SampleState{st.prefix, 0.f, st.prefix, 0u};
        return;
    }
    // SAMPLE_KEEP: the final threshold is the larger of the two searches'; kept mass of the
    // slice in index order (thread pieces in thread order)
    const uint32_t tau_bits = max(st.prefix, st.floor_bits);
    const float tau = __uint_as_float(tau_bits);
    {
        const int piece = (slice + kSampleThreads - 1) / kSampleThreads;
        const int j0 = min(i0 + tid * piece, i1), j1 = min(j0 + piece, i1);
        float mine = 0.f;
        for (int i = j0; i < j1; i++) mine += (p[i] >= tau) ? p[i] : 0.f;
        scan[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
            for (int k = 0; k < kSampleThreads; k++) t += scan[k];
            part_out[0] = t;
            if (g == 0) a.st_out[b] = SampleState{tau_bits, 0.f, 0u, 0u};
        }
    }
}

}  // namespace dk
