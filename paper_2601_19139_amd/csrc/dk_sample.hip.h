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
// spread over kSampleBlocks blocks (slice g of the row belongs to block g).  In general the
// work is a chain of launches of one kernel (its `stage` argument says which step):
// thresholds are found by a radix search on the bit pattern of the (non-negative) float
// threshold - count / mass above a threshold is monotone, so a pass tries the 15 next-digit
// candidates at once and settles four bits; eight passes settle all of them.  A pass leaves
// per-block partial totals; the next launch adds them in block order (every block does,
// redundantly) and decides the digit.  With a small top_k (the usual serving setting) the
// candidates are selected slice by slice instead and a call is three launches (below).
// Float sums have a fixed order everywhere and counts are integers: a call is repeatable
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

// ---- small top_k: candidates by selection instead of a search over the whole row -------------
// With 0 < top_k <= kSampleFastK a call is three launches (maximum; weights and the slices' top k;
// thresholds and draw) instead of up to 21.  The block that computes a slice's weights also selects
// the k-th largest of them (tau_g) and hands on the weights above it (fewer than k values, in index
// order) plus (tau_g, how many equal it): an element of the row's top k is in its slice's top k, so
// the row's k-th largest weight - and every weight at or above it - is among those items, ties
// counted.  One block per row then selects the k-th largest of that multiset (tau_k), gathers the
// candidates (items >= tau_k; a few dozen unless many weights are equal), finds the nucleus
// threshold among them (a candidate per thread adds up the mass at or above its own value; beyond a
// block's worth of candidates, the four-bit search of the general path), adds up each slice's kept
// mass from its items and draws: the slice that holds r by those masses, then the index inside it
// from the weights themselves.  Selections are radix selections on the bit pattern (weights are
// non-negative floats), eight bits per pass through an integer LDS histogram, on items held in
// registers.  Integer counts and fixed summation orders: repeatable bit for bit.
constexpr int kSampleFastK = 64;
constexpr int kSampleSlot = kSampleFastK + 1;                 // a slice's values, then its (tau_g, ties) entry
constexpr int kSampleItems = kSampleBlocks * kSampleSlot;
constexpr int kSampleSliceMax = 4096;                         // weights of a slice staged in LDS

struct SampleSelectArgs {
    const float *logits;   // [B][V]
    float *p;              // [B][V]
    const float *pmax;     // [B][kSampleBlocks]
    float *item_val;       // [B][kSampleItems]
    uint32_t *item_cnt;    // [B][kSampleItems]: how many weights of the row an item stands for (0: unused)
    int *out;              // [B]
    int V, top_k;
    float temperature, top_p;
    uint32_t seed_lo, seed_hi, step_lo, step_hi;
};

// Sum of v over the block (every thread gets it) and, in *before, over the threads below this one.
__device__ __forceinline__ uint32_t sample_block_scan(uint32_t v, uint32_t *sm_w /*[4]*/, uint32_t *before)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)inc, d, 64);
        inc += (lane >= d) ? o : 0u;
    }
    __syncthreads();
    if (lane == 63) sm_w[wave] = inc;
    __syncthreads();
    uint32_t below = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        below += (w < wave) ? sm_w[w] : 0u;
        total += sm_w[w];
    }
    *before = below + inc - v;
    return total;
}

// The k-th largest, counting multiplicities, of the block's items: every thread brings N of them in
// registers, item j with bit pattern bits[j], standing for cnt[j] weights (0: no item).  Returns the bit
// pattern.  Needs k <= the total count.  hist: LDS [256]; sm_u: LDS [2].  Called by all threads of the block.
template <int N>
__device__ __forceinline__ uint32_t sample_select_kth(const uint32_t (&bits)[N], const uint32_t (&cnt)[N], uint32_t k,
                                                      uint32_t *hist, uint32_t *sm_u)
{
    const int tid = threadIdx.x;
    uint32_t prefix = 0, need = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        __syncthreads();
        hist[tid] = 0u;
        if (tid == 0) { sm_u[0] = 0u; sm_u[1] = 0u; }
        __syncthreads();
        const uint32_t mask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
        for (int j = 0; j < N; j++)
            if (cnt[j] && (bits[j] & mask) == prefix) atomicAdd(&hist[(bits[j] >> shift) & 255u], cnt[j]);
        __syncthreads();
        // digits from the top: the first whose count, added to those above it, reaches `need`.  Lane l of
        // the first wave holds digits 4l..4l+3; a suffix sum over the lanes says what is above a lane's.
        if (tid < 64) {
            const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
            const uint32_t own = h0 + h1 + h2 + h3;
            uint32_t inc = own;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t o = (uint32_t)__shfl_down((int)inc, d, 64);
                inc += (tid + d < 64) ? o : 0u;
            }
            const uint32_t over = inc - own;          // counts of the digits above this lane's four
            if (over < need && inc >= need) {         // exactly one lane (the counts reach `need` in all)
                uint32_t run = over;
                int d = 3;
                if (run + h3 >= need) d = 3;
                else if (run + h3 + h2 >= need) { d = 2; run += h3; }
                else if (run + h3 + h2 + h1 >= need) { d = 1; run += h3 + h2; }
                else { d = 0; run += h3 + h2 + h1; }
                sm_u[0] = (uint32_t)(4 * tid + d);
                sm_u[1] = run;
            }
        }
        __syncthreads();
        prefix |= sm_u[0] << shift;
        need -= sm_u[1];
    }
    return prefix;
}

// Inclusive prefix sums over the lanes of a wave, in a fixed order (a doubling scan).
__device__ __forceinline__ float sample_wave_scan(float v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_up(v, d, 64);
        v += (lane >= d) ? o : 0.f;
    }
    return v;
}

// The draw for row b: r = u * (sum of mass[k * stride], k in slice order); the slice that holds r, then
// the index inside it by a running sum of the kept weights (p >= tau) in index order.  Two levels of
// prefix sums (the slices' masses across a wave; inside the slice a contiguous piece per thread, the
// pieces' sums across the block) name the thread whose piece holds r; that thread walks its piece.  Where
// rounding leaves r beyond the last prefix, the last kept weight is taken.  Called by all threads of a
// block; sm: LDS [8], sm_i: LDS [12].
constexpr int kSampleDrawPiece = 16;     // weights of a piece held in registers (slices up to 4096)
__device__ __forceinline__ void sample_draw_row(const float *p, const float *mass, int stride, float tau, int V, int b,
                                                uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo, uint32_t step_hi,
                                                int *out, float *sm, int *sm_i)
{
    static_assert(kSampleBlocks == 64, "one slice per lane of the first wave");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slice = (V + kSampleBlocks - 1) / kSampleBlocks;
    __syncthreads();
    if (wave == 0) {
        const float m = mass[lane * stride];
        const float inc = sample_wave_scan(m);
        const float total = __shfl(inc, 63, 64);
        const uint32_t x0 = philox4x32_10_first(step_lo, step_hi, (uint32_t)b, 0u, seed_lo, seed_hi);
        const float r = (float)(x0 >> 8) * (1.0f / 16777216.0f) * total;
        const uint64_t hit = __ballot(inc > r), any = __ballot(m > 0.f);
        const int owner = hit ? __ffsll((unsigned long long)hit) - 1 : (any ? 63 - __clzll((long long)any) : 0);
        const float before = __shfl(inc - m, owner, 64);
        if (lane == 0) {
            sm_i[0] = owner;
            sm[0] = before;
            sm[1] = r;
        }
    }
    __syncthreads();
    const float r = sm[1];
    const int k0 = min(sm_i[0] * slice, V), k1 = min(k0 + slice, V);
    // thread t owns a contiguous piece of the slice; pieces in thread order = index order
    const int piece = (slice + kSampleThreads - 1) / kSampleThreads;
    const int j0 = min(k0 + tid * piece, k1), j1 = min(j0 + piece, k1);
    const bool in_regs = piece <= kSampleDrawPiece;
    float pv[kSampleDrawPiece];
    uint32_t kept = 0;
    float mine = 0.f;
    if (in_regs) {
        // loads from clamped addresses, all in flight together; what is outside the piece is dropped afterwards
#pragma unroll
        for (int j = 0; j < kSampleDrawPiece; j++) pv[j] = p[min(j0 + j, V - 1)];
#pragma unroll
        for (int j = 0; j < kSampleDrawPiece; j++) {
            const bool k = j0 + j < j1 && pv[j] >= tau;
            kept |= k ? (1u << j) : 0u;
            mine += k ? pv[j] : 0.f;
        }
    } else {
        for (int i = j0; i < j1; i++) mine += (p[i] >= tau) ? p[i] : 0.f;
    }
    const float incw = sample_wave_scan(mine);
    if (lane == 63) sm[4 + wave] = incw;
    __syncthreads();
    float off = sm[0];
    for (int w = 0; w < wave; w++) off += sm[4 + w];
    const float inc = off + incw;
    {
        const uint64_t hit = __ballot(inc > r), any = __ballot(mine > 0.f);
        if (lane == 0) {
            sm_i[2 + wave] = hit ? __ffsll((unsigned long long)hit) - 1 : 64;
            sm_i[6 + wave] = any ? 63 - __clzll((long long)any) : -1;
        }
    }
    __syncthreads();
    int owner_t = -1;
#pragma unroll
    for (int w = 0; w < 4; w++)
        if (owner_t < 0 && sm_i[2 + w] < 64) owner_t = w * 64 + sm_i[2 + w];
    if (owner_t < 0) {
#pragma unroll
        for (int w = 0; w < 4; w++)
            if (sm_i[6 + w] >= 0) owner_t = w * 64 + sm_i[6 + w];     // the last piece that keeps anything
    }
    if (owner_t < 0) owner_t = 0;
    if (tid == owner_t) {
        float run = inc - mine;
        int pick = -1, last = j0;
        if (in_regs) {
#pragma unroll
            for (int j = 0; j < kSampleDrawPiece; j++)
                if (kept & (1u << j)) {
                    last = j0 + j;
                    run += pv[j];
                    if (pick < 0 && run > r) pick = j0 + j;
                }
        } else {
            for (int i = j0; i < j1; i++)
                if (p[i] >= tau) {
                    last = i;
                    run += p[i];
                    if (run > r) { pick = i; break; }
                }
        }
        out[b] = pick >= 0 ? pick : last;
    }
}

// grid (kSampleBlocks, B): the slice's weights and its top k.  Needs a slice of at most kSampleSliceMax.
__global__ __launch_bounds__(kSampleThreads) void sample_exp_topk_kernel(SampleSelectArgs a)
{
    constexpr int N = kSampleSliceMax / kSampleThreads;
    __shared__ float sl[kSampleSliceMax];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sm_u[2];
    __shared__ uint32_t sm_w[4];
    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, V = a.V;
    const int slice = (V + kSampleBlocks - 1) / kSampleBlocks;
    const int i0 = min(g * slice, V), i1 = min(i0 + slice, V), n = i1 - i0;
    float *val = a.item_val + ((int64_t)b * kSampleBlocks + g) * kSampleSlot;
    uint32_t *cnt = a.item_cnt + ((int64_t)b * kSampleBlocks + g) * kSampleSlot;
    if (n <= 0) {     // a slice beyond the end of a short row
        for (int i = tid; i < kSampleSlot; i += kSampleThreads) {
            val[i] = 0.f;
            cnt[i] = 0u;
        }
        return;
    }
    const float *l = a.logits + (int64_t)b * V + i0;
    float *p = a.p + (int64_t)b * V + i0;
    const float mx = max64(a.pmax[b * kSampleBlocks + (tid & 63)]);
    // the weights: element tid + 256 j in register j (loads from clamped addresses, all in flight together)
    float x[N];
    uint32_t bits[N], one[N];
#pragma unroll
    for (int j = 0; j < N; j++) x[j] = l[min(tid + kSampleThreads * j, n - 1)];
#pragma unroll
    for (int j = 0; j < N; j++) {
        const int i = tid + kSampleThreads * j;
        const float v = expf(x[j] / a.temperature - mx);
        bits[j] = __float_as_uint(v);
        one[j] = i < n ? 1u : 0u;
        if (i < n) {
            p[i] = v;
            sl[i] = v;
        }
    }
    // a slice with fewer than k weights hands on all of them ("the k-th largest" is below everything)
    const bool all = n < a.top_k;
    uint32_t tau = 0;
    if (!all) tau = sample_select_kth(bits, one, (uint32_t)a.top_k, hist, sm_u);
    else __syncthreads();
    // the weights above tau in index order: thread t owns a contiguous piece of the slice
    const int piece = (n + kSampleThreads - 1) / kSampleThreads;
    const int j0 = min(tid * piece, n), j1 = min(j0 + piece, n);
    uint32_t above = 0, mine = 0;     // bit j: element j0 + j is listed; counts: listed | equal to tau << 16
#pragma unroll
    for (int j = 0; j < N; j++) {
        x[j] = sl[min(j0 + j, n - 1)];
        const uint32_t w = __float_as_uint(x[j]);
        const bool in = j0 + j < j1;
        const bool up = in && (all || w > tau);
        above |= up ? (1u << j) : 0u;
        mine += (up ? 1u : 0u) + ((in && !all && w == tau) ? 0x10000u : 0u);
    }
    uint32_t pos;
    const uint32_t total = sample_block_scan(mine, sm_w, &pos);
    const uint32_t listed = total & 0xffffu, ties = total >> 16;        // listed < k by construction
    pos &= 0xffffu;
#pragma unroll
    for (int j = 0; j < N; j++)
        if ((above >> j) & 1u) {
            if (pos < (uint32_t)kSampleFastK) {
                val[pos] = x[j];
                cnt[pos] = 1u;
            }
            pos++;
        }
    for (uint32_t i = listed + tid; i < (uint32_t)kSampleFastK; i += kSampleThreads) {
        val[i] = 0.f;
        cnt[i] = 0u;
    }
    if (tid == 0) {
        val[kSampleFastK] = __uint_as_float(tau);
        cnt[kSampleFastK] = ties;
    }
}

// Largest value of v over the block; every thread gets it.
__device__ __forceinline__ uint32_t sample_block_max(uint32_t v, uint32_t *sm_w /*[4]*/)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, d, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm_w[threadIdx.x >> 6] = v;
    __syncthreads();
    return max(max(sm_w[0], sm_w[1]), max(sm_w[2], sm_w[3]));
}

// grid (1, B): both thresholds from the slices' items, the slices' kept masses, the draw
__global__ __launch_bounds__(kSampleThreads) void sample_merge_draw_kernel(SampleSelectArgs a)
{
    __shared__ float val[kSampleItems];      // items; from the gathering on: the candidates' values
    __shared__ uint32_t cnt[kSampleItems];   // how many weights an item stands for; then: float value x count
    __shared__ uint32_t hist[256];
    __shared__ uint32_t per_slice[kSampleBlocks];
    __shared__ float mass[kSampleBlocks];
    __shared__ uint32_t sm_u[2];
    __shared__ uint32_t sm_w[4];
    __shared__ float sm[8];
    __shared__ int sm_i[12];
    __shared__ float red[4 * 15];
    const int b = blockIdx.y, tid = threadIdx.x;
    constexpr int PIECE = (kSampleItems + kSampleThreads - 1) / kSampleThreads;
    // the items into LDS (loads from clamped addresses, all in flight together), then a contiguous piece of
    // them - item order: slice by slice, index order inside a slice, its ties entry last - into registers
    {
        float lv[PIECE];
        uint32_t lc[PIECE];
#pragma unroll
        for (int j = 0; j < PIECE; j++) {
            const int i = min(tid + kSampleThreads * j, kSampleItems - 1);
            lv[j] = a.item_val[(int64_t)b * kSampleItems + i];
            lc[j] = a.item_cnt[(int64_t)b * kSampleItems + i];
        }
#pragma unroll
        for (int j = 0; j < PIECE; j++)
            if (tid + kSampleThreads * j < kSampleItems) {
                val[tid + kSampleThreads * j] = lv[j];
                cnt[tid + kSampleThreads * j] = lc[j];
            }
    }
    if (tid < kSampleBlocks) per_slice[tid] = 0u;
    __syncthreads();
    float pv[PIECE];
    uint32_t pb[PIECE], pc[PIECE];
#pragma unroll
    for (int j = 0; j < PIECE; j++) {
        const int i = min(tid * PIECE + j, kSampleItems - 1);
        pv[j] = val[i];
        pb[j] = __float_as_uint(pv[j]);
        pc[j] = tid * PIECE + j < kSampleItems ? cnt[i] : 0u;
    }
    const uint32_t tau_k = sample_select_kth(pb, pc, (uint32_t)a.top_k, hist, sm_u);
    const float tau_kf = __uint_as_float(tau_k);
    // gather the candidates (items at or above tau_k) in item order
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < PIECE; j++) {
        pc[j] = pv[j] >= tau_kf ? pc[j] : 0u;
        mine += pc[j] ? 1u : 0u;
    }
    uint32_t pos;
    const int nc = (int)sample_block_scan(mine, sm_w, &pos);     // its barriers separate the reads from the writes
    float *wgt = reinterpret_cast<float *>(cnt);
#pragma unroll
    for (int j = 0; j < PIECE; j++)
        if (pc[j]) {
            val[pos] = pv[j];
            wgt[pos] = pv[j] * (float)pc[j];
            atomicAdd(&per_slice[(tid * PIECE + j) / kSampleSlot], 1u);
            pos++;
        }
    __syncthreads();
    uint32_t tau = tau_k;
    if (a.top_p < 1.f && nc <= kSampleThreads) {
        // a candidate per thread: the mass at or above its value, every thread adding in candidate order; the
        // nucleus threshold is the largest value whose mass reaches top_p of the total
        const float vi = tid < nc ? val[tid] : INFINITY;
        float z = 0.f, ge = 0.f;
        for (int j = 0; j < nc; j++) {
            const float w = wgt[j];
            z += w;
            ge += (val[j] >= vi) ? w : 0.f;
        }
        tau = max(tau_k, sample_block_max((tid < nc && ge >= a.top_p * z) ? __float_as_uint(vi) : 0u, sm_w));
    } else if (a.top_p < 1.f) {
        // many equal weights: the search of the general path (four bits per pass; the 15 candidates of a digit
        // in registers, added over the block in a fixed order) on the candidates' values
        float z = 0.f;
        for (int i = tid; i < nc; i += kSampleThreads) z += wgt[i];
        z = sample_block_sum(z, sm);
        const float need = a.top_p * z;
        uint32_t prefix = 0;
        for (int shift = 28; shift >= 0; shift -= 4) {
            float acc[15];
#pragma unroll
            for (int d = 0; d < 15; d++) acc[d] = 0.f;
            for (int i = tid; i < nc; i += kSampleThreads) {
                const float w = wgt[i];
                const uint32_t bits = __float_as_uint(val[i]);
#pragma unroll
                for (int d = 0; d < 15; d++) acc[d] += (bits >= (prefix | ((uint32_t)(d + 1) << shift))) ? w : 0.f;
            }
#pragma unroll
            for (int d = 0; d < 15; d++) acc[d] = sum64(acc[d]);
            __syncthreads();
            if ((tid & 63) == 0) {
#pragma unroll
                for (int d = 0; d < 15; d++) red[(tid >> 6) * 15 + d] = acc[d];
            }
            __syncthreads();
            uint32_t digit = 0;
#pragma unroll
            for (int d = 0; d < 15; d++)
                if (red[d] + red[15 + d] + red[30 + d] + red[45 + d] >= need) digit = (uint32_t)(d + 1);
            prefix |= digit << shift;
        }
        tau = max(tau_k, prefix);
    }
    const float tau_f = __uint_as_float(tau);
    // every slice's kept mass from its candidates (the gathering kept a slice's together and in order)
    if (tid < kSampleBlocks) {
        const uint32_t c = per_slice[tid];
        uint32_t inc = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)inc, d, 64);
            inc += (tid >= d) ? o : 0u;
        }
        float m = 0.f;
        for (uint32_t i = inc - c; i < inc; i++) m += (val[i] >= tau_f) ? wgt[i] : 0.f;
        mass[tid] = m;
    }
    sample_draw_row(a.p + (int64_t)b * a.V, mass, 1, tau_f, a.V, b, a.seed_lo, a.seed_hi, a.step_lo, a.step_hi, a.out, sm,
                    sm_i);
}

__global__ __launch_bounds__(kSampleThreads) void sample_kernel(SampleArgs a)
{
    __shared__ float sm[16];
    __shared__ float red[4 * 15];
    __shared__ float scan[kSampleThreads];
    __shared__ int sm_i[12];
    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, V = a.V;
    const int slice = (V + kSampleBlocks - 1) / kSampleBlocks;
    const int i0 = min(g * slice, V), i1 = min(i0 + slice, V);
    const float *l = a.logits + (int64_t)b * V;
    float *p = a.p + (int64_t)b * V;
    float *part_out = a.part_out + ((int64_t)b * kSampleBlocks + g) * 16;
    const float *part_in = a.part_in + (int64_t)b * kSampleBlocks * 16;

    if (a.stage == SAMPLE_MAX) {
        // four loads in flight; an address past the slice is clamped (a value twice does not change a maximum)
        float mx = -INFINITY;
        for (int i = i0 + tid; i < i1; i += 4 * kSampleThreads) {
            const float x0 = l[i], x1 = l[min(i + kSampleThreads, i1 - 1)], x2 = l[min(i + 2 * kSampleThreads, i1 - 1)],
                        x3 = l[min(i + 3 * kSampleThreads, i1 - 1)];
            mx = fmaxf(fmaxf(fmaxf(mx, x0 / a.temperature), fmaxf(x1 / a.temperature, x2 / a.temperature)), x3 / a.temperature);
        }
        mx = max64(mx);
        if ((tid & 63) == 0) sm[tid >> 6] = mx;
        __syncthreads();
        if (tid == 0) a.pmax[b * kSampleBlocks + g] = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
        return;
    }
    if (a.stage == SAMPLE_EXP) {
        const float mx = max64(a.pmax[b * kSampleBlocks + (tid & 63)]);
        float z = 0.f;
        for (int i = i0 + tid; i < i1; i += 4 * kSampleThreads) {     // four loads in flight
            float x[4];
#pragma unroll
            for (int j = 0; j < 4; j++) x[j] = l[min(i + j * kSampleThreads, i1 - 1)];
#pragma unroll
            for (int j = 0; j < 4; j++)
                if (i + j * kSampleThreads < i1) {
                    const float v = expf(x[j] / a.temperature - mx);
                    p[i + j * kSampleThreads] = v;
                    z += v;
                }
        }
        z = sample_block_sum(z, sm);
        if (tid == 0) part_out[0] = z;
        if (g == 0 && tid == 0) a.st_out[b] = SampleState{0u, 0.f, 0u, 0u};
        return;
    }
    if (a.stage == SAMPLE_DRAW) {
        // g == 0 only (grid.x = 1)
        sample_draw_row(p, part_in, 16, __uint_as_float(a.st_in[b].prefix), V, b, a.seed_lo, a.seed_hi, a.step_lo,
                        a.step_hi, a.out, sm, sm_i);
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
