// Device helpers shared by the decode-step kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dk {

constexpr int kWave = 64;

// ---- bf16 <-> f32 ---------------------------------------------------------
// A 32-bit word holds two bf16: element 2i in the low half, 2i+1 in the high.
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// float32 -> bf16, round to nearest, ties to even (NaN stays a quiet NaN, denormals are kept):
// the gfx950 conversion instruction (v_cvt_pk_bf16_f32), which the compiler emits for a
// float -> __bf16 conversion.  Checked on the device against the integer formula
// (u + 0x7fff + ((u >> 16) & 1)) >> 16 for every upper half-word with the lower halves around
// the tie and a million random patterns: identical bits, NaNs included.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    const __bf16 h = (__bf16)f;
    uint16_t bits;
    __builtin_memcpy(&bits, &h, 2);
    return bits;
}
// two at once: a in the low half-word, b in the high one
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_rne(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    uint32_t bits;
    __builtin_memcpy(&bits, &r, 4);
    return bits;
}

__device__ __forceinline__ void unpack8(const uint4 &w, float (&f)[8])
{
    f[0] = bf16lo(w.x); f[1] = bf16hi(w.x);
    f[2] = bf16lo(w.y); f[3] = bf16hi(w.y);
    f[4] = bf16lo(w.z); f[5] = bf16hi(w.z);
    f[6] = bf16lo(w.w); f[7] = bf16hi(w.w);
}

// ---- cross-lane reductions with DPP ---------------------------------------
// dpp_ctrl encodings: quad_perm = perm bits; 0x140 row_mirror; 0x141
// row_half_mirror; 0x142 row_bcast15; 0x143 row_bcast31.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, true));
}

// Sum over each aligned group of 8 lanes; every lane of the group gets it.
__device__ __forceinline__ float sum8(float v)
{
    v += dpp_f<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);  // mirror within 8
    return v;
}
// Sum over each row of 16 lanes; every lane of the row gets it.
__device__ __forceinline__ float sum16(float v)
{
    v = sum8(v);
    v += dpp_f<0x140>(v);  // mirror within 16
    return v;
}
// Sum over the 64 lanes of the wave; every lane gets it.
__device__ __forceinline__ float sum64(float v)
{
    v = sum16(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}
__device__ __forceinline__ float max64(float v)
{
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

// Waits until every store this wave has issued is complete.  A block that hands partial results
// to "whichever block takes the last ticket" calls this in every storing thread before the barrier
// that precedes the ticket: the barrier alone orders the waves of the block, not their outstanding
// device-coherent stores against another wave's atomic.
__device__ __forceinline__ void drain_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ float4 ldf4(const float *p) { return *reinterpret_cast<const float4 *>(p); }

// Element offset of the first element of a (layer, block, kv, head) tile of
// the KV pool: pool[layer][block][kv][head][slot][dim].
__device__ __forceinline__ int64_t kv_tile_offset(int layer, int num_blocks, int block, int kv,
                                                  int n_kv_heads, int head, int block_size, int d)
{
    return ((((int64_t)layer * num_blocks + block) * 2 + kv) * n_kv_heads + head) *
           (int64_t)(block_size * d);
}

// Layout of an activation matrix X[n][k] that feeds the matrix-core GEMM as
// bf16: stored in the order the MFMA B-operand loads consume it, so that every
// wave load is one contiguous 1 KB run.  For batch tile t = n/16, K-step
// ks = k/128 and MFMA sub-step s = (k%128)/32, lane (lg = (k%32)/8, ln = n%16)
// holds the 8 elements k%8:
//     offset = (((t*nks + ks)*4 + s)*64 + lg*16 + ln)*8 + k%8,  nks = ceil(K/128)
__device__ __forceinline__ int64_t act_offset(int n, int k, int nks)
{
    const int t = n >> 4, ln = n & 15, ks = k >> 7, s = (k >> 5) & 3, lg = (k >> 3) & 3;
    return ((((int64_t)t * nks + ks) * 4 + s) * 64 + lg * 16 + ln) * 8 + (k & 7);
}

}  // namespace dk
