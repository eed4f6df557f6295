// bf16 helpers and the activation operand layout shared by the kernels that produce GEMM inputs
// and the GEMM that reads them.
//
// Activations are carried as TWO bf16 numbers per value, x = hi + lo with hi = bf16(x) and
// lo = bf16(x - hi): about 16 mantissa bits.  The weights and the cache are bf16 by definition,
// but rounding every activation to 8 mantissa bits at every projection input accumulates, over
// 32 layers, to logits errors several times the parity tolerance (2e-2 abs + 1e-2 rel against an
// fp64 oracle).  The second MFMA per fragment is free where the GEMM is bound by the weight
// stream from HBM.
//
// Operand order "xp": [k-step (16 wide)][32-row block][hi | lo][lane 0..63][8 bf16], lane =
// (row % 32) + 32 * ((k % 16) / 8): exactly what v_mfma_f32_32x32x16_bf16 wants as its A operand,
// so the GEMM copies it to LDS and from there to registers without touching it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specv {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;

// two floats -> two bf16 in one 32-bit word (a in the low half); round to nearest even in hardware
// (v_cvt_pk_bf16_f32 on gfx950)
__device__ inline unsigned int pack_bf16x2(float a, float b)
{
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
// fp32 -> OCP E4M3 code (1-4-3 bits, bias 7, no infinities, largest magnitude 448 = 0x7e): round to nearest even,
// saturating; NaN is not handled (it saturates).
__device__ inline unsigned int to_e4m3(float x)
{
    const unsigned int u = __float_as_uint(x), sign = (u >> 24) & 0x80u, au = u & 0x7fffffffu;
    const float a = __uint_as_float(au);
    if (!(a < 448.0f)) return sign | 0x7eu;
    if (a < 0.015625f) return sign | (unsigned int)__float2int_rn(a * 512.0f);      // zero, subnormals (steps of 2^-9), up to 2^-6 itself
    const unsigned int r = (au + 0x7ffffu + ((au >> 20) & 1u)) >> 20;                // keep 3 mantissa bits, ties to even
    return sign | (r - ((127u - 7u) << 3));
}

__device__ inline unsigned short to_bf16(float f) { return (unsigned short)(pack_bf16x2(f, 0.f) & 0xffffu); }
__device__ inline float from_bf16(unsigned short h) { return __uint_as_float((unsigned int)h << 16); }

// (a, b) -> hi word and lo word: x = hi + lo with hi = bf16(x), lo = bf16(x - hi)
__device__ inline void split2(float a, float b, unsigned int& hi, unsigned int& lo)
{
    hi = pack_bf16x2(a, b);
    lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

// v[0..7] -> 8 x hi and 8 x lo, each packed into 16 bytes
__device__ inline void split8(const float* v, uint4& hi, uint4& lo)
{
    split2(v[0], v[1], hi.x, lo.x);
    split2(v[2], v[3], hi.y, lo.y);
    split2(v[4], v[5], hi.z, lo.z);
    split2(v[6], v[7], hi.w, lo.w);
}

// index (in 16-byte words) of the hi operand holding elements k .. k+7 (k % 8 == 0) of row m;
// the lo operand sits 64 words further
__device__ inline int64_t xp_index(int m, int k, int mb_pad)
{
    return (((int64_t)(k >> 4) * mb_pad + (m >> 5)) * 2) * 64 + (m & 31) + 32 * ((k >> 3) & 1);
}

__device__ inline void xp_store8(uint4* xp, int m, int k, int mb_pad, const float* v)
{
    uint4 hi, lo;
    split8(v, hi, lo);
    int64_t at = xp_index(m, k, mb_pad);
    xp[at] = hi;
    xp[at + 64] = lo;
}

}  // namespace specv
