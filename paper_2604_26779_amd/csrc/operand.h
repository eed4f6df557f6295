// 16-bit helpers and the activation operand layouts shared by the kernels that produce GEMM inputs
// and the GEMM that reads them.
//
// The weights and the cache are bf16 by definition, but rounding every activation to bf16's 8 mantissa
// bits at every projection input accumulates, over 32 layers, to logits errors several times the parity
// tolerance (2e-2 abs + 1e-2 rel against an fp64 oracle).  Two operand formats carry more:
//   XF_HILO  two bf16 numbers per value, x = hi + lo with hi = bf16(x), lo = bf16(x - hi): about 16
//            mantissa bits, two MFMAs per weight fragment (v_mfma_f32_32x32x16_bf16);
//   XF_F16   one fp16 number per value: 11 mantissa bits, one MFMA per fragment
//            (v_mfma_f32_32x32x16_f16, against the weights converted to fp16 once at model creation).
// Which input takes which is decided per projection from a measured error budget: the inputs of the
// attention block (QKV and output projections, queries, probabilities) are the sensitive ones and
// stay hi + lo; the feed-forward projections and the output head, 80 % of the weight bytes, take fp16.
//
// Operand order "xp": [k-step (16 wide)][32-row block][part: hi | lo, or the one fp16][lane 0..63][8 values],
// lane = (row % 32) + 32 * ((k % 16) / 8): exactly what the 32x32x16 MFMAs want as their A operand,
// so the GEMM copies it to LDS and from there to registers without touching it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specv {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2_t;

constexpr int XF_F16 = 1, XF_HILO = 2;      // operand format = number of 16-byte words per (lane, k-step)

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

// two floats -> two fp16 in one 32-bit word (a in the low half), round to nearest even; magnitudes beyond the
// largest finite fp16 saturate instead of becoming infinite
__device__ inline unsigned int pack_f16x2(float a, float b)
{
    a = __builtin_amdgcn_fmed3f(a, -65504.0f, 65504.0f);
    b = __builtin_amdgcn_fmed3f(b, -65504.0f, 65504.0f);
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(f32x2_t{a, b}, f16x2_t));
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

// the same for either format: the word (XF_HILO: the hi word, lo 64 further) holding elements k .. k+7 of row m
template <int XF>
__device__ inline int64_t xp_index_t(int m, int k, int mb_pad)
{
    return (((int64_t)(k >> 4) * mb_pad + (m >> 5)) * XF) * 64 + (m & 31) + 32 * ((k >> 3) & 1);
}

template <int XF>
__device__ inline void xp_store8_t(uint4* xp, int m, int k, int mb_pad, const float* v)
{
    if constexpr (XF == XF_HILO) {
        xp_store8(xp, m, k, mb_pad, v);
    } else {
        xp[xp_index_t<XF_F16>(m, k, mb_pad)] = make_uint4(pack_f16x2(v[0], v[1]), pack_f16x2(v[2], v[3]), pack_f16x2(v[4], v[5]), pack_f16x2(v[6], v[7]));
    }
}

// format chosen at run time (the same for every thread of a launch)
__device__ inline void xp_store8_rt(uint4* xp, int xf, int m, int k, int mb_pad, const float* v)
{
    if (xf == XF_F16) xp_store8_t<XF_F16>(xp, m, k, mb_pad, v);
    else xp_store8(xp, m, k, mb_pad, v);
}

}  // namespace specv
