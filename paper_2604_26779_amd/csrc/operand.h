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

__device__ inline unsigned short to_bf16(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (unsigned short)((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u));
    u += 0x7fffu + ((u >> 16) & 1u);           // round to nearest even
    return (unsigned short)(u >> 16);
}
__device__ inline float from_bf16(unsigned short h) { return __uint_as_float((unsigned int)h << 16); }

// v[0..7] -> 8 x hi and 8 x lo, each packed into 16 bytes
__device__ inline void split8(const float* v, uint4& hi, uint4& lo)
{
    unsigned short h[8], l[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        h[j] = to_bf16(v[j]);
        l[j] = to_bf16(v[j] - from_bf16(h[j]));
    }
    hi = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    lo = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
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
