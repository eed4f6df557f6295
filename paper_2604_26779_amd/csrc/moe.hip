// Routed mixture-of-experts feed-forward around the grouped GEMM: routing, the permutation of rows into
// per-expert tiles, the gather of their activations, and the weighted combine fused with the residual
// add and the next RMSNorm.  (The 235B-A22B-class target of the paper's Section 3.1 is of this kind;
// the routing rule is the header's.)
//
// Order of the rows inside an expert's tile list is the order of the (row, rank) pairs, so every buffer
// and every sum is a pure function of the inputs (no atomics on results).
#include "common.h"
#include "operand.h"

namespace specv {

constexpr int MOE_TILE_ROWS = 64;          // rows per grouped-GEMM tile; an expert's rows are padded to this

// One wavefront per row: router logits (summed over the K splits of the router GEMM) -> the top_k most
// probable experts, most probable first, and their probabilities renormalised over the chosen ones
// (the softmax denominator cancels).  E <= 256.
__global__ __launch_bounds__(64) void moe_route_kernel(const float* __restrict__ part, int splits, int64_t split_stride, int E,
                                                        int top_k, int32_t* __restrict__ ids, float* __restrict__ wts)
{
    const int m = blockIdx.x, lane = threadIdx.x;
    float r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int e = lane + 64 * j;
        float v = -INFINITY;
        if (e < E) {
            v = 0.f;
            for (int s = 0; s < splits; ++s) v += part[s * split_stride + (int64_t)m * E + e];
            // a logit that is not finite (overflowed or corrupt router weights) must not poison the row: NaN counts as the
            // lowest finite value, infinities as the largest, so that top_k distinct experts inside [0, E) are always found
            // (-INFINITY is reserved for "taken" and "beyond E") and the weights stay finite with a sum >= 1
            v = v == v ? fminf(fmaxf(v, -3.0e38f), 3.0e38f) : -3.0e38f;
        }
        r[j] = v;
    }
    float mx = fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3]));
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float chosen_p = 0.f, sum = 0.f;
    int chosen_e = -1;
    for (int t = 0; t < top_k; ++t) {
        float best = -INFINITY;
        int be = 1 << 30;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (r[j] > best) { best = r[j]; be = lane + 64 * j; }           // ascending e inside a lane: ties keep the lowest
        for (int off = 32; off > 0; off >>= 1) {
            float b2 = __shfl_xor(best, off);
            int e2 = __shfl_xor(be, off);
            if (b2 > best || (b2 == best && e2 < be)) { best = b2; be = e2; }
        }
        float p = expf(best - mx);
        if (be >= E) { be = t; p = 0.f; }                 // cannot happen with top_k <= E (kept so that an id is never out of range)
        sum += p;
        if (lane == t) { chosen_p = p; chosen_e = be; }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (be == lane + 64 * j) r[j] = -INFINITY;
    }
    if (lane < top_k) {
        ids[(int64_t)m * top_k + lane] = chosen_e;
        wts[(int64_t)m * top_k + lane] = chosen_p / sum;
    }
}

// One workgroup: how many rows every expert received, where its (padded) rows start, and the tile list
// of the grouped GEMM.  row0 [E + 1] (row0[E] = all padded rows); tiles: [0] = count, then (expert, first
// 32-row block) pairs.
__global__ __launch_bounds__(256) void moe_plan_kernel(const int32_t* __restrict__ ids, int n_pairs, int E,
                                                        int32_t* __restrict__ row0, int32_t* __restrict__ tiles)
{
    __shared__ int hist[256];
    hist[threadIdx.x] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < n_pairs; p += 256) {
        int e = ids[p];
        if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int at = 0, nt = 0;
        for (int e = 0; e < E; ++e) {
            row0[e] = at;
            int t = (hist[e] + MOE_TILE_ROWS - 1) / MOE_TILE_ROWS;
            for (int j = 0; j < t; ++j) {
                tiles[1 + 2 * nt] = e;
                tiles[2 + 2 * nt] = (at + j * MOE_TILE_ROWS) / 32;
                ++nt;
            }
            at += t * MOE_TILE_ROWS;
        }
        row0[E] = at;
        tiles[0] = nt;
    }
}

// Workgroup e lists the pairs routed to expert e in pair order: src_row[row] = input row of padded row
// `row` (-1 for padding), pair_row[pair] = padded row that holds the pair.
__global__ __launch_bounds__(256) void moe_permute_kernel(const int32_t* __restrict__ ids, int n_pairs, int top_k,
                                                           const int32_t* __restrict__ row0, int32_t* __restrict__ src_row,
                                                           int32_t* __restrict__ pair_row)
{
    __shared__ int wave_total[4];
    const int e = blockIdx.x, base = row0[e], end = row0[e + 1];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int running = 0;
    for (int p0 = 0; p0 < n_pairs; p0 += 256) {
        int p = p0 + threadIdx.x;
        bool mine = p < n_pairs && ids[p] == e;
        unsigned long long mask = __builtin_amdgcn_ballot_w64(mine);
        int before = __builtin_popcountll(mask & ((1ull << lane) - 1ull));
        __syncthreads();
        if (lane == 0) wave_total[wave] = __builtin_popcountll(mask);
        __syncthreads();
        int off = 0, tot = 0;
        for (int w = 0; w < 4; ++w) { if (w < wave) off += wave_total[w]; tot += wave_total[w]; }
        if (mine) {
            int row = base + running + off + before;
            src_row[row] = p / top_k;
            pair_row[p] = row;
        }
        running += tot;
    }
    for (int row = base + running + threadIdx.x; row < end; row += 256) src_row[row] = -1;
}

// Activations of the permuted rows in the GEMM's operand order (hi and lo words), zeros for padding.
// One thread per 16-byte destination word: writes are contiguous, reads gather rows of one k-step.
// The source is always hi + lo (the router reads it too); with xf_dst = XF_F16 (expert projections that take fp16
// activations, 64 threads per workgroup) a destination word is fp16(hi + lo) of the same eight values.
__device__ inline unsigned int hilo_to_f16x2(unsigned int hi, unsigned int lo)
{
    return pack_f16x2(__uint_as_float(hi << 16) + __uint_as_float(lo << 16), __uint_as_float(hi & 0xffff0000u) + __uint_as_float(lo & 0xffff0000u));
}

__global__ void moe_gather_kernel(const uint4* __restrict__ xp_src, int mb_pad_src, const int32_t* __restrict__ src_row,
                                  const int32_t* __restrict__ row0, int E, int k_steps, int mb_pad_dst, int xf_dst,
                                  uint4* __restrict__ xp_dst)
{
    const int blocks = row0[E] / 32;
    const int mblk = blockIdx.x, ks = blockIdx.y;
    if (mblk >= blocks) return;
    const int part = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = src_row[mblk * 32 + (lane & 31)];
    uint4 v = make_uint4(0, 0, 0, 0);
    if (xf_dst == XF_F16) {
        if (m >= 0) {
            const int64_t at = (((int64_t)ks * mb_pad_src + (m >> 5)) * 2) * 64 + (m & 31) + (lane & 32);
            const uint4 hi = xp_src[at], lo = xp_src[at + 64];
            v = make_uint4(hilo_to_f16x2(hi.x, lo.x), hilo_to_f16x2(hi.y, lo.y), hilo_to_f16x2(hi.z, lo.z), hilo_to_f16x2(hi.w, lo.w));
        }
        xp_dst[((int64_t)ks * mb_pad_dst + mblk) * 64 + lane] = v;
        return;
    }
    if (m >= 0) v = xp_src[(((int64_t)ks * mb_pad_src + (m >> 5)) * 2 + part) * 64 + (m & 31) + (lane & 32)];
    xp_dst[(((int64_t)ks * mb_pad_dst + mblk) * 2 + part) * 64 + lane] = v;
}

// x[m] += sum over the row's experts (in rank order) of weight * expert output; xp = RMSNorm(x[m]) * gain.
// One workgroup per row, 8 elements per thread and pass.
__global__ __launch_bounds__(512) void moe_combine_norm_kernel(float* __restrict__ x, const float* __restrict__ y,
                                                                const int32_t* __restrict__ pair_row, const float* __restrict__ wts,
                                                                int top_k, const unsigned short* __restrict__ gain, int d, float eps,
                                                                int mb_pad, int xf, uint4* __restrict__ xp)
{
    __shared__ float lds16[16];
    __shared__ int s_row[16];
    __shared__ float s_w[16];
    const int m = blockIdx.x;
    if ((int)threadIdx.x < top_k) {
        s_row[threadIdx.x] = pair_row[(int64_t)m * top_k + threadIdx.x];
        s_w[threadIdx.x] = wts[(int64_t)m * top_k + threadIdx.x];
    }
    __syncthreads();
    const int stride = blockDim.x * 8;
    float* xr = x + (int64_t)m * d;
    float ss = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += stride) {
        float4 a = *(const float4*)(xr + c), b = *(const float4*)(xr + c + 4);
        float4 sa = make_float4(0.f, 0.f, 0.f, 0.f), sb = sa;
        for (int t = 0; t < top_k; ++t) {
            const float* ys = y + (int64_t)s_row[t] * d + c;
            float4 p0 = *(const float4*)ys, p1 = *(const float4*)(ys + 4);
            float w = s_w[t];
            sa.x += w * p0.x; sa.y += w * p0.y; sa.z += w * p0.z; sa.w += w * p0.w;
            sb.x += w * p1.x; sb.y += w * p1.y; sb.z += w * p1.z; sb.w += w * p1.w;
        }
        a.x += sa.x; a.y += sa.y; a.z += sa.z; a.w += sa.w;
        b.x += sb.x; b.y += sb.y; b.z += sb.z; b.w += sb.w;
        *(float4*)(xr + c) = a;
        *(float4*)(xr + c + 4) = b;
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) lds16[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += lds16[w];
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x * 8; c < d; c += stride) {
        float4 a = *(const float4*)(xr + c), b = *(const float4*)(xr + c + 4);      // this thread's own writes
        uint4 g = *(const uint4*)(gain + c);
        float v[8] = {a.x * r * from_bf16(g.x & 0xffff), a.y * r * from_bf16(g.x >> 16), a.z * r * from_bf16(g.y & 0xffff),
                      a.w * r * from_bf16(g.y >> 16),    b.x * r * from_bf16(g.z & 0xffff), b.y * r * from_bf16(g.z >> 16),
                      b.z * r * from_bf16(g.w & 0xffff), b.w * r * from_bf16(g.w >> 16)};
        xp_store8_rt(xp, xf, m, c, mb_pad, v);
    }
}

// upper bound of the padded rows for M input rows: every pair, plus one tile's padding per expert
int moe_rows_bound(int M, int top_k, int E)
{
    int64_t rows = (int64_t)M * top_k + (int64_t)E * (MOE_TILE_ROWS - 1);
    return (int)(cdiv(rows, MOE_TILE_ROWS) * MOE_TILE_ROWS);
}

spec_status launch_moe_route(const float* part, int splits, int64_t split_stride, int M, int E, int top_k, int32_t* ids, float* wts,
                             int32_t* row0, int32_t* tiles, int32_t* src_row, int32_t* pair_row, hipStream_t s)
{
    moe_route_kernel<<<M, 64, 0, s>>>(part, splits, split_stride, E, top_k, ids, wts);
    moe_plan_kernel<<<1, 256, 0, s>>>(ids, M * top_k, E, row0, tiles);
    moe_permute_kernel<<<E, 256, 0, s>>>(ids, M * top_k, top_k, row0, src_row, pair_row);
    SPEC_LAUNCH_CHECK("moe routing kernels");
    return SPEC_OK;
}

spec_status launch_moe_gather(const bf16_t* xp_src, int mb_pad_src, const int32_t* src_row, const int32_t* row0, int E, int d,
                              int rows_bound, int xf_dst, bf16_t* xp_dst, hipStream_t s)
{
    dim3 grid((unsigned)(rows_bound / 32), (unsigned)(d / 16));
    moe_gather_kernel<<<grid, xf_dst == XF_F16 ? 64 : 128, 0, s>>>((const uint4*)xp_src, mb_pad_src, src_row, row0, E, d / 16, rows_bound / 32, xf_dst,
                                                                  (uint4*)xp_dst);
    SPEC_LAUNCH_CHECK("moe_gather_kernel");
    return SPEC_OK;
}

spec_status launch_moe_combine_norm(float* x, const float* y, const int32_t* pair_row, const float* wts, int M, int top_k,
                                    const void* gain, int d, float eps, int mb_pad, int xf, bf16_t* xp, hipStream_t s)
{
    moe_combine_norm_kernel<<<M, d >= 4096 ? 512 : 256, 0, s>>>(x, y, pair_row, wts, top_k, (const unsigned short*)gain, d, eps,
                                                               mb_pad, xf, (uint4*)xp);
    SPEC_LAUNCH_CHECK("moe_combine_norm_kernel");
    return SPEC_OK;
}

}  // namespace specv
