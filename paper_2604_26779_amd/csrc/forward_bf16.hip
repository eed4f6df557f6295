// bf16 verify forward: orchestration and the small kernels between the GEMMs and the attention.
//
// Per layer (residual stream x in fp32; every GEMM input in operand order "xp", as hi + lo bf16 pairs or as one fp16
// value, whichever its matrix was tiled for, see operand.h):
//   xp_h  = RMSNorm(x) * g                         (fused into the kernel that last touched x)
//   part  = xp_h W_qkv^T                           gemm, split-K slices
//   q, K, V = rotary(sum part)                     qkv_rope_kernel: q -> bf16 rows, K/V -> paged cache
//   xp_a  = attention(q, cache)                    attn_bf16.hip
//   part  = xp_a W_o^T ; x += sum part ; xp_h = RMSNorm(x) * g2        residual_rmsnorm_kernel
//   part  = xp_h [W_g; W_u]^T ; xp_f = silu(gate) * up                  swiglu_pack_kernel
//   part  = xp_f W_d^T ; x += sum part ; xp_h = RMSNorm(x) * g_next     residual_rmsnorm_kernel
//   (gate/up normally ends in the fused SwiGLU epilogue of the GEMM instead of swiglu_pack_kernel)
// logits = xp_h W_head^T (fp32, written in place by the GEMM).
// Around that: a draft model's input fusion (fuse_input_kernel; with multi-layer features pack_rows_kernel and the
// w_fc GEMM before it), the hidden-state and feature outputs (a copy of x after the last layer, tap_copy_kernel after
// the tapped ones), and the mixture-of-experts feed-forward (moe.hip) in place of the dense one.
#include <algorithm>

#include "common.h"
#include "operand.h"

namespace specv {

// from gemm_bf16.hip / attn_bf16.hip
int gemm_mb_pad(int M);
int gemm_pick_splits(const PackedW& W, int M, int forced);
spec_status launch_gemm_bf16(const PackedW& W, const bf16_t* Xp, int M, float* out, int ldo, int splits, bool swiglu, hipStream_t s);
bool gemm_can_fuse_swiglu(const PackedW& W, int M, int splits);
int attn_max_items(int R, int B, int Hkv, int pages_bound);
size_t attn_item_bytes();
int attn_rows_padded(int R);
spec_status launch_attention_plan(int B, int T, int G, int Hkv, const KvView& kv, int pages_bound, void* items, void* entry_items, hipStream_t s);
int moe_rows_bound(int M, int top_k, int E);
spec_status launch_gemm_bf16_grouped(const PackedW& W0, int64_t group_stride, const bf16_t* Xp, int rows_pad, int max_tiles,
                                     const int32_t* tiles, float* out, int ldo, bool swiglu, hipStream_t s);
spec_status launch_moe_route(const float* part, int splits, int64_t split_stride, int M, int E, int top_k, int32_t* ids, float* wts,
                             int32_t* row0, int32_t* tiles, int32_t* src_row, int32_t* pair_row, hipStream_t s);
spec_status launch_moe_gather(const bf16_t* xp_src, int mb_pad_src, const int32_t* src_row, const int32_t* row0, int E, int d,
                              int rows_bound, int xf_dst, bf16_t* xp_dst, hipStream_t s);
spec_status launch_moe_combine_norm(float* x, const float* y, const int32_t* pair_row, const float* wts, int M, int top_k,
                                    const void* gain, int d, float eps, int mb_pad, int xf, bf16_t* xp, hipStream_t s);
spec_status launch_attention_bf16(const float* q, int B, int T, int G, int Hq, int Hkv, const KvView& kv, int layer_pool, int layer,
                                  int pages_bound, const void* items, const void* entry_items, float* part_o, float* part_ml,
                                  int mb_pad, int xf_out, bf16_t* xp_out, hipStream_t s);

// sum over the workgroup (blockDim.x a multiple of 64, at most 1024)
__device__ inline float block_sum(float v, float* lds16)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds16[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += lds16[w];
    return t;
}

// x[m] = embed[token] (RES_EMBED), x[m] + sum_s part[s][m] (RES_ADD) or sum_s part[s][m] (RES_SET);  xp = RMSNorm(x[m]) * gain
// one workgroup per row (256 or 512 threads, 8 elements per thread and pass); d % 8 == 0
constexpr int RES_ADD = 0, RES_EMBED = 1, RES_SET = 2;
template <int MODE>
__global__ __launch_bounds__(512) void residual_rmsnorm_kernel(
    float* __restrict__ x, const float* __restrict__ part, int splits, int64_t split_stride, const int32_t* __restrict__ tokens,
    const unsigned short* __restrict__ embed, int vocab, const unsigned short* __restrict__ gain, int d, float eps, int mb_pad,
    int xf, uint4* __restrict__ xp)
{
    __shared__ float lds16[16];
    const int m = blockIdx.x;
    const int stride = blockDim.x * 8;
    float* xr = x + (int64_t)m * d;
    float ss = 0.f;
    int tok = 0;
    constexpr bool FIRST = MODE == RES_EMBED;
    if (FIRST) { tok = tokens[m]; tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok); }
    for (int c = threadIdx.x * 8; c < d; c += stride) {
        float v[8];
        if (FIRST) {
            uint4 e = *(const uint4*)(embed + (int64_t)tok * d + c);
            unsigned int w[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[2 * j] = from_bf16(w[j] & 0xffff); v[2 * j + 1] = from_bf16(w[j] >> 16); }
        } else {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (MODE == RES_ADD) { a = *(const float4*)(xr + c); b = *(const float4*)(xr + c + 4); }
            // the slices are summed in order, but loaded eight (then four) at a time: left as a plain loop the compiler
            // waits for each slice before it asks for the next, one trip to memory per slice
            const float* p_row = part + (int64_t)m * d + c;
            int s = 0;
            auto add_group = [&](auto n_c) {
                constexpr int GN = decltype(n_c)::value;
                float4 p0[GN], p1[GN];
#pragma unroll
                for (int u = 0; u < GN; ++u) {
                    const float* ps = p_row + (s + u) * split_stride;
                    p0[u] = *(const float4*)ps;
                    p1[u] = *(const float4*)(ps + 4);
                }
#pragma unroll
                for (int u = 0; u < GN; ++u) {
                    a.x += p0[u].x; a.y += p0[u].y; a.z += p0[u].z; a.w += p0[u].w;
                    b.x += p1[u].x; b.y += p1[u].y; b.z += p1[u].z; b.w += p1[u].w;
                }
                s += GN;
            };
            while (s + 8 <= splits) add_group(std::integral_constant<int, 8>{});
            if (s + 4 <= splits) add_group(std::integral_constant<int, 4>{});
            if (s + 2 <= splits) add_group(std::integral_constant<int, 2>{});
            if (s < splits) add_group(std::integral_constant<int, 1>{});
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        }
        *(float4*)(xr + c) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(xr + c + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
    }
    float tot = block_sum(ss, lds16);
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

// Input of a draft model that also takes hidden states: the operand of the fusion projection,
// [RMSNorm(embed[token]) * g_e ; RMSNorm(hidden_in[m]) * g_h] (2d channels), as hi + lo bf16.  One workgroup per row.
// hidden_in may come as h_splits partial sums h_split_stride floats apart (the K-split output of the feature projection).
__global__ __launch_bounds__(512) void fuse_input_kernel(
    const int32_t* __restrict__ tokens, const unsigned short* __restrict__ embed, int vocab, const float* __restrict__ hidden_in,
    int h_splits, int64_t h_split_stride,
    const unsigned short* __restrict__ gain_e, const unsigned short* __restrict__ gain_h, int d, float eps, int mb_pad,
    uint4* __restrict__ xp)
{
    __shared__ float lds16[16];
    const int m = blockIdx.x;
    const int stride = blockDim.x * 8;
    int tok = tokens[m];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const unsigned short* er = embed + (int64_t)tok * d;
    const float* hr = hidden_in + (int64_t)m * d;
    float ss_e = 0.f, ss_h = 0.f;
    for (int c = threadIdx.x * 8; c < d; c += stride) {
        uint4 e = *(const uint4*)(er + c);
        unsigned int w[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) { float lo = from_bf16(w[j] & 0xffff), hi = from_bf16(w[j] >> 16); ss_e += lo * lo + hi * hi; }
        float4 a = *(const float4*)(hr + c), b = *(const float4*)(hr + c + 4);
        for (int sp = 1; sp < h_splits; ++sp) {
            float4 a2 = *(const float4*)(hr + sp * h_split_stride + c), b2 = *(const float4*)(hr + sp * h_split_stride + c + 4);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
        }
        ss_h += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
    }
    const float re = 1.0f / sqrtf(block_sum(ss_e, lds16) / (float)d + eps);
    const float rh = 1.0f / sqrtf(block_sum(ss_h, lds16) / (float)d + eps);
    for (int c = threadIdx.x * 8; c < d; c += stride) {
        uint4 e = *(const uint4*)(er + c), ge = *(const uint4*)(gain_e + c), gh = *(const uint4*)(gain_h + c);
        unsigned int w[4] = {e.x, e.y, e.z, e.w}, g1[4] = {ge.x, ge.y, ge.z, ge.w}, g2[4] = {gh.x, gh.y, gh.z, gh.w};
        float4 a = *(const float4*)(hr + c), b = *(const float4*)(hr + c + 4);
        for (int sp = 1; sp < h_splits; ++sp) {               // the same sums, in the same order, as in the first sweep
            float4 a2 = *(const float4*)(hr + sp * h_split_stride + c), b2 = *(const float4*)(hr + sp * h_split_stride + c + 4);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
        }
        float hv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        float ve[8], vh[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ve[2 * j] = from_bf16(w[j] & 0xffff) * re * from_bf16(g1[j] & 0xffff);
            ve[2 * j + 1] = from_bf16(w[j] >> 16) * re * from_bf16(g1[j] >> 16);
            vh[2 * j] = hv[2 * j] * rh * from_bf16(g2[j] & 0xffff);
            vh[2 * j + 1] = hv[2 * j + 1] * rh * from_bf16(g2[j] >> 16);
        }
        xp_store8(xp, m, c, mb_pad, ve);
        xp_store8(xp, m, d + c, mb_pad, vh);
    }
}

// Once per forward pass, per input row: cos/sin of pos * theta^(-2j/dh) in fp64 (the angle reaches thousands of radians),
// and where the row's key and value go: row_slot[m] = page * SPEC_PAGE_SIZE + position in the page, or -1 (the batch entry
// was dropped, or its sequence holds no page for that position).  The per-layer kernels then need no walk through the
// bookkeeping (batch entry -> sequence -> length -> page list), three dependent loads each.
__global__ void rope_table_kernel(int M, int T, KvView kv, int half, double theta, float2* __restrict__ table,
                                  int32_t* __restrict__ row_slot)
{
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * half) return;
    int m = idx / half, j = idx % half;
    const int seq = kv.entry_seq[m / T];
    const int pos = seq >= 0 ? kv.ctx_len[seq] + m % T : 0;
    double ang = (double)pos * pow(theta, -2.0 * (double)j / (double)(2 * half));
    table[idx] = make_float2((float)cos(ang), (float)sin(ang));
    if (j == 0) {
        int slot = -1;
        if (seq >= 0) {
            const int lp = pos / SPEC_PAGE_SIZE;
            if (lp < kv.n_held[seq]) slot = kv.page_table[(int64_t)seq * kv.max_pages + lp] * SPEC_PAGE_SIZE + pos % SPEC_PAGE_SIZE;
        }
        row_slot[m] = slot;
    }
}

// sums the split-K slices of the QKV projection, rotates q and k, writes q as bf16 rows and the
// new k, v into their cache slots (speculatively: positions ctx .. ctx+k).  One workgroup per row.
// KV8: the cache holds E4M3 codes of x / scale, one scale per (layer, kv head) for keys and one for values.
template <bool KV8>
__global__ __launch_bounds__(256) void qkv_rope_kernel(
    const float* __restrict__ part, int splits, int64_t split_stride, int T, int Hq, int Hkv,
    const float2* __restrict__ rope, const int32_t* __restrict__ row_slot, KvView kv, int layer_pool, int layer,
    float* __restrict__ q_out)
{
    constexpr int DHc = 128, HALF = 64;
    const int m = blockIdx.x;
    const int slot = row_slot[m];
    const bool writable = slot >= 0;
    const int64_t page = writable ? slot / SPEC_PAGE_SIZE : 0;
    const int t = writable ? slot % SPEC_PAGE_SIZE : 0;
    const int nqkv = (Hq + 2 * Hkv) * DHc;
    const float* row = part + (int64_t)m * nqkv;
    unsigned short* pool = (unsigned short*)kv.pool;
    const int64_t block = (int64_t)SPEC_PAGE_SIZE * DHc;
    // sum of the slices of 4 adjacent columns, in slice order; the loads go out eight (four, two) at a time - a plain
    // loop would wait for each slice before asking for the next
    auto sum4 = [&](int n) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        int s = 0;
        auto add_group = [&](auto n_c) {
            constexpr int GN = decltype(n_c)::value;
            float4 p[GN];
#pragma unroll
            for (int u = 0; u < GN; ++u) p[u] = *(const float4*)(row + (s + u) * split_stride + n);
#pragma unroll
            for (int u = 0; u < GN; ++u) { v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w; }
            s += GN;
        };
        while (s + 8 <= splits) add_group(std::integral_constant<int, 8>{});
        if (s + 4 <= splits) add_group(std::integral_constant<int, 4>{});
        if (s + 2 <= splits) add_group(std::integral_constant<int, 2>{});
        if (s < splits) add_group(std::integral_constant<int, 1>{});
        return v;
    };
    // rotary part: heads 0 .. Hq+Hkv-1, 16 quads of the lower half each
    for (int e = threadIdx.x + 256 * blockIdx.y; e < (Hq + Hkv) * (HALF / 4); e += 256 * gridDim.y) {
        int h = e / (HALF / 4), j = (e % (HALF / 4)) * 4;
        float4 lo = sum4(h * DHc + j), hi = sum4(h * DHc + j + HALF);
        const float2* cs = rope + (int64_t)m * HALF + j;
        float l[4] = {lo.x, lo.y, lo.z, lo.w}, u[4] = {hi.x, hi.y, hi.z, hi.w}, rl[4], ru[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            float2 c = cs[a];
            rl[a] = l[a] * c.x - u[a] * c.y;
            ru[a] = u[a] * c.x + l[a] * c.y;
        }
        uint2 plo = make_uint2(to_bf16(rl[0]) | (to_bf16(rl[1]) << 16), to_bf16(rl[2]) | (to_bf16(rl[3]) << 16));
        uint2 phi = make_uint2(to_bf16(ru[0]) | (to_bf16(ru[1]) << 16), to_bf16(ru[2]) | (to_bf16(ru[3]) << 16));
        if (h < Hq) {
            float* dst = q_out + ((int64_t)m * Hq + h) * DHc;
            *(float4*)(dst + j) = make_float4(rl[0], rl[1], rl[2], rl[3]);
            *(float4*)(dst + j + HALF) = make_float4(ru[0], ru[1], ru[2], ru[3]);
        } else if (writable) {
            int kh = h - Hq;
            if constexpr (KV8) {
                const float ks = kv.k_scale[layer * Hkv + kh];
                unsigned char* dst = (unsigned char*)kv.pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 0) * Hkv + kh) * block;
                *(unsigned int*)(dst + kv_block_offset(SPEC_FP8_E4M3, 0, t, j, DHc)) =
                    to_e4m3(rl[0] / ks) | (to_e4m3(rl[1] / ks) << 8) | (to_e4m3(rl[2] / ks) << 16) | (to_e4m3(rl[3] / ks) << 24);
                *(unsigned int*)(dst + kv_block_offset(SPEC_FP8_E4M3, 0, t, j + HALF, DHc)) =
                    to_e4m3(ru[0] / ks) | (to_e4m3(ru[1] / ks) << 8) | (to_e4m3(ru[2] / ks) << 16) | (to_e4m3(ru[3] / ks) << 24);
            } else {
                unsigned short* dst = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 0) * Hkv + kh) * block;
                *(uint2*)(dst + kv_block_offset(SPEC_BF16, 0, t, j, DHc)) = plo;
                *(uint2*)(dst + kv_block_offset(SPEC_BF16, 0, t, j + HALF, DHc)) = phi;
            }
        }
    }
    // values: no rotation
    if (writable)
        for (int e = threadIdx.x + 256 * blockIdx.y; e < Hkv * (DHc / 4); e += 256 * gridDim.y) {
            int kh = e / (DHc / 4), c = (e % (DHc / 4)) * 4;
            float4 v = sum4((Hq + Hkv + kh) * DHc + c);
            if constexpr (KV8) {
                const float vs = kv.v_scale[layer * Hkv + kh];
                unsigned char* dst8 = (unsigned char*)kv.pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 1) * Hkv + kh) * block;
                dst8[kv_block_offset(SPEC_FP8_E4M3, 1, t, c + 0, DHc)] = (unsigned char)to_e4m3(v.x / vs);
                dst8[kv_block_offset(SPEC_FP8_E4M3, 1, t, c + 1, DHc)] = (unsigned char)to_e4m3(v.y / vs);
                dst8[kv_block_offset(SPEC_FP8_E4M3, 1, t, c + 2, DHc)] = (unsigned char)to_e4m3(v.z / vs);
                dst8[kv_block_offset(SPEC_FP8_E4M3, 1, t, c + 3, DHc)] = (unsigned char)to_e4m3(v.w / vs);
                continue;
            }
            unsigned short* dst = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 1) * Hkv + kh) * block;
            dst[kv_block_offset(SPEC_BF16, 1, t, c + 0, DHc)] = to_bf16(v.x);
            dst[kv_block_offset(SPEC_BF16, 1, t, c + 1, DHc)] = to_bf16(v.y);
            dst[kv_block_offset(SPEC_BF16, 1, t, c + 2, DHc)] = to_bf16(v.z);
            dst[kv_block_offset(SPEC_BF16, 1, t, c + 3, DHc)] = to_bf16(v.w);
        }
}

// act = silu(sum gate) * (sum up) from the gate/up projection [M][2F] -> bf16 operand order (K = F)
__global__ void swiglu_pack_kernel(const float* __restrict__ part, int splits, int64_t split_stride, int M, int F, int mb_pad,
                                   int xf, uint4* __restrict__ xp)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int f8 = F / 8;
    if (idx >= (int64_t)M * f8) return;
    int m = (int)(idx / f8), f = (int)(idx % f8) * 8;
    // the gate/up weights are tiled with their 32-column blocks interleaved: gate channel f sits in
    // column (f/32)*64 + f%32 of the projection's output, up channel f 32 columns further
    const float* row = part + (int64_t)m * 2 * F + (f >> 5) * 64 + (f & 31);
    float g[8], u[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float4 a = *(const float4*)(row + 4 * h), c = *(const float4*)(row + 32 + 4 * h);
        for (int s = 1; s < splits; ++s) {
            float4 a2 = *(const float4*)(row + s * split_stride + 4 * h), c2 = *(const float4*)(row + s * split_stride + 32 + 4 * h);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            c.x += c2.x; c.y += c2.y; c.z += c2.z; c.w += c2.w;
        }
        g[4 * h] = a.x; g[4 * h + 1] = a.y; g[4 * h + 2] = a.z; g[4 * h + 3] = a.w;
        u[4 * h] = c.x; u[4 * h + 1] = c.y; u[4 * h + 2] = c.z; u[4 * h + 3] = c.w;
    }
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = g[j] / (1.0f + expf(-g[j])) * u[j];
    xp_store8_rt(xp, xf, m, f, mb_pad, v);
}

// fp32 rows [M, K] -> the hi + lo operand of a projection, unchanged in value (the multi-layer features before w_fc)
__global__ __launch_bounds__(256) void pack_rows_kernel(const float* __restrict__ src, int M, int K, int mb_pad, uint4* __restrict__ xp)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = K / 8;
    if (i >= (int64_t)M * per_row) return;
    const int m = (int)(i / per_row), c = (int)(i % per_row) * 8;
    const float4 a = *(const float4*)(src + (int64_t)m * K + c), b = *(const float4*)(src + (int64_t)m * K + c + 4);
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    xp_store8(xp, m, c, mb_pad, v);
}

// the residual stream [M, d] into columns col0 .. col0+d-1 of the feature rows [M, width]
__global__ __launch_bounds__(256) void tap_copy_kernel(const float* __restrict__ x, int M, int d, float* __restrict__ taps, int width, int col0)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = d / 4;
    if (i >= (int64_t)M * per_row) return;
    const int m = (int)(i / per_row), c = (int)(i % per_row) * 4;
    *(float4*)(taps + (int64_t)m * width + col0 + c) = *(const float4*)(x + (int64_t)m * d + c);
}

// ------------------------------------------------------------------ host side
struct Bf16Plan {
    int M, mb_pad, max_chunks, RBrows;
    bool fuse_swiglu;
    int s_qkv, s_o, s_gu, s_down, s_head, s_fuse, s_fc;
    size_t off_x, off_xp_h, off_xp_a, off_xp_f, off_part, off_q, off_rope, off_att_o, off_att_ml, total;
    int max_items;                          // attention work items the buffers hold
    size_t off_row_slot, off_items, off_entry_items;
    // mixture of experts: padded-row bound, router splits, routing tables, permuted activations, expert outputs
    int moe_rows, s_router;
    size_t off_ids, off_wts, off_row0, off_tiles, off_src_row, off_pair_row, off_xp_e, off_y_e;
};

static Bf16Plan make_plan(const spec_model* m, int B, int k, int64_t max_ctx_plus)
{
    const spec_model_desc& d = m->desc;
    Bf16Plan p;
    int T = k + 1;
    p.M = B * T;
    p.mb_pad = gemm_mb_pad(p.M);
    int G = d.n_q_heads / d.n_kv_heads;
    p.RBrows = attn_rows_padded(T * G);
    p.max_chunks = 0;
    p.max_items = attn_max_items(T * G, B, d.n_kv_heads, (int)cdiv(max_ctx_plus, SPEC_PAGE_SIZE));   // the most any launch may use
    p.s_qkv = gemm_pick_splits(m->wqkv[0], p.M, tune("splits_qkv"));
    p.s_o = gemm_pick_splits(m->wo[0], p.M, tune("splits_o"));
    const bool moe = m->moe();
    p.fuse_swiglu = !moe && tune("fuse_swiglu") != 0 && gemm_can_fuse_swiglu(m->wgu[0], p.M, 1);
    p.s_gu = (p.fuse_swiglu || moe) ? 1 : gemm_pick_splits(m->wgu[0], p.M, tune("splits_gu"));
    p.s_down = moe ? 1 : gemm_pick_splits(m->wd[0], p.M, tune("splits_down"));
    p.s_head = 1;
    p.s_fuse = d.fuse_hidden ? gemm_pick_splits(m->wfuse, p.M, 0) : 0;
    p.s_fc = d.fuse_taps ? gemm_pick_splits(m->wfc, p.M, 0) : 0;
    p.s_router = moe ? gemm_pick_splits(m->router[0], p.M, 0) : 0;
    p.moe_rows = moe ? moe_rows_bound(p.M, d.top_k, d.n_experts) : 0;
    int D = d.d_model, F = moe ? d.expert_ffn_dim : d.ffn_dim, nq = d.n_q_heads * d.head_dim, nqkv = nq + 2 * d.n_kv_heads * d.head_dim;
    size_t rows = (size_t)p.mb_pad * 32;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p.off_x = take((size_t)p.M * D * 4);
    p.off_xp_h = take(rows * D * 4);          // hi + lo
    p.off_xp_a = take(rows * nq * 4);
    // (mixture: the permuted rows' silu(gate)*up; a feature-fed draft stages its features here first)
    p.off_xp_f = take((moe ? (size_t)p.moe_rows : rows) * (size_t)std::max(F, d.fuse_taps * D) * 4);
    size_t part = std::max(std::max((size_t)p.s_qkv * nqkv, (size_t)p.s_o * D), std::max((size_t)p.s_gu * 2 * F, (size_t)p.s_down * D));
    if (moe) part = std::max(std::max((size_t)p.s_qkv * nqkv, (size_t)p.s_o * D), (size_t)p.s_router * d.n_experts);
    part = std::max(part, (size_t)std::max(p.s_fuse, p.s_fc) * D);
    p.off_part = take(part * p.M * 4);
    if (moe) {
        size_t pairs = (size_t)p.M * d.top_k;
        p.off_ids = take(pairs * 4);
        p.off_wts = take(pairs * 4);
        p.off_pair_row = take(pairs * 4);
        p.off_row0 = take((size_t)(d.n_experts + 1) * 4);
        p.off_tiles = take((size_t)(1 + 2 * (p.moe_rows / 64)) * 4);
        p.off_src_row = take((size_t)p.moe_rows * 4);
        p.off_xp_e = take((size_t)p.moe_rows * D * 4);
        p.off_y_e = take((size_t)p.moe_rows * D * 4);
    }
    p.off_q = take((size_t)p.M * nq * 4);
    p.off_rope = take((size_t)p.M * (d.head_dim / 2) * 8);
    p.off_row_slot = take((size_t)p.M * 4);
    p.off_items = take((size_t)p.max_items * attn_item_bytes());
    p.off_entry_items = take((size_t)B * 8);
    size_t items = (size_t)p.max_items * d.n_kv_heads;
    p.off_att_o = take(items * p.RBrows * d.head_dim * 4);
    p.off_att_ml = take(items * p.RBrows * 2 * 4);
    p.total = off;
    return p;
}

size_t bf16_workspace_bytes(const spec_model* m, const spec_kv* kv, int B, int k)
{
    return make_plan(m, B, k, (int64_t)kv->max_pages * SPEC_PAGE_SIZE).total;
}

spec_status bf16_forward(spec_model* mdl, spec_kv* kv, int B, int k, const int32_t* dev_seq_ids, const int32_t* dev_tokens,
                         const Bf16Extras& io, float* dev_logits, void* ws, size_t ws_bytes, hipStream_t s)
{
    const spec_model_desc& d = mdl->desc;
    float* const dev_hidden_out = io.dev_hidden_out;
    const int T = k + 1, G = d.n_q_heads / d.n_kv_heads;
    if (T * G > 256) { set_error("bf16 path: (k+1) * (query heads per kv head) = %d exceeds 256", T * G); return SPEC_EUNSUPPORTED; }
    // the workspace is laid out for the longest context the cache allows; the launch only spans
    // the chunks the current bound on the longest sequence needs
    Bf16Plan p = make_plan(mdl, B, k, (int64_t)kv->max_pages * SPEC_PAGE_SIZE);
    if (p.total > ws_bytes) { set_error("spec_verify_forward: workspace too small for the current split settings (%zu < %zu)", ws_bytes, p.total); return SPEC_EINVAL; }
    // pages of the longest live context (the host's bound), capped by what the buffers were sized for
    int live_pages = (int)cdiv(kv->ub.max_ctx + T, SPEC_PAGE_SIZE);
    if (live_pages > kv->max_pages) live_pages = kv->max_pages;
    if (live_pages < 1) live_pages = 1;

    char* base = (char*)ws;
    float* x = (float*)(base + p.off_x);
    bf16_t* xp_h = (bf16_t*)(base + p.off_xp_h);
    bf16_t* xp_a = (bf16_t*)(base + p.off_xp_a);
    bf16_t* xp_f = (bf16_t*)(base + p.off_xp_f);
    float* part = (float*)(base + p.off_part);
    float* qbuf = (float*)(base + p.off_q);
    float2* rope = (float2*)(base + p.off_rope);
    float* att_o = (float*)(base + p.off_att_o);
    float* att_ml = (float*)(base + p.off_att_ml);
    int32_t* row_slot = (int32_t*)(base + p.off_row_slot);
    void* att_items = base + p.off_items;
    void* att_entry_items = base + p.off_entry_items;

    const int M = p.M, D = d.d_model, F = d.ffn_dim, Hq = d.n_q_heads, Hkv = d.n_kv_heads;
    const int nqkv = (Hq + 2 * Hkv) * d.head_dim;
    KvView view = kv->view();
    spec_status st;
    const int norm_threads = D >= 4096 ? 512 : 256;
    // operand format each projection's input is written in: the one its matrix was tiled for at model creation
    auto xf_of = [](const PackedW& W) { return W.f16 ? XF_F16 : XF_HILO; };
    if (!mdl->moe() && mdl->wgu[0].f16 != mdl->wd[0].f16) { set_error("bf16 forward: gate/up and down projection must take the same activation format"); return SPEC_ESTATE; }

    rope_table_kernel<<<(unsigned)cdiv((int64_t)M * 64, 256), 256, 0, s>>>(M, T, view, 64, (double)d.rope_theta, rope, row_slot);
    if ((st = launch_attention_plan(B, T, G, Hkv, view, live_pages, att_items, att_entry_items, s)) != SPEC_OK) return st;
    if (d.fuse_hidden) {
        // hidden-state input: x = w_fuse . [RMSNorm(embed) ; RMSNorm(hidden_in)] (the feed-forward operand buffer is free here)
        const float* hidden = io.dev_hidden_in;
        int h_splits = 1;
        if (io.dev_features_in) {
            // multi-layer features: hidden = w_fc . features, left as K-split partial sums for the kernel below
            const int Kf = d.fuse_taps * D;
            pack_rows_kernel<<<(unsigned)cdiv((int64_t)M * (Kf / 8), 256), 256, 0, s>>>(io.dev_features_in, M, Kf, p.mb_pad, (uint4*)xp_f);
            if ((st = launch_gemm_bf16(mdl->wfc, xp_f, M, part, D, p.s_fc, false, s)) != SPEC_OK) return st;
            hidden = part;
            h_splits = p.s_fc;
        }
        fuse_input_kernel<<<M, norm_threads, 0, s>>>(dev_tokens, (const unsigned short*)mdl->embed(), d.vocab, hidden, h_splits, (int64_t)M * D,
                                                     (const unsigned short*)mdl->fuse_w(1), (const unsigned short*)mdl->fuse_w(2), D, d.rms_eps,
                                                     p.mb_pad, (uint4*)xp_f);
        if ((st = launch_gemm_bf16(mdl->wfuse, xp_f, M, part, D, p.s_fuse, false, s)) != SPEC_OK) return st;
        residual_rmsnorm_kernel<RES_SET><<<M, norm_threads, 0, s>>>(x, part, p.s_fuse, (int64_t)M * D, nullptr, nullptr, 0,
                                                                   (const unsigned short*)mdl->layer_w(0, 0), D, d.rms_eps, p.mb_pad, xf_of(mdl->wqkv[0]), (uint4*)xp_h);
    } else {
        residual_rmsnorm_kernel<RES_EMBED><<<M, norm_threads, 0, s>>>(x, nullptr, 0, 0, dev_tokens, (const unsigned short*)mdl->embed(), d.vocab,
                                                        (const unsigned short*)mdl->layer_w(0, 0), D, d.rms_eps, p.mb_pad, xf_of(mdl->wqkv[0]), (uint4*)xp_h);
    }
    prof_mark(PC_EMBED_NORM, s);
    // the residual stream after `done` layers into every feature column block that asks for it
    auto write_taps = [&](int done) {
        for (int j = 0; j < io.n_taps; ++j)
            if (io.tap_layers[j] == done)
                tap_copy_kernel<<<(unsigned)cdiv((int64_t)M * (D / 4), 256), 256, 0, s>>>(x, M, D, io.dev_taps_out, io.n_taps * D, j * D);
    };
    for (int l = 0; l < d.n_layers; ++l) {
        int lp = kv->alias_mod > 0 ? l % kv->alias_mod : l;
        if ((st = launch_gemm_bf16(mdl->wqkv[l], xp_h, M, part, nqkv, p.s_qkv, false, s)) != SPEC_OK) return st;
        prof_mark(PC_GEMM_QKV, s);
        if (view.fp8)
            qkv_rope_kernel<true><<<dim3(M, 4), 256, 0, s>>>(part, p.s_qkv, (int64_t)M * nqkv, T, Hq, Hkv, rope, row_slot, view, lp, l, qbuf);
        else
            qkv_rope_kernel<false><<<dim3(M, 4), 256, 0, s>>>(part, p.s_qkv, (int64_t)M * nqkv, T, Hq, Hkv, rope, row_slot, view, lp, l, qbuf);
        prof_mark(PC_QKV_ROPE, s);
        if ((st = launch_attention_bf16(qbuf, B, T, G, Hq, Hkv, view, lp, l, live_pages, att_items, att_entry_items, att_o, att_ml, p.mb_pad, xf_of(mdl->wo[l]), xp_a, s)) != SPEC_OK) return st;
        if ((st = launch_gemm_bf16(mdl->wo[l], xp_a, M, part, D, p.s_o, false, s)) != SPEC_OK) return st;
        prof_mark(PC_GEMM_O, s);
        // (mixture of experts: the router reads this buffer and stays hi + lo; the gather below converts for the experts)
        residual_rmsnorm_kernel<RES_ADD><<<M, norm_threads, 0, s>>>(x, part, p.s_o, (int64_t)M * D, nullptr, nullptr, 0,
                                                         (const unsigned short*)mdl->layer_w(l, 5), D, d.rms_eps, p.mb_pad,
                                                         mdl->moe() ? xf_of(mdl->router[l]) : xf_of(mdl->wgu[l]), (uint4*)xp_h);
        prof_mark(PC_RESID_NORM, s);
        const void* next_gain = l + 1 < d.n_layers ? mdl->layer_w(l + 1, 0) : mdl->final_norm();
        const int next_xf = l + 1 < d.n_layers ? xf_of(mdl->wqkv[l + 1]) : xf_of(mdl->head);
        if (mdl->moe()) {
            // router -> top-k -> rows permuted into per-expert tiles -> grouped gate/up (SwiGLU fused) and down
            // projections over the tile list -> weighted combine + residual + next RMSNorm
            const int E = d.n_experts, Fe = d.expert_ffn_dim, max_tiles = p.moe_rows / 64;
            int32_t* ids = (int32_t*)(base + p.off_ids);
            float* wts = (float*)(base + p.off_wts);
            int32_t* pair_row = (int32_t*)(base + p.off_pair_row);
            int32_t* row0 = (int32_t*)(base + p.off_row0);
            int32_t* tiles = (int32_t*)(base + p.off_tiles);
            int32_t* src_row = (int32_t*)(base + p.off_src_row);
            bf16_t* xp_e = (bf16_t*)(base + p.off_xp_e);
            float* y_e = (float*)(base + p.off_y_e);
            if ((st = launch_gemm_bf16(mdl->router[l], xp_h, M, part, E, p.s_router, false, s)) != SPEC_OK) return st;
            if ((st = launch_moe_route(part, p.s_router, (int64_t)M * E, M, E, d.top_k, ids, wts, row0, tiles, src_row, pair_row, s)) != SPEC_OK) return st;
            prof_mark(PC_MOE_ROUTE, s);
            if ((st = launch_moe_gather(xp_h, p.mb_pad, src_row, row0, E, D, p.moe_rows, xf_of(mdl->wgu[l]), xp_e, s)) != SPEC_OK) return st;
            prof_mark(PC_MOE_GATHER, s);
            if ((st = launch_gemm_bf16_grouped(mdl->wgu[l], mdl->moe_gu_stride, xp_e, p.moe_rows, max_tiles, tiles, (float*)xp_f, 2 * Fe, true, s)) != SPEC_OK) return st;
            prof_mark(PC_GEMM_GU, s);
            if ((st = launch_gemm_bf16_grouped(mdl->wd[l], mdl->moe_d_stride, xp_f, p.moe_rows, max_tiles, tiles, y_e, D, false, s)) != SPEC_OK) return st;
            prof_mark(PC_GEMM_DOWN, s);
            if ((st = launch_moe_combine_norm(x, y_e, pair_row, wts, M, d.top_k, next_gain, D, d.rms_eps, p.mb_pad, next_xf, xp_h, s)) != SPEC_OK) return st;
            prof_mark(PC_RESID_NORM, s);
            write_taps(l + 1);
            continue;
        }
        if (p.fuse_swiglu) {
            // gate/up projection with silu(gate) * up in its epilogue: writes the down projection's operand
            if ((st = launch_gemm_bf16(mdl->wgu[l], xp_h, M, (float*)xp_f, 2 * F, 1, true, s)) != SPEC_OK) return st;
            prof_mark(PC_GEMM_GU, s);
        } else {
            if ((st = launch_gemm_bf16(mdl->wgu[l], xp_h, M, part, 2 * F, p.s_gu, false, s)) != SPEC_OK) return st;
            prof_mark(PC_GEMM_GU, s);
            swiglu_pack_kernel<<<(unsigned)cdiv((int64_t)M * (F / 8), 256), 256, 0, s>>>(part, p.s_gu, (int64_t)M * 2 * F, M, F, p.mb_pad, xf_of(mdl->wd[l]), (uint4*)xp_f);
            prof_mark(PC_SWIGLU, s);
        }
        if ((st = launch_gemm_bf16(mdl->wd[l], xp_f, M, part, D, p.s_down, false, s)) != SPEC_OK) return st;
        prof_mark(PC_GEMM_DOWN, s);
        residual_rmsnorm_kernel<RES_ADD><<<M, norm_threads, 0, s>>>(x, part, p.s_down, (int64_t)M * D, nullptr, nullptr, 0,
                                                         (const unsigned short*)next_gain, D, d.rms_eps, p.mb_pad, next_xf, (uint4*)xp_h);
        prof_mark(PC_RESID_NORM, s);
        write_taps(l + 1);
    }
    if (dev_hidden_out) {
        // the residual stream after the last layer: what a hidden-state-consuming draft model is fed
        if (hipMemcpyAsync(dev_hidden_out, x, (size_t)M * D * sizeof(float), hipMemcpyDeviceToDevice, s) != hipSuccess) {
            set_error("spec_verify_forward_hidden: copy of the hidden states failed");
            return SPEC_EHIP;
        }
    }
    if ((st = launch_gemm_bf16(mdl->head, xp_h, M, dev_logits, head_rows(d), 1, false, s)) != SPEC_OK) return st;
    prof_mark(PC_GEMM_HEAD, s);
    SPEC_LAUNCH_CHECK("bf16 forward");
    return SPEC_OK;
}

}  // namespace specv
