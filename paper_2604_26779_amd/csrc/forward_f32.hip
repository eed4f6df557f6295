// Generic fp32 verify forward: plain kernels for any model shape (the tiny fp32 configuration and
// a bring-up reference for shapes the MFMA path does not cover).  Same step order as the bf16
// path: embed -> per layer [RMSNorm, QKV, rotary + speculative KV write, causal attention over the
// paged cache, O + residual, RMSNorm, gate/up, SwiGLU, down + residual] -> final RMSNorm -> head.
#include "common.h"

namespace specv {

// ------------------------------------------------------------------ small kernels
__global__ void f32_embed_kernel(const int32_t* __restrict__ tokens, const float* __restrict__ embed, int d, int vocab,
                                 float* __restrict__ x)
{
    int m = blockIdx.x;
    int t = tokens[m];
    t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
    for (int c = threadIdx.x; c < d; c += blockDim.x) x[(int64_t)m * d + c] = embed[(int64_t)t * d + c];
}

__global__ __launch_bounds__(256) void f32_rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                          int d, float eps, float* __restrict__ y)
{
    int m = blockIdx.x;
    const float* xr = x + (int64_t)m * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) ss += xr[c] * xr[c];
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = part[0] + part[1] + part[2] + part[3];
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) y[(int64_t)m * d + c] = xr[c] * r * gain[c];
}

// y[m][n] (+)= sum_k a[m][k] * w[n][k], y has leading dimension ldy;
// 32x32 output tile per workgroup, 16x16 threads, 2x2 outputs per thread
template <bool ACCUM>
__global__ __launch_bounds__(256) void f32_gemm_kernel(const float* __restrict__ a, const float* __restrict__ w, int M,
                                                       int N, int K, float* __restrict__ y, int ldy)
{
    __shared__ float sa[32][33], sw[32][33];
    int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int i = threadIdx.x; i < 32 * 32; i += 256) {
            int r = i >> 5, c = i & 31;
            int kk = k0 + c;
            sa[r][c] = (m0 + r < M && kk < K) ? a[(int64_t)(m0 + r) * K + kk] : 0.f;
            sw[r][c] = (n0 + r < N && kk < K) ? w[(int64_t)(n0 + r) * K + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < 32; ++c) {
            float a0 = sa[ty][c], a1 = sa[ty + 16][c], w0 = sw[tx][c], w1 = sw[tx + 16][c];
            acc[0][0] += a0 * w0; acc[0][1] += a0 * w1; acc[1][0] += a1 * w0; acc[1][1] += a1 * w1;
        }
        __syncthreads();
    }
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            int m = m0 + ty + 16 * i, n = n0 + tx + 16 * j;
            if (m < M && n < N) {
                float* dst = y + (int64_t)m * ldy + n;
                *dst = ACCUM ? *dst + acc[i][j] : acc[i][j];
            }
        }
}

// rotary embedding of q (in place) and k, and the speculative write of k, v into the paged cache.
// one workgroup per input row; qkv row = [q heads | k heads | v heads]
__global__ void f32_rope_kv_write_kernel(float* __restrict__ qkv, int T, const int32_t* __restrict__ seq_ids,
                                         KvView kv, int layer_pool, int Hq, int Hkv, int dh, float theta)
{
    int m = blockIdx.x;
    int b = m / T, i = m % T;
    int seq = kv.entry_seq[b];                     // -1: the entry was dropped (id out of range or named twice)
    int pos = seq >= 0 ? kv.ctx_len[seq] + i : 0;
    int half = dh >> 1;
    float* row = qkv + (int64_t)m * (Hq + 2 * Hkv) * dh;
    int lp = pos / SPEC_PAGE_SIZE, t = pos % SPEC_PAGE_SIZE;
    bool writable = seq >= 0 && lp < kv.n_held[seq];
    int64_t page = writable ? kv.page_table[(int64_t)seq * kv.max_pages + lp] : 0;
    float* pool = (float*)kv.pool;
    int64_t block = (int64_t)SPEC_PAGE_SIZE * dh;
    for (int e = threadIdx.x; e < (Hq + Hkv) * half; e += blockDim.x) {
        int h = e / half, j = e % half;
        float inv_freq = powf(theta, -2.0f * (float)j / (float)dh);
        float ang = (float)pos * inv_freq;
        float c = cosf(ang), s = sinf(ang);
        float* v = row + (int64_t)h * dh;
        float lo = v[j], hi = v[j + half];
        float rlo = lo * c - hi * s, rhi = hi * c + lo * s;
        if (h < Hq) { v[j] = rlo; v[j + half] = rhi; }
        else if (writable) {
            int kh = h - Hq;
            float* dst = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 0) * Hkv + kh) * block;
            dst[(int64_t)t * dh + j] = rlo;
            dst[(int64_t)t * dh + j + half] = rhi;
        }
    }
    if (writable)
        for (int e = threadIdx.x; e < Hkv * dh; e += blockDim.x) {
            int kh = e / dh, c = e % dh;
            float* dst = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 1) * Hkv + kh) * block;
            dst[(int64_t)t * dh + c] = row[(int64_t)(Hq + Hkv + kh) * dh + c];
        }
}

// one wavefront per (input row, query head): online softmax over the visible cache positions
__global__ __launch_bounds__(64) void f32_attention_kernel(const float* __restrict__ qkv, int T,
                                                           const int32_t* __restrict__ seq_ids, KvView kv,
                                                           int layer_pool, int Hq, int Hkv, int dh, float scale,
                                                           float* __restrict__ out)
{
    int m = blockIdx.x, j = blockIdx.y;
    int b = m / T, i = m % T;
    int seq = kv.entry_seq[b];
    int visible = seq >= 0 ? kv.ctx_len[seq] + i + 1 : 0;
    int cap = seq >= 0 ? kv.n_held[seq] * SPEC_PAGE_SIZE : 0;
    if (visible > cap) visible = cap;
    int g = j / (Hq / Hkv);
    const float* q = qkv + (int64_t)m * (Hq + 2 * Hkv) * dh + (int64_t)j * dh;
    const float* pool = (const float*)kv.pool;
    int64_t block = (int64_t)SPEC_PAGE_SIZE * dh;
    int lane = threadIdx.x;
    __shared__ float sq[256];
    __shared__ float sp[64];
    for (int c = lane; c < dh; c += 64) sq[c] = q[c];
    __syncthreads();
    float mx = -INFINITY, sum = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};                  // channels lane, lane+64, ... (dh <= 256)
    for (int p0 = 0; p0 < visible; p0 += 64) {
        int pos = p0 + lane;
        float s = -INFINITY;
        if (pos < visible) {
            int64_t page = kv.page_table[(int64_t)seq * kv.max_pages + pos / SPEC_PAGE_SIZE];
            const float* kr = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 0) * Hkv + g) * block +
                              (int64_t)(pos % SPEC_PAGE_SIZE) * dh;
            float d = 0.f;
            for (int c = 0; c < dh; ++c) d += kr[c] * sq[c];
            s = d * scale;
        }
        float cm = s;
        for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
        float nm = fmaxf(mx, cm);
        float corr = expf(mx - nm);
        float p = (pos < visible) ? expf(s - nm) : 0.f;
        float ps = p;
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
        sum = sum * corr + ps;
        mx = nm;
        __syncthreads();
        sp[lane] = p;
        __syncthreads();
        int cnt = visible - p0 < 64 ? visible - p0 : 64;
        for (int a = 0; a < 4; ++a) {
            int c = lane + 64 * a;
            if (c < dh) {
                float o = acc[a] * corr;
                for (int t = 0; t < cnt; ++t) {
                    int pp = p0 + t;
                    int64_t page = kv.page_table[(int64_t)seq * kv.max_pages + pp / SPEC_PAGE_SIZE];
                    const float* vr = pool + ((((int64_t)layer_pool * kv.n_pages + page) * 2 + 1) * Hkv + g) * block +
                                      (int64_t)(pp % SPEC_PAGE_SIZE) * dh;
                    o += sp[t] * vr[c];
                }
                acc[a] = o;
            }
        }
    }
    for (int a = 0; a < 4; ++a) {
        int c = lane + 64 * a;
        if (c < dh) out[(int64_t)m * Hq * dh + (int64_t)j * dh + c] = sum > 0.f ? acc[a] / sum : 0.f;
    }
}

__global__ void f32_swiglu_kernel(const float* __restrict__ gu, int M, int F, float* __restrict__ act)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)M * F) return;
    int m = idx / F, f = idx % F;
    float g = gu[(int64_t)m * 2 * F + f], u = gu[(int64_t)m * 2 * F + F + f];
    act[idx] = g / (1.0f + expf(-g)) * u;
}

// ------------------------------------------------------------------ host side
struct F32Ws { float *x, *h, *qkv, *attn, *gu, *act; };

static size_t f32_carve(const spec_model_desc& d, int M, char* base, F32Ws* w)
{
    size_t off = 0;
    auto take = [&](size_t elems) { size_t o = off; off = align_up(off + elems * sizeof(float), 256); return base ? (float*)(base + o) : nullptr; };
    int nqkv = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    F32Ws t;
    t.x = take((size_t)M * d.d_model);
    t.h = take((size_t)M * d.d_model);
    t.qkv = take((size_t)M * nqkv);
    t.attn = take((size_t)M * d.n_q_heads * d.head_dim);
    t.gu = take((size_t)M * 2 * d.ffn_dim);
    t.act = take((size_t)M * d.ffn_dim);
    if (w) *w = t;
    return off;
}

size_t f32_workspace_bytes(const spec_model_desc& d, int B, int k) { return f32_carve(d, B * (k + 1), nullptr, nullptr); }

static void gemm(const float* a, const float* w, int M, int N, int K, float* y, int ldy, bool accum, hipStream_t s)
{
    dim3 grid((unsigned)cdiv(N, 32), (unsigned)cdiv(M, 32));
    if (accum) f32_gemm_kernel<true><<<grid, 256, 0, s>>>(a, w, M, N, K, y, ldy);
    else f32_gemm_kernel<false><<<grid, 256, 0, s>>>(a, w, M, N, K, y, ldy);
}

spec_status f32_forward(spec_model* mdl, spec_kv* kv, int B, int k, const int32_t* dev_seq_ids,
                        const int32_t* dev_tokens, float* dev_logits, void* ws, hipStream_t s)
{
    const spec_model_desc& d = mdl->desc;
    if (d.head_dim > 256 || (d.head_dim & 1)) { set_error("fp32 path needs an even head_dim <= 256"); return SPEC_EUNSUPPORTED; }
    int T = k + 1, M = B * T;
    int Hq = d.n_q_heads, Hkv = d.n_kv_heads, dh = d.head_dim, D = d.d_model, F = d.ffn_dim;
    int nq = Hq * dh, nkv = Hkv * dh, nqkv = nq + 2 * nkv;
    F32Ws w;
    f32_carve(d, M, (char*)ws, &w);
    KvView view = kv->view();
    float scale = 1.0f / sqrtf((float)dh);

    f32_embed_kernel<<<M, 256, 0, s>>>(dev_tokens, (const float*)mdl->embed(), D, d.vocab, w.x);
    for (int l = 0; l < d.n_layers; ++l) {
        int lp = kv->alias_mod > 0 ? l % kv->alias_mod : l;
        auto W = [&](int i) { return (const float*)mdl->layer_w(l, i); };
        f32_rmsnorm_kernel<<<M, 256, 0, s>>>(w.x, W(0), D, d.rms_eps, w.h);
        gemm(w.h, W(1), M, nq, D, w.qkv, nqkv, false, s);
        gemm(w.h, W(2), M, nkv, D, w.qkv + nq, nqkv, false, s);
        gemm(w.h, W(3), M, nkv, D, w.qkv + nq + nkv, nqkv, false, s);
        f32_rope_kv_write_kernel<<<M, 256, 0, s>>>(w.qkv, T, dev_seq_ids, view, lp, Hq, Hkv, dh, d.rope_theta);
        f32_attention_kernel<<<dim3(M, Hq), 64, 0, s>>>(w.qkv, T, dev_seq_ids, view, lp, Hq, Hkv, dh, scale, w.attn);
        gemm(w.attn, W(4), M, D, nq, w.x, D, true, s);
        f32_rmsnorm_kernel<<<M, 256, 0, s>>>(w.x, W(5), D, d.rms_eps, w.h);
        gemm(w.h, W(6), M, F, D, w.gu, 2 * F, false, s);
        gemm(w.h, W(7), M, F, D, w.gu + F, 2 * F, false, s);
        f32_swiglu_kernel<<<(unsigned)cdiv((int64_t)M * F, 256), 256, 0, s>>>(w.gu, M, F, w.act);
        gemm(w.act, W(8), M, D, F, w.x, D, true, s);
    }
    f32_rmsnorm_kernel<<<M, 256, 0, s>>>(w.x, (const float*)mdl->final_norm(), D, d.rms_eps, w.h);
    gemm(w.h, (const float*)mdl->head_w(), M, head_rows(d), D, dev_logits, head_rows(d), false, s);
    SPEC_LAUNCH_CHECK("fp32 forward");
    return SPEC_OK;
}

}  // namespace specv
