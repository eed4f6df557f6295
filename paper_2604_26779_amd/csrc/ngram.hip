// Model-free n-gram drafting (the paper's n-gram baseline, Section 3.2 / Table 2; prompt-lookup reading): drafts
// are copied from behind the most recent earlier occurrence of the history's current ending.
//
// One workgroup per sequence.  Every position e <= L-2 is a candidate for "where an occurrence of the ending
// ends": its match length m(e) = number of tokens, counted backwards from e, that equal the history's last
// tokens counted backwards from L-1, capped at n_max.  An occurrence of length n ends at e exactly when
// m(e) >= n, so the longest ending that occurs anywhere is max_e m(e), and its most recent occurrence is the
// largest e that reaches it: one max-reduction over the key (m(e), e).
#include "common.h"

namespace specv {

__global__ __launch_bounds__(256) void ngram_draft_kernel(int k, int n_max, int n_min, const int32_t* __restrict__ hist,
                                                          int64_t hist_stride, int n_rows, const int32_t* __restrict__ hist_len,
                                                          const int32_t* __restrict__ seq_ids, int32_t* __restrict__ tokens,
                                                          int32_t* __restrict__ n_drafted)
{
    const int b = blockIdx.x;
    const int row = seq_ids ? seq_ids[b] : b;
    int32_t* out = tokens + (int64_t)b * (k + 1);
    int L = 0;
    if (row >= 0 && row < n_rows) {
        L = hist_len[row];
        if (L > hist_stride) L = (int)hist_stride;
    }
    if (L < 1) {                                            // wave-uniform: depends on the sequence only
        for (int i = threadIdx.x; i <= k; i += blockDim.x) out[i] = 0;
        if (threadIdx.x == 0 && n_drafted) n_drafted[b] = -1;
        return;
    }
    const int32_t* h = hist + (int64_t)row * hist_stride;
    int32_t tail[16];                                       // the ending, last token first
#pragma unroll
    for (int i = 0; i < 16; ++i) tail[i] = i < n_max && i < L ? h[L - 1 - i] : 0;

    unsigned long long best = 0;                            // (m << 32) | e, m >= 1; 0 = nothing
    for (int e = threadIdx.x; e <= L - 2; e += blockDim.x) {
        int m = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            // m counts the leading run of equal tokens: stop at the first difference
            if (i < n_max && i <= e && m == i && h[e - i] == tail[i]) m = i + 1;
        }
        unsigned long long key = ((unsigned long long)m << 32) | (unsigned int)e;
        if (m > 0 && key > best) best = key;
    }
    for (int off = 32; off > 0; off >>= 1) {
        unsigned long long o = __shfl_xor(best, off);
        if (o > best) best = o;
    }
    __shared__ unsigned long long s_best[4];
    if ((threadIdx.x & 63) == 0) s_best[threadIdx.x >> 6] = best;
    __syncthreads();
    best = s_best[0];
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) if (s_best[w] > best) best = s_best[w];

    const int m = (int)(best >> 32), e = (int)(best & 0xffffffffu);
    const int32_t last = h[L - 1];
    if (m < n_min) {
        for (int i = threadIdx.x; i <= k; i += blockDim.x) out[i] = last;
        if (threadIdx.x == 0 && n_drafted) n_drafted[b] = 0;
        return;
    }
    const int start = e + 1;                                // first token behind the occurrence
    int c = L - start;
    if (c > k) c = k;
    for (int i = threadIdx.x; i <= k; i += blockDim.x) {
        if (i == 0) out[0] = last;
        else out[i] = h[start + (i - 1 < c ? i - 1 : c - 1)];
    }
    if (threadIdx.x == 0 && n_drafted) n_drafted[b] = c;
}

__global__ void ngram_append_kernel(int B, int k, int32_t* __restrict__ hist, int64_t hist_stride, int n_rows,
                                    int32_t* __restrict__ hist_len, const int32_t* __restrict__ seq_ids,
                                    const int32_t* __restrict__ out_tokens, const int32_t* __restrict__ accept_len)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int row = seq_ids ? seq_ids[b] : b;
    if (row < 0 || row >= n_rows) return;
    int n = accept_len[b];
    n = n < 0 ? 0 : (n > k ? k : n);
    int L = hist_len[row];
    if (L < 0) L = 0;
    int32_t* h = hist + (int64_t)row * hist_stride;
    for (int i = 0; i <= n && L < hist_stride; ++i) h[L++] = out_tokens[(int64_t)b * (k + 1) + i];
    hist_len[row] = L;
}

}  // namespace specv

extern "C" spec_status spec_ngram_draft(int32_t B, int32_t k, int32_t n_max, int32_t n_min, const int32_t* dev_hist,
                                        int64_t hist_stride, int32_t n_rows, const int32_t* dev_hist_len,
                                        const int32_t* dev_seq_ids, int32_t* dev_tokens, int32_t* dev_n_drafted, void* stream)
{
    using namespace specv;
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_ngram_draft: B or k out of range"); return SPEC_EINVAL; }
    if (n_min < 1 || n_max < n_min || n_max > 16) { set_error("spec_ngram_draft: need 1 <= n_min <= n_max <= 16"); return SPEC_EINVAL; }
    if (hist_stride < 1 || n_rows < 1) { set_error("spec_ngram_draft: empty history array"); return SPEC_EINVAL; }
    if (!dev_hist || !dev_hist_len || !dev_tokens) { set_error("spec_ngram_draft: null pointer"); return SPEC_EINVAL; }
    ngram_draft_kernel<<<(unsigned)B, 256, 0, (hipStream_t)stream>>>(k, n_max, n_min, dev_hist, hist_stride, n_rows, dev_hist_len,
                                                                     dev_seq_ids, dev_tokens, dev_n_drafted);
    SPEC_LAUNCH_CHECK("ngram_draft_kernel");
    prof_mark(PC_NGRAM, (hipStream_t)stream);
    return SPEC_OK;
}

extern "C" spec_status spec_ngram_append(int32_t B, int32_t k, int32_t* dev_hist, int64_t hist_stride, int32_t n_rows,
                                         int32_t* dev_hist_len, const int32_t* dev_seq_ids, const int32_t* dev_out_tokens,
                                         const int32_t* dev_accept_len, void* stream)
{
    using namespace specv;
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_ngram_append: B or k out of range"); return SPEC_EINVAL; }
    if (hist_stride < 1 || n_rows < 1) { set_error("spec_ngram_append: empty history array"); return SPEC_EINVAL; }
    if (!dev_hist || !dev_hist_len || !dev_out_tokens || !dev_accept_len) { set_error("spec_ngram_append: null pointer"); return SPEC_EINVAL; }
    ngram_append_kernel<<<(unsigned)cdiv(B, 256), 256, 0, (hipStream_t)stream>>>(B, k, dev_hist, hist_stride, n_rows, dev_hist_len,
                                                                                  dev_seq_ids, dev_out_tokens, dev_accept_len);
    SPEC_LAUNCH_CHECK("ngram_append_kernel");
    prof_mark(PC_NGRAM, (hipStream_t)stream);
    return SPEC_OK;
}
