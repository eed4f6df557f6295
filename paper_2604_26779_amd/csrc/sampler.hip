// Fused vocabulary-wide softmax + lossless rejection sampling (the rejection procedure the
// paper's Section 2.1 relies on; acceptance length as defined in its Section 2.2).
//
// Three launches per step, the vocabulary cut into SAMP_PARTS ranges so that a batch of a few dozen
// sequences still occupies the whole chip (one workgroup per row or sequence left 7/8 of the CUs idle):
//   1. row_stats_kernel: workgroup = (logits row, range) -> (max, sum of exp) of logits / T over the range;
//   2. reject_scan_kernel: workgroup = (sequence, range): the accept tests in order (every range's workgroup
//      repeats these few scalar steps and arrives at the same n), then the exponential race over its range of
//      the single row that decides the emitted token (residual row at the first rejection, bonus row after k
//      acceptances) -> the range's best key;
//   3. reject_merge_kernel: the best key over the ranges, ties to the lowest token -> outputs.
// Only the rows' statistics, the k probed q entries and one q row are read: (k+1+2) V floats
// per sequence at most.
#include <mutex>

#include "common.h"

namespace specv {

constexpr int SAMP_THREADS = 1024;

struct Philox4 { uint32_t x, y, z, w; };

__device__ inline Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{c0, c1, c2, c3};
}

constexpr int SAMP_PARTS = 8;                 // ranges the vocabulary is cut into (whole groups of 4 entries: one Philox call each)

// groups of 4 vocabulary entries of range `part`: [g0, g1)
__device__ inline void part_groups(int V, int part, int* g0, int* g1)
{
    const int groups = (V + 3) >> 2, per = (groups + SAMP_PARTS - 1) / SAMP_PARTS;
    *g0 = part * per < groups ? part * per : groups;
    *g1 = (part + 1) * per < groups ? (part + 1) * per : groups;
}

// Everything a decision hangs on is fp64, as the definition has it: z = logit / T (a division, not a product with
// 1 / T), e = exp(z - max), p = e / sum, the accept test u * q < p, the race keys w / (-ln u).  With fp32 keys two
// candidates closer than 1e-6 relative could swap, and a residual p - q that cancels to a few ulps was noise; in fp64
// the choice differs from an fp64 reference's only where its own keys agree to 15 digits.  The cost is small: about 140
// fp64 instructions per vocabulary entry of the B rows that draw, 50 per entry of the statistics.

// (max, sum of exp) of one range of a row; the maximum of z is taken over the raw fp32 logits (z is monotone in them)
// (zero_rows != null: the workgroup also clears its eighth of row blockIdx.x of that array, zero_width entries wide - the
// q rows a mapped draft draw then fills at scattered positions)
__global__ __launch_bounds__(SAMP_THREADS) void row_stats_kernel(const float* __restrict__ logits, int64_t row_stride, int V, double T,
                                                                  double2* __restrict__ stats, float* __restrict__ zero_rows = nullptr,
                                                                  int64_t zero_stride = 0, int zero_width = 0)
{
    if (zero_rows) {
        const int per = (zero_width + SAMP_PARTS - 1) / SAMP_PARTS;
        const int z0 = blockIdx.y * per, z1 = z0 + per < zero_width ? z0 + per : zero_width;
        float* zr = zero_rows + (int64_t)blockIdx.x * zero_stride;
        for (int v = z0 + threadIdx.x; v < z1; v += SAMP_THREADS) zr[v] = 0.f;
    }
    const float* row = logits + (int64_t)blockIdx.x * row_stride;
    int g0, g1;
    part_groups(V, blockIdx.y, &g0, &g1);
    const int v1 = g1 * 4 < V ? g1 * 4 : V;
    __shared__ float lmax[SAMP_THREADS / 64];
    __shared__ double lsum[SAMP_THREADS / 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float mx = -INFINITY;
    for (int v = g0 * 4 + threadIdx.x; v < v1; v += SAMP_THREADS) {
        const float l = row[v];
        if (l > mx) mx = l;                                      // NaN compares false: left out, as below
    }
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) lmax[wave] = mx;
    __syncthreads();
    mx = lmax[0];
    for (int w = 1; w < SAMP_THREADS / 64; ++w) mx = fmaxf(mx, lmax[w]);
    const double m = (double)mx / T;
    double sum = 0.0;
    if (mx > -INFINITY) {
        for (int v = g0 * 4 + threadIdx.x; v < v1; v += SAMP_THREADS) {
            const float l = row[v];
            if (l > -INFINITY) sum += exp((double)l / T - m);
        }
    }
    // fixed order: butterfly inside a wavefront, then the 16 wavefronts one after the other
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) lsum[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double S = lsum[0];
        for (int w = 1; w < SAMP_THREADS / 64; ++w) S += lsum[w];
        stats[(int64_t)blockIdx.x * SAMP_PARTS + blockIdx.y] = make_double2(m, S);
    }
}

// a row's statistics from those of its ranges, in range order: M = max m_p, S = sum_p s_p exp(m_p - M)
__device__ inline double2 row_stat(const double2* __restrict__ stats, int64_t row)
{
    double M = -INFINITY;
    for (int p = 0; p < SAMP_PARTS; ++p) M = fmax(M, stats[row * SAMP_PARTS + p].x);
    double S = 0.0;
    for (int p = 0; p < SAMP_PARTS; ++p) {
        const double2 c = stats[row * SAMP_PARTS + p];
        if (c.y > 0.0) S += c.y * exp(c.x - M);
    }
    return make_double2(M, S);
}

// Exponential race over the groups [g0, g1) of one row.  Two races share the scan: the residual one (RES: weights
// max(0, p - q); HOT: p except 0 at the drafted token `hot`, the residual of a one-hot draft distribution) and the
// plain one over p = exp(z - m) / S, which decides the bonus row and stands in where a residual is identically zero.
template <bool RES, bool HOT>
__device__ inline void race_scan(const float* __restrict__ lrow, const float* __restrict__ qrow, int V, int g0, int g1, double T,
                                 double m, double S, uint32_t k0, uint32_t k1, uint32_t c1, uint32_t c2, uint32_t c3,
                                 double& best, int& best_v, double& best_res, int& best_res_v, int hot = -1)
{
    for (int g = g0 + threadIdx.x; g < g1; g += SAMP_THREADS) {
        Philox4 r = philox4x32_10((uint32_t)g, c1, c2, c3, k0, k1);
        uint32_t words[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int v = g * 4 + j;
            if (v >= V) break;
            const double pv = exp((double)lrow[v] / T - m) / S;
            if (!(pv > 0.0)) continue;
            const double u = ((double)(words[j] >> 9) + 0.5) * (1.0 / 8388608.0);
            const double nl = -log(u);
            const double key = pv / nl;
            if (key > best) { best = key; best_v = v; }     // v ascends inside a thread: ties keep the lowest
            if (RES || HOT) {
                const double w = RES ? fmax(0.0, pv - (double)qrow[v]) : (v == hot ? 0.0 : pv);
                if (w > 0.0) {
                    const double kr = w / nl;
                    if (kr > best_res) { best_res = kr; best_res_v = v; }
                }
            }
        }
    }
}

__device__ inline void argmax_merge(double& key, int& v, double key2, int v2)
{
    if (key2 > key || (key2 == key && v2 >= 0 && (v < 0 || v2 < v))) { key = key2; v = v2; }
}

__device__ inline void block_argmax(double& key, int& v, double* lk, int* lv)
{
    for (int off = 32; off > 0; off >>= 1) {
        double k2 = __shfl_xor(key, off);
        int v2 = __shfl_xor(v, off);
        argmax_merge(key, v, k2, v2);
    }
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) { lk[wave] = key; lv[wave] = v; }
    __syncthreads();
    key = lk[0]; v = lv[0];
    for (int w = 1; w < SAMP_THREADS / 64; ++w) argmax_merge(key, v, lk[w], lv[w]);
}

// what a range's workgroup hands to the merge: n, and its best (key, token) of the residual race and of the plain race
struct RacePart { int32_t n, v_res, v, pad; double key_res, key; };

__global__ __launch_bounds__(SAMP_THREADS) void reject_scan_kernel(
    int k, int V, const float* __restrict__ logits, const float* __restrict__ q, const int32_t* __restrict__ draft,
    double T, uint32_t seed_lo, uint32_t seed_hi, uint32_t step4, const double2* __restrict__ stats,
    RacePart* __restrict__ parts, float* __restrict__ dbg)
{
    const int b = blockIdx.x, part = blockIdx.y;
    const float* L = logits + (int64_t)b * (k + 1) * V;
    const float* Qb = q ? q + (int64_t)b * k * V : nullptr;
    __shared__ int s_n;
    __shared__ double2 s_st;
    __shared__ double lk[SAMP_THREADS / 64];
    __shared__ int lv[SAMP_THREADS / 64];

    if (threadIdx.x == 0) {
        int n = 0;
        const bool log_it = dbg && part == 0;
        for (int i = 0; i < k; ++i) {
            if (log_it) { float* d = dbg + ((int64_t)b * k + i) * 3; d[0] = d[1] = d[2] = NAN; }
        }
        for (int i = 0; i < k; ++i) {
            int x = draft[(int64_t)b * k + i];
            if (x < 0 || x >= V) break;
            const double2 st = row_stat(stats, (int64_t)b * (k + 1) + i);
            const double P = exp((double)L[(int64_t)i * V + x] / T - st.x) / st.y;
            const double Q = Qb ? (double)Qb[(int64_t)i * V + x] : 1.0;     // no q array: one-hot drafts (a deterministic drafter)
            Philox4 r = philox4x32_10(0u, (uint32_t)i, (uint32_t)b, step4 + 0u, seed_lo, seed_hi);
            const double u = (double)(r.x >> 8) * (1.0 / 16777216.0);
            if (log_it) { float* d = dbg + ((int64_t)b * k + i) * 3; d[0] = (float)P; d[1] = (float)Q; d[2] = (float)u; }
            if (u * Q < P) n += 1; else break;
        }
        s_n = n;
        s_st = row_stat(stats, (int64_t)b * (k + 1) + n);
    }
    __syncthreads();
    const int n = s_n;
    const double2 st = s_st;
    const float* lrow = L + (int64_t)n * V;
    int g0, g1;
    part_groups(V, part, &g0, &g1);
    double best = -1.0, best_res = -1.0;
    int best_v = -1, best_res_v = -1;
    const uint32_t c1 = (uint32_t)n, c2 = (uint32_t)b, c3 = step4 + 1u;
    if (n < k && Qb) race_scan<true, false>(lrow, Qb + (int64_t)n * V, V, g0, g1, T, st.x, st.y, seed_lo, seed_hi, c1, c2, c3, best, best_v, best_res, best_res_v);
    else if (n < k) race_scan<false, true>(lrow, nullptr, V, g0, g1, T, st.x, st.y, seed_lo, seed_hi, c1, c2, c3, best, best_v, best_res, best_res_v, draft[(int64_t)b * k + n]);
    else race_scan<false, false>(lrow, nullptr, V, g0, g1, T, st.x, st.y, seed_lo, seed_hi, c1, c2, c3, best, best_v, best_res, best_res_v);
    block_argmax(best, best_v, lk, lv);
    block_argmax(best_res, best_res_v, lk, lv);
    if (threadIdx.x == 0) {
        RacePart r;
        r.n = n; r.key_res = best_res; r.v_res = best_res_v; r.key = best; r.v = best_v; r.pad = 0;
        parts[(int64_t)b * SAMP_PARTS + part] = r;
    }
}

// one thread per sequence: the winner over the ranges (which ascend in token id, so an equal key never replaces an
// earlier one), the residual race's if it has one (n < k and a residual that is not identically zero), else the plain one's
__global__ void reject_merge_kernel(int B, int k, const RacePart* __restrict__ parts, const int32_t* __restrict__ draft,
                                    int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const RacePart* p = parts + (int64_t)b * SAMP_PARTS;
    const int n = p[0].n;
    double key = -1.0, key_res = -1.0;
    int v = -1, v_res = -1;
    for (int i = 0; i < SAMP_PARTS; ++i) {
        argmax_merge(key, v, p[i].key, p[i].v);
        argmax_merge(key_res, v_res, p[i].key_res, p[i].v_res);
    }
    const int y = (n < k && v_res >= 0) ? v_res : v;
    accept_len[b] = n;
    int32_t* o = out_tokens + (int64_t)b * (k + 1);
    for (int i = 0; i < n; ++i) o[i] = draft[(int64_t)b * k + i];
    o[n] = y;
    for (int i = n + 1; i <= k; ++i) o[i] = -1;
}

// The draft model's own draw, over the same SAMP_PARTS vocabulary ranges as the verifier's: q = softmax(logits / T)
// written out for the verifier (rounded to fp32 from the fp64 value), and x = argmax_v q_v / (-ln u_v) on random
// stream 2.  row_stats_kernel gives the ranges' (max, sum); draft_scan_kernel (workgroup = sequence, range) merges them,
// writes its range of q and finds its range's best key; draft_merge_kernel picks the token.
struct DraftPart { double key; int32_t v, pad; };

__global__ __launch_bounds__(SAMP_THREADS) void draft_scan_kernel(
    int V, const float* __restrict__ logits, int64_t logits_stride, double T, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t step4, uint32_t row, const double2* __restrict__ stats, float* __restrict__ q, int64_t q_stride,
    DraftPart* __restrict__ parts, const int32_t* __restrict__ token_map, int q_width)
{
    const int b = blockIdx.x, part = blockIdx.y;
    const float* lrow = logits + (int64_t)b * logits_stride;
    float* qrow = q + (int64_t)b * q_stride;
    __shared__ double lk[SAMP_THREADS / 64];
    __shared__ int lv[SAMP_THREADS / 64];
    __shared__ double2 s_st;
    if (threadIdx.x == 0) s_st = row_stat(stats, b);
    __syncthreads();
    const double m = s_st.x, S = s_st.y;
    int g0, g1;
    part_groups(V, part, &g0, &g1);
    double best = -1.0;
    int best_v = -1;
    for (int g = g0 + threadIdx.x; g < g1; g += SAMP_THREADS) {
        Philox4 r = philox4x32_10((uint32_t)g, row, (uint32_t)b, step4 + 2u, seed_lo, seed_hi);
        uint32_t words[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int v = g * 4 + j;
            if (v >= V) break;
            const double pv = exp((double)lrow[v] / T - m) / S;
            const int at = token_map ? token_map[v] : v;         // (a mapped row was cleared by the statistics kernel)
            if ((unsigned)at >= (unsigned)q_width) continue;     // a map entry outside the target's vocabulary: never written, never drawn
            qrow[at] = (float)pv;
            if (!(pv > 0.0)) continue;
            const double u = ((double)(words[j] >> 9) + 0.5) * (1.0 / 8388608.0);
            const double key = pv / (-log(u));
            if (key > best) { best = key; best_v = v; }
        }
    }
    block_argmax(best, best_v, lk, lv);
    if (threadIdx.x == 0) { DraftPart d; d.key = best; d.v = best_v; d.pad = 0; parts[(int64_t)b * SAMP_PARTS + part] = d; }
}

__global__ void draft_merge_kernel(int B, const DraftPart* __restrict__ parts, int32_t* __restrict__ tok_a, int stride_a,
                                   int32_t* __restrict__ tok_b, int stride_b, const int32_t* __restrict__ token_map)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    double key = -1.0;
    int v = -1;
    for (int i = 0; i < SAMP_PARTS; ++i) argmax_merge(key, v, parts[(int64_t)b * SAMP_PARTS + i].key, parts[(int64_t)b * SAMP_PARTS + i].v);
    if (token_map && v >= 0) v = token_map[v];
    if (tok_a) tok_a[(int64_t)b * stride_a] = v;
    if (tok_b) tok_b[(int64_t)b * stride_b] = v;
}

}  // namespace specv

// workspace: the ranges' row statistics [B * (k + 1)][SAMP_PARTS] double2, then the ranges' race results [B][SAMP_PARTS]
static size_t sample_stats_bytes(int64_t rows) { return specv::align_up((size_t)rows * specv::SAMP_PARTS * sizeof(double2), 256); }
static size_t sample_parts_bytes(int64_t B) { return specv::align_up((size_t)B * specv::SAMP_PARTS * sizeof(specv::RacePart), 256); }

extern "C" size_t spec_sample_workspace_bytes(int32_t B, int32_t k)
{
    if (B < 1 || k < 0) return 0;
    return sample_stats_bytes((int64_t)B * (k + 1)) + sample_parts_bytes(B);
}

namespace specv {

// argument checks and the launches shared by both entry points; ws: spec_sample_workspace_bytes(B, k) bytes of device memory
static spec_status reject_sample_launch(const char* who, int32_t B, int32_t k, int32_t V, const float* dev_logits, const float* dev_q,
                                        const int32_t* dev_draft_tokens, float temperature, uint64_t seed, uint64_t step,
                                        int32_t* dev_accept_len, int32_t* dev_out_tokens, float* dev_dbg, void* ws, hipStream_t s)
{
    double2* stats = (double2*)ws;
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT || V < 1) { set_error("%s: B, k or V out of range", who); return SPEC_EINVAL; }
    if (!(temperature > 0.f)) { set_error("%s: temperature must be > 0", who); return SPEC_EINVAL; }
    if (step >= (1ull << 30)) { set_error("%s: step must be < 2^30", who); return SPEC_EINVAL; }
    if (!dev_logits || !dev_accept_len || !dev_out_tokens || !ws || (k > 0 && !dev_draft_tokens)) {
        set_error("%s: null pointer", who); return SPEC_EINVAL;
    }
    const double T = (double)temperature;
    RacePart* parts = (RacePart*)((char*)ws + sample_stats_bytes((int64_t)B * (k + 1)));
    prof_mark(PC_OTHER, s);
    row_stats_kernel<<<dim3((unsigned)(B * (k + 1)), SAMP_PARTS), SAMP_THREADS, 0, s>>>(dev_logits, (int64_t)V, V, T, stats);
    SPEC_LAUNCH_CHECK("row_stats_kernel");
    prof_mark(PC_SAMPLE_STATS, s);
    reject_scan_kernel<<<dim3((unsigned)B, SAMP_PARTS), SAMP_THREADS, 0, s>>>(k, V, dev_logits, dev_q, dev_draft_tokens, T, (uint32_t)seed,
                                                                             (uint32_t)(seed >> 32), (uint32_t)(step * 4u), stats, parts, dev_dbg);
    SPEC_LAUNCH_CHECK("reject_scan_kernel");
    reject_merge_kernel<<<(unsigned)cdiv(B, 256), 256, 0, s>>>(B, k, parts, dev_draft_tokens, dev_accept_len, dev_out_tokens);
    SPEC_LAUNCH_CHECK("reject_merge_kernel");
    prof_mark(PC_SAMPLE_DRAW, s);
    return SPEC_OK;
}

// Workspace of spec_reject_sample_static: device memory that exists from the moment the library is loaded, so
// that entry point never allocates.  Every GPU holds its own copy at its own address; the array's name is only a
// host-side handle, the address kernels are given comes from hipGetSymbolAddress with that GPU current.
constexpr int SAMP_STATIC_ROWS = 4096;                  // B * (k + 1) at most: 512 KiB of row statistics + 1 MiB of race results (sized for k = 0, B = 4096) per GPU
constexpr size_t SAMP_STATIC_BYTES = (size_t)SAMP_STATIC_ROWS * SAMP_PARTS * (sizeof(double2) + sizeof(RacePart)) + 512;
static __device__ __align__(256) unsigned char scratch[SAMP_STATIC_BYTES];
constexpr int SAMP_MAX_DEVICES = 64;
static void* g_scratch_ptr[SAMP_MAX_DEVICES];
static std::mutex g_scratch_mutex;

static spec_status static_scratch(void** out)
{
    int dev = -1;
    SPEC_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= SAMP_MAX_DEVICES) { set_error("spec_reject_sample_static: device index %d is beyond %d", dev, SAMP_MAX_DEVICES - 1); return SPEC_EUNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { set_error("spec_reject_sample_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e)); return SPEC_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SPEC_OK;
}

}  // namespace specv

extern "C" spec_status spec_reject_sample(int32_t B, int32_t k, int32_t V, const float* dev_logits, const float* dev_q,
                                          const int32_t* dev_draft_tokens, float temperature, uint64_t seed,
                                          uint64_t step, int32_t* dev_accept_len, int32_t* dev_out_tokens,
                                          float* dev_dbg, void* dev_workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
    if (B >= 1 && k >= 0 && dev_workspace && workspace_bytes < spec_sample_workspace_bytes(B, k)) { set_error("spec_reject_sample: workspace too small"); return SPEC_EINVAL; }
    return reject_sample_launch("spec_reject_sample", B, k, V, dev_logits, dev_q, dev_draft_tokens, temperature, seed, step, dev_accept_len,
                                dev_out_tokens, dev_dbg, dev_workspace, (hipStream_t)stream);
}

extern "C" spec_status spec_reject_sample_static(int32_t B, int32_t k, int32_t V, const float* dev_logits, const float* dev_q,
                                                 const int32_t* dev_draft_tokens, float temperature, uint64_t seed,
                                                 uint64_t step, int32_t* dev_accept_len, int32_t* dev_out_tokens,
                                                 float* dev_dbg, void* stream)
{
    using namespace specv;
    if (B >= 1 && k >= 0 && k <= SPEC_MAX_DRAFT && (int64_t)B * (k + 1) > SAMP_STATIC_ROWS) {
        set_error("spec_reject_sample_static: B * (k + 1) = %lld rows exceed the built-in scratch of %d rows (use spec_reject_sample with a workspace)",
                  (long long)B * (k + 1), SAMP_STATIC_ROWS);
        return SPEC_EINVAL;
    }
    void* stats = nullptr;
    spec_status st = static_scratch(&stats);
    if (st != SPEC_OK) return st;
    return reject_sample_launch("spec_reject_sample_static", B, k, V, dev_logits, dev_q, dev_draft_tokens, temperature, seed, step,
                                dev_accept_len, dev_out_tokens, dev_dbg, stats, (hipStream_t)stream);
}

extern "C" size_t spec_draft_sample_workspace_bytes(int32_t B)
{
    if (B < 1) return 0;
    return sample_stats_bytes(B) + specv::align_up((size_t)B * specv::SAMP_PARTS * sizeof(specv::DraftPart), 256);
}

static spec_status draft_sample_launch(const char* who, int32_t B, int32_t V, const float* dev_logits, int64_t logits_row_stride,
                                       float temperature, uint64_t seed, uint64_t step, int32_t row,
                                       int32_t* dev_tokens_a, int32_t stride_a, int32_t* dev_tokens_b, int32_t stride_b,
                                       float* dev_q, int64_t q_row_stride, const int32_t* dev_token_map, int32_t q_width,
                                       void* dev_workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
    if (B < 1 || V < 1 || row < 0 || row > SPEC_MAX_DRAFT) { set_error("%s: B, V or row out of range", who); return SPEC_EINVAL; }
    if (!(temperature > 0.f)) { set_error("%s: temperature must be > 0", who); return SPEC_EINVAL; }
    if (step >= (1ull << 30)) { set_error("%s: step must be < 2^30", who); return SPEC_EINVAL; }
    if (!dev_logits || !dev_q || (!dev_tokens_a && !dev_tokens_b)) { set_error("%s: null pointer", who); return SPEC_EINVAL; }
    if (logits_row_stride < V || q_row_stride < q_width || (dev_tokens_a && stride_a < 1) || (dev_tokens_b && stride_b < 1)) {
        set_error("%s: a row stride is smaller than the row", who); return SPEC_EINVAL;
    }
    if (!dev_workspace || workspace_bytes < spec_draft_sample_workspace_bytes(B)) { set_error("%s: workspace missing or too small", who); return SPEC_EINVAL; }
    hipStream_t s = (hipStream_t)stream;
    prof_mark(PC_OTHER, s);
    double2* stats = (double2*)dev_workspace;
    DraftPart* parts = (DraftPart*)((char*)dev_workspace + sample_stats_bytes(B));
    const double T = (double)temperature;
    row_stats_kernel<<<dim3((unsigned)B, SAMP_PARTS), SAMP_THREADS, 0, s>>>(dev_logits, logits_row_stride, V, T, stats,
                                                                           dev_token_map ? dev_q : nullptr, q_row_stride, q_width);
    draft_scan_kernel<<<dim3((unsigned)B, SAMP_PARTS), SAMP_THREADS, 0, s>>>(V, dev_logits, logits_row_stride, T, (uint32_t)seed,
                                                                            (uint32_t)(seed >> 32), (uint32_t)(step * 4u), (uint32_t)row, stats,
                                                                            dev_q, q_row_stride, parts, dev_token_map, dev_token_map ? q_width : V);
    draft_merge_kernel<<<(unsigned)cdiv(B, 256), 256, 0, s>>>(B, parts, dev_tokens_a, stride_a, dev_tokens_b, stride_b, dev_token_map);
    SPEC_LAUNCH_CHECK("draft sampling kernels");
    prof_mark(PC_DRAFT_SAMPLE, s);
    return SPEC_OK;
}

extern "C" spec_status spec_draft_sample(int32_t B, int32_t V, const float* dev_logits, int64_t logits_row_stride,
                                         float temperature, uint64_t seed, uint64_t step, int32_t row,
                                         int32_t* dev_tokens_a, int32_t stride_a, int32_t* dev_tokens_b, int32_t stride_b,
                                         float* dev_q, int64_t q_row_stride, void* dev_workspace, size_t workspace_bytes, void* stream)
{
    return draft_sample_launch("spec_draft_sample", B, V, dev_logits, logits_row_stride, temperature, seed, step, row, dev_tokens_a, stride_a,
                               dev_tokens_b, stride_b, dev_q, q_row_stride, nullptr, V, dev_workspace, workspace_bytes, stream);
}

extern "C" spec_status spec_draft_sample_mapped(int32_t B, int32_t V_d, const float* dev_logits, int64_t logits_row_stride,
                                                float temperature, uint64_t seed, uint64_t step, int32_t row,
                                                int32_t* dev_tokens_a, int32_t stride_a, int32_t* dev_tokens_b, int32_t stride_b,
                                                float* dev_q, int64_t q_row_stride, const int32_t* dev_token_map, int32_t V_full,
                                                void* dev_workspace, size_t workspace_bytes, void* stream)
{
    if (!dev_token_map || V_full < V_d) { specv::set_error("spec_draft_sample_mapped: no token map, or V_full below V_d"); return SPEC_EINVAL; }
    return draft_sample_launch("spec_draft_sample_mapped", B, V_d, dev_logits, logits_row_stride, temperature, seed, step, row, dev_tokens_a,
                               stride_a, dev_tokens_b, stride_b, dev_q, q_row_stride, dev_token_map, V_full, dev_workspace, workspace_bytes, stream);
}

namespace specv {

// pending[b] = (tokens[b][n_b], out[b][n_b]) and tokens[b][0] = out[b][n_b]: the inputs of the next step
__global__ void next_inputs_kernel(int B, int k, int32_t* __restrict__ tokens, const int32_t* __restrict__ out_tokens,
                                   const int32_t* __restrict__ accept_len, int32_t* __restrict__ pending)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int n = accept_len[b];
    n = n < 0 ? 0 : (n > k ? k : n);
    int32_t last_input = tokens[(int64_t)b * (k + 1) + n];
    int32_t emitted = out_tokens[(int64_t)b * (k + 1) + n];
    if (pending) { pending[2 * b] = last_input; pending[2 * b + 1] = emitted; }
    tokens[(int64_t)b * (k + 1)] = emitted;
}

}  // namespace specv

namespace specv {

// pending_hidden[b] = (H[b][n-1] or its own old row 1 if n = 0, H[b][n]); workgroup = (batch entry, 1024 channels)
__global__ void next_hidden_kernel(int k, int d, const float* __restrict__ target_hidden, const int32_t* __restrict__ accept_len,
                                   float* __restrict__ pending_hidden)
{
    const int b = blockIdx.x;
    int n = accept_len[b];
    n = n < 0 ? 0 : (n > k ? k : n);
    const float* H = target_hidden + (int64_t)b * (k + 1) * d;
    float* p = pending_hidden + (int64_t)b * 2 * d;
    const int c_end = min(d, (int)(blockIdx.y + 1) * 1024);
    for (int c = blockIdx.y * 1024 + threadIdx.x; c < c_end; c += blockDim.x) {
        const float before_kept = n >= 1 ? H[(int64_t)(n - 1) * d + c] : p[d + c];     // read row 1 before it is overwritten
        const float before_emitted = H[(int64_t)n * d + c];
        p[c] = before_kept;
        p[d + c] = before_emitted;
    }
}

}  // namespace specv

extern "C" spec_status spec_next_step_hidden(int32_t B, int32_t k, int32_t d, const float* dev_target_hidden,
                                             const int32_t* dev_accept_len, float* dev_pending_hidden, void* stream)
{
    using namespace specv;
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT || d < 1) { set_error("spec_next_step_hidden: B, k or d out of range"); return SPEC_EINVAL; }
    if (!dev_target_hidden || !dev_accept_len || !dev_pending_hidden) { set_error("spec_next_step_hidden: null pointer"); return SPEC_EINVAL; }
    next_hidden_kernel<<<dim3((unsigned)B, (unsigned)cdiv(d, 1024)), 256, 0, (hipStream_t)stream>>>(k, d, dev_target_hidden, dev_accept_len, dev_pending_hidden);
    SPEC_LAUNCH_CHECK("next_hidden_kernel");
    return SPEC_OK;
}

extern "C" spec_status spec_next_step_inputs(int32_t B, int32_t k, int32_t* dev_tokens, const int32_t* dev_out_tokens,
                                             const int32_t* dev_accept_len, int32_t* dev_pending, void* stream)
{
    using namespace specv;
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_next_step_inputs: B or k out of range"); return SPEC_EINVAL; }
    if (!dev_tokens || !dev_out_tokens || !dev_accept_len) { set_error("spec_next_step_inputs: null pointer"); return SPEC_EINVAL; }
    next_inputs_kernel<<<(unsigned)cdiv(B, 256), 256, 0, (hipStream_t)stream>>>(B, k, dev_tokens, dev_out_tokens, dev_accept_len, dev_pending);
    SPEC_LAUNCH_CHECK("next_inputs_kernel");
    return SPEC_OK;
}
