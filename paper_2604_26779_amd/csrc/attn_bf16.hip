// Paged multi-query causal decode attention for the verify step (bf16 cache, head_dim 128).
//
// All (k+1) * G query rows that share a KV head (k+1 input positions x G query heads per KV head)
// ride on ONE pass over that head's cached keys and values: that sharing is what makes verifying
// k drafts cost about one decode step.  The pass is split along the context so that short and
// long sequences fill the machine evenly:
//   attn_plan_kernel    : once per forward pass (the contexts do not change between layers): the work list.  Every
//                         sequence's pages are cut into chunks of (nearly) equal length, the length chosen on the
//                         device, from the contexts the batch actually has, as the shortest for which the whole list
//                         still fits the number of workgroups the chip holds in the rounds asked for - so a small
//                         batch of ragged contexts fills every CU about equally instead of leaving a tail of
//                         half-empty rounds;
//   attn_partial_kernel : workgroup = (work item = chunk of a sequence's pages, kv head[, group of row blocks]); each of
//                         its 4 wavefronts walks every 4th page of the chunk with its own online softmax,
//                         reading K and V blocks straight into MFMA operand registers (the cache's
//                         in-block layout is the operand order, so every load is a contiguous
//                         1 KiB), two pages in flight per wavefront; every block is used for all the
//                         workgroup's 1..4 blocks of 16 query rows;
//                           S^T = K Q^T   v_mfma_f32_16x16x32_bf16 (keys x queries; Q as hi + lo bf16)
//                           O^T += V^T P^T v_mfma_f32_16x16x16_bf16 (P^T comes out of S^T's
//                                          accumulator layout without any shuffle);
//                         the wavefronts' results are merged through LDS and written as an
//                         un-normalised partial (O, reference point, sum).
//   attn_reduce_kernel  : merges the chunks of a (batch entry, kv head) and writes the bf16 result
//                         in the operand order the O-projection GEMM reads.
// Row r of a (batch entry, kv head) tile is input position r / G, query head kvh*G + r % G.
// Row i sees cache positions 0 .. ctx+i (causal over the k+1 new positions).
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "operand.h"

namespace specv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

constexpr int ATT_CP_MAX = 256;              // longest chunk (pages per workgroup): a wavefront's page ids sit in one register
constexpr int KV_ERR_BOUND = 8;              // error bit: more work items than the launch was sized for
constexpr int ATT_WAVES = 4;
constexpr int ATT_DEPTH = 3;                 // pages in flight per wavefront
constexpr int DH = 128;
constexpr int BLOCK_U4 = SPEC_PAGE_SIZE * DH * 2 / 16;   // 256 16-byte words per K or V block

// max / sum over the 4 lanes {l, l^16, l^32, l^48} with the two lane-swap instructions of gfx950 (rows of 16
// lanes, then halves of 32): plain vector ALU work, where a shuffle would take a round trip through the LDS
// crossbar on the softmax's critical path.  After a swap of x with itself the two results hold, lane by lane,
// the two values to combine.
__device__ inline float quad_max(float x)
{
    unsigned u = __float_as_uint(x);
    auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    u = __float_as_uint(x);
    auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ inline float quad_sum(float x)
{
    unsigned u = __float_as_uint(x);
    auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    u = __float_as_uint(x);
    auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// One work item: pages [page0, page_end) of batch entry b (sequence seq, cached length ctx, `total` keys visible to the
// last row; b = -1: unused slot of the list).  32 bytes, read with two 16-byte loads.
struct AttnItem { int32_t b, seq, page0, page_end, ctx, total, chunk, pad; };

// The work list of one forward pass.  One workgroup of 256.  pages(b) = pages holding the keys batch entry b may see
// (0 for a dropped entry).  Chunk length L: the smallest multiple of 4 in [min_pages, 256] with sum_b ceil(pages(b) / L)
// <= budget (256 if none; `forced` > 0 fixes L instead); entry b then has n = ceil(pages / L) items of
// ceil(pages / n) pages rounded up to a multiple of 4 (the 4 wavefronts take every 4th page).  Items are listed in batch
// order; entry_items[b] = (first item, number of items).  Slots of the list beyond the last item get b = -1.  More
// items than max_items (contexts beyond the bound the launch was sized for) set KV_ERR_BOUND and are dropped.
__global__ __launch_bounds__(256) void attn_plan_kernel(int B, int T, KvView kv, int budget, int min_pages, int forced, int max_items,
                                                        AttnItem* __restrict__ items, int2* __restrict__ entry_items)
{
    __shared__ int s_cnt[256];
    __shared__ int s_len, s_carry;
    auto pages_of = [&](int b, int* seq_o, int* ctx_o, int* total_o) {
        const int seq = kv.entry_seq[b];
        int ctx = 0, total = 0;
        if (seq >= 0) {
            ctx = kv.ctx_len[seq];
            total = ctx + T;
            const int cap = kv.n_held[seq] * SPEC_PAGE_SIZE;
            if (total > cap) total = cap;
        }
        if (seq_o) { *seq_o = seq; *ctx_o = ctx; *total_o = total; }
        return (total + SPEC_PAGE_SIZE - 1) / SPEC_PAGE_SIZE;
    };
    {
        // candidate j: chunks of 4 (j + 1) pages; thread t counts candidate t % 64 over the entries t / 64, t / 64 + 4, ...
        const int j = threadIdx.x & 63, len = 4 * (j + 1);
        int cnt = 0;
        for (int b = threadIdx.x >> 6; b < B; b += 4) cnt += (pages_of(b, nullptr, nullptr, nullptr) + len - 1) / len;
        s_cnt[threadIdx.x] = cnt;
        __syncthreads();
        if (threadIdx.x == 0) {
            int best = ATT_CP_MAX;
            for (int c = 63; c >= 0; --c) {
                const int l = 4 * (c + 1);
                if (l >= min_pages && s_cnt[c] + s_cnt[c + 64] + s_cnt[c + 128] + s_cnt[c + 192] <= budget) best = l;
            }
            s_len = forced > 0 ? forced : best;
            s_carry = 0;
        }
        __syncthreads();
    }
    const int L = s_len;
    for (int base = 0; base < B; base += 256) {
        const int b = base + threadIdx.x;
        int seq = -1, ctx = 0, total = 0;
        const int p = b < B ? pages_of(b, &seq, &ctx, &total) : 0;
        const int n = (p + L - 1) / L;
        // exclusive scan of n over the workgroup
        s_cnt[threadIdx.x] = n;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int add = (int)threadIdx.x >= off ? s_cnt[threadIdx.x - off] : 0;
            __syncthreads();
            s_cnt[threadIdx.x] += add;
            __syncthreads();
        }
        const int first = s_carry + s_cnt[threadIdx.x] - n, group_total = s_cnt[255];
        __syncthreads();
        if (b < B) {
            const int len = n > 0 ? ((p + n - 1) / n + ATT_WAVES - 1) / ATT_WAVES * ATT_WAVES : 0;
            int wrote = 0;
            for (int c = 0; c < n; ++c) {
                const int it = first + c;
                if (it >= max_items) break;
                AttnItem a;
                a.b = b; a.seq = seq; a.page0 = c * len; a.page_end = (c + 1) * len < p ? (c + 1) * len : p;
                a.ctx = ctx; a.total = total; a.chunk = c; a.pad = 0;
                items[it] = a;
                ++wrote;
            }
            entry_items[b] = make_int2(first < max_items ? first : 0, wrote);
            if (wrote < n) atomicOr(kv.error, KV_ERR_BOUND);
        }
        if (threadIdx.x == 0) s_carry += group_total;
        __syncthreads();
    }
    const int n_items = s_carry < max_items ? s_carry : max_items;
    for (int it = n_items + threadIdx.x; it < max_items; it += 256) {
        AttnItem a;
        a.b = -1; a.seq = -1; a.page0 = 0; a.page_end = 0; a.ctx = 0; a.total = 0; a.chunk = 0; a.pad = 0;
        items[it] = a;
    }
}

// part_o : [item * Hkv + kv head][rows][128] fp32, part_ml : [..][rows][2] (reference point in log2 domain, sum relative
// to it); rows = attn_rows_padded(R)
// A workgroup takes NRB (1..4) blocks of 16 query rows.  What does not fit in registers for 4 of them moves: the
// queries (hi + lo) sit in LDS in operand order and are re-read per page (double buffered, one row block ahead),
// the accumulators of all row blocks stay in registers.  More than 64 query rows per kv head (deep drafts with many
// query heads per kv head) are split into RG groups of NRB row blocks, one workgroup each; the groups of a (batch
// entry, kv head, chunk) re-read the same pages, so they are placed on the same XCD (workgroups go to XCDs
// round-robin by linear id: blockIdx.x spans a multiple of 8 values - kv head and the low bits of the item index -
// and the row group sits in blockIdx.y, 8 ids apart) and next to each other in dispatch order: the repeated reads
// hit that XCD's L2.
// The page loop is a run-time loop over groups of ATT_DEPTH pages (the register ring needs compile-time slots,
// nothing else does), so the code stays a few KiB whatever the chunk length; a wavefront's physical page ids sit
// in one register, lane j holding its j-th page, and are broadcast with v_readlane.  Pages that need masks (those
// reaching into the new positions, or past the end of the sequence: the last one or two) are left out of the
// pipelined loop and done last.
// KV8: the blocks hold E4M3 codes (half the bytes, two MFMA fragments per 16-byte word); a page's codes are widened to
// bf16 in registers once (exact: 3 mantissa bits) and feed the same MFMAs.  The key scale of the (layer, kv head) is
// folded into the score scale here, the value scale into the final normalisation (attn_reduce_kernel).
template <int NRB, bool KV8>
__global__ __launch_bounds__(256, NRB <= 2 ? 2 : 1) void attn_partial_kernel(
    const float* __restrict__ q, int T, int G, int Hq, const AttnItem* __restrict__ items, int max_items, KvView kv,
    int layer_pool, int layer, float scale_log2_in, int RG, int rows, int Hkv, int IP,
    float* __restrict__ part_o, float* __restrict__ part_ml)
{
    const int kvh = blockIdx.x % Hkv, rb0 = (blockIdx.y % RG) * NRB;
    const int it = (blockIdx.y / RG) * IP + blockIdx.x / Hkv;
    if (it >= max_items) return;
    int b, seq, page0, page_end, ctx, total;
    {
        const int4 i0 = ((const int4*)items)[2 * it], i1 = ((const int4*)items)[2 * it + 1];
        b = i0.x; seq = i0.y; page0 = i0.z; page_end = i0.w; ctx = i1.x; total = i1.y;
    }
    if (b < 0 || seq < 0 || page0 >= page_end) return;
    int plain_end = ctx / SPEC_PAGE_SIZE;          // pages before this one are visible to every row, every slot valid
    if (plain_end > page_end) plain_end = page_end;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int lq = lane & 15, lg = lane >> 4;
    const int R = T * G;
    const float scale_log2 = KV8 ? scale_log2_in * kv.k_scale[layer * Hkv + kvh] : scale_log2_in;

    __shared__ u32x4_t s_q[NRB][4][2][64];                      // [row block][32 channels][hi | lo][lane]
    __shared__ float s_o[ATT_WAVES][8][64][4];
    __shared__ float s_m[ATT_WAVES][16], s_l[ATT_WAVES][16];
    for (int f = wave; f < NRB * 4; f += ATT_WAVES) {
        const int rb = f >> 2, sgm = f & 3;
        const int r = (rb0 + rb) * 16 + lq;
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (r < R) {
            const float* src = q + ((int64_t)(b * T + r / G) * Hq + kvh * G + r % G) * DH + lg * 8 + sgm * 32;
            float4 a = *(const float4*)src, c = *(const float4*)(src + 4);
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c.x; v[5] = c.y; v[6] = c.z; v[7] = c.w;
        }
        uint4 h4, l4;
        split8(v, h4, l4);
        s_q[rb][sgm][0][lane] = u32x4_t{h4.x, h4.y, h4.z, h4.w};
        s_q[rb][sgm][1][lane] = u32x4_t{l4.x, l4.y, l4.z, l4.w};
    }
    int row_limit[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        int r = (rb0 + rb) * 16 + lq;
        row_limit[rb] = r < R ? ctx + r / G : -1;
    }

    const int32_t* pt = kv.page_table + (int64_t)seq * kv.max_pages;
    const u32x4_t* pool = (const u32x4_t*)kv.pool;
    const int64_t layer_base = (int64_t)layer_pool * kv.n_pages;
    auto block_ptr = [&](int physical_page, int is_v) {
        return pool + ((((layer_base + physical_page) * 2 + is_v) * Hkv + kvh) * (KV8 ? BLOCK_U4 / 2 : BLOCK_U4)) + lane;
    };
    // lane j: physical id of this wavefront's j-th page (chunk_pages <= 256: at most 64 per wavefront), clamped to the chunk
    int my_pid;
    {
        int pg = page0 + wave + ATT_WAVES * lane;
        my_pid = pt[pg < page_end ? pg : page_end - 1];
    }
    auto pid_at = [&](int it) { return __builtin_amdgcn_readlane(my_pid, it < 63 ? it : 63); };

    float mrow[NRB], lrow[NRB];
    f32x4_t oacc[NRB][8];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        mrow[rb] = -INFINITY;
        lrow[rb] = 0.f;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) oacc[rb][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    constexpr int NF = KV8 ? 2 : 4;                   // 16-byte words per lane and block
    u32x4_t kf[ATT_DEPTH][NF], vf[ATT_DEPTH][NF];
    auto load_page = [&](int slot, int physical_page) {
        const u32x4_t* kp = block_ptr(physical_page, 0);
        const u32x4_t* vp = block_ptr(physical_page, 1);
#pragma unroll
        for (int s = 0; s < NF; ++s) kf[slot][s] = __builtin_nontemporal_load(kp + s * 64);
#pragma unroll
        for (int s = 0; s < NF; ++s) vf[slot][s] = __builtin_nontemporal_load(vp + s * 64);
    };
    // fragment i (8 bf16) of a block held as codes: the i-th group of 8 bytes
    auto widen = [&](const u32x4_t (&f)[NF], int i) {
        if constexpr (KV8) {
            const unsigned int wa = f[i >> 1][(i & 1) * 2], wb = f[i >> 1][(i & 1) * 2 + 1];
            return u32x4_t{__builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wa, 1.0f, false)),
                           __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wa, 1.0f, true)),
                           __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wb, 1.0f, false)),
                           __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wb, 1.0f, true))};
        } else {
            return f[i];
        }
    };
    __syncthreads();                                  // the queries are in LDS

    // query fragments of one row block, double buffered: those of the next row block (of the next page after the
    // last) are read from LDS while the softmax of the current one runs
    bf16x8_t qh[2][4], ql[2][4];
    auto load_q = [&](int buf, int rb) {
#pragma unroll
        for (int sg = 0; sg < 4; ++sg) {
            qh[buf][sg] = __builtin_bit_cast(bf16x8_t, s_q[rb][sg][0][lane]);
            ql[buf][sg] = __builtin_bit_cast(bf16x8_t, s_q[rb][sg][1][lane]);
        }
    };
    load_q(0, 0);

    // One page for all row blocks.  The exponentials are taken against a reference point per row, which only has to
    // keep them in range; three ways of handling it (MODE):
    //   REF_INIT  : first page of the wavefront - the reference becomes this page's row maximum;
    //   REF_FIXED : the reference stays where it is, whatever the scores (fp32 has 2^127 of headroom; the largest
    //               exponent seen is tracked in mrel and checked after the loop).  No branch, no rescaling: the
    //               accumulators are touched by MFMAs only, which is what lets them stay in the accumulation
    //               registers without copies;
    //   REF_ADAPT : the reference follows the running maximum in steps of 2^8 and the accumulators are rescaled in
    //               place when it moves (masked pages, and the recomputation after an exponent check failed).
    constexpr int REF_INIT = 0, REF_FIXED = 1, REF_ADAPT = 2;
    float mrel[NRB];                                  // largest (score - reference) this lane has seen, log2 units
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) mrel[rb] = -INFINITY;
    auto process = [&](auto mask_c, auto mode_c, int slot, int logical_page) {
        constexpr bool need_mask = decltype(mask_c)::value;
        constexpr int MODE = decltype(mode_c)::value;
        const int key0 = logical_page * SPEC_PAGE_SIZE + lg * 4;
        u32x4_t kcur[4], vcur[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { kcur[i] = widen(kf[slot], i); vcur[i] = widen(vf[slot], i); }
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            // the three phases of a row block are pinned in this order (left alone, the scheduler hoists the query
            // reads of all row blocks to the top of the page and runs out of registers)
            __builtin_amdgcn_sched_barrier(0);
            f32x4_t sacc = {0.f, 0.f, 0.f, 0.f}, sacc2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sg = 0; sg < 4; ++sg) {
                const bf16x8_t kk = __builtin_bit_cast(bf16x8_t, kcur[sg]);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, qh[rb & 1][sg], sacc, 0, 0, 0);
                sacc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk, ql[rb & 1][sg], sacc2, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            load_q((rb + 1 < NRB ? rb + 1 : 0) & 1, rb + 1 < NRB ? rb + 1 : 0);
            __builtin_amdgcn_sched_barrier(0);
            sacc += sacc2;
            float sv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sv[j] = sacc[j] * scale_log2;
                if (need_mask && key0 + j > row_limit[rb]) sv[j] = -INFINITY;
            }
            if (MODE != REF_FIXED) {
                const float mx = quad_max(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])));
                if (MODE == REF_INIT) {
                    mrow[rb] = mx;
                } else if (__builtin_amdgcn_ballot_w64(mx > mrow[rb] + 8.0f) != 0) {
                    // the accumulators were last written by MFMAs of the previous page: far more than the 18 wait
                    // states an accumulator read needs after one, but the assembler block is opaque to the
                    // compiler's hazard pass, so spell them out
                    asm volatile("s_nop 15\n\ts_nop 15");
                    const float mnew = fmaxf(mrow[rb], mx);
                    const float alpha = mnew > -INFINITY ? __builtin_amdgcn_exp2f(mrow[rb] - mnew) : 1.0f;
                    mrow[rb] = mnew;
                    lrow[rb] *= alpha;
#pragma unroll
                    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            // in place, in the accumulation registers
                            float t;
                            asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %2, %1\n\tv_accvgpr_write_b32 %0, %1"
                                         : "+a"(oacc[rb][cb][j]), "=&v"(t) : "v"(alpha));
                        }
                }
            }
            const float msafe = mrow[rb] > -INFINITY ? mrow[rb] : 0.f;
            float p[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float e = sv[j] - msafe;
                if (MODE == REF_FIXED) mrel[rb] = fmaxf(mrel[rb], e);
                p[j] = __builtin_amdgcn_exp2f(e);
            }
            lrow[rb] += (p[0] + p[1]) + (p[2] + p[3]);
            unsigned int h01, l01, h23, l23;
            split2(p[0], p[1], h01, l01);
            split2(p[2], p[3], h23, l23);
            const s16x4_t pb = __builtin_bit_cast(s16x4_t, u32x2_t{h01, h23});
            const s16x4_t pl = __builtin_bit_cast(s16x4_t, u32x2_t{l01, l23});
            s16x4_t va[4], vb[4];
#pragma unroll
            for (int cp = 0; cp < 4; ++cp) {
                u32x4_t v = vcur[cp];
                if (need_mask) {
                    unsigned int m01 = (key0 + 0 < total ? 0x0000ffffu : 0u) | (key0 + 1 < total ? 0xffff0000u : 0u);
                    unsigned int m23 = (key0 + 2 < total ? 0x0000ffffu : 0u) | (key0 + 3 < total ? 0xffff0000u : 0u);
                    v.x &= m01; v.y &= m23; v.z &= m01; v.w &= m23;
                }
                va[cp] = __builtin_bit_cast(s16x4_t, u32x2_t{v.x, v.y});
                vb[cp] = __builtin_bit_cast(s16x4_t, u32x2_t{v.z, v.w});
            }
#pragma unroll
            for (int cp = 0; cp < 4; ++cp) {
                oacc[rb][2 * cp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[cp], pb, oacc[rb][2 * cp], 0, 0, 0);
                oacc[rb][2 * cp + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb[cp], pb, oacc[rb][2 * cp + 1], 0, 0, 0);
            }
#pragma unroll
            for (int cp = 0; cp < 4; ++cp) {
                oacc[rb][2 * cp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[cp], pl, oacc[rb][2 * cp], 0, 0, 0);
                oacc[rb][2 * cp + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb[cp], pl, oacc[rb][2 * cp + 1], 0, 0, 0);
            }
        }
    };
    using plain_t = std::false_type;
    using masked_t = std::true_type;
    using init_t = std::integral_constant<int, REF_INIT>;
    using fixed_t = std::integral_constant<int, REF_FIXED>;
    using adapt_t = std::integral_constant<int, REF_ADAPT>;

    // mask-free pages of this wavefront: page0 + wave + 4 * it, it < n_plain.  Ring of ATT_DEPTH pages (page `it` in
    // slot it % 3); the first page sets the reference points, the main loop then takes whole groups of three pages
    // and has no branch in its body, so that the compiler can count the loads in flight exactly; the last one or two
    // pages follow it.  Loads past the wavefront's last page re-read its clamped id (cache hits, results unused).
    static_assert(ATT_DEPTH == 3, "the loop body below is written for a ring of 3");
    const int n_plain = plain_end > page0 + wave ? (plain_end - page0 - wave + ATT_WAVES - 1) / ATT_WAVES : 0;
    auto lpage_of = [&](int it) { return page0 + wave + ATT_WAVES * it; };
    if (n_plain > 0) {
        load_page(0, pid_at(0));
        load_page(1, pid_at(1));
        load_page(2, pid_at(2));
        process(plain_t{}, init_t{}, 0, lpage_of(0));
        int it = 1;
        for (; it + 3 <= n_plain; it += 3) {
            load_page(0, pid_at(it + 2));
            process(plain_t{}, fixed_t{}, 1, lpage_of(it));
            load_page(1, pid_at(it + 3));
            process(plain_t{}, fixed_t{}, 2, lpage_of(it + 1));
            load_page(2, pid_at(it + 4));
            process(plain_t{}, fixed_t{}, 0, lpage_of(it + 2));
        }
        if (it < n_plain) process(plain_t{}, fixed_t{}, 1, lpage_of(it));
        if (it + 1 < n_plain) process(plain_t{}, fixed_t{}, 2, lpage_of(it + 1));
        // exponent check: 2^100 per term leaves room for the sums; beyond it, start over with the moving reference
        bool redo = false;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) redo = redo || mrel[rb] > 100.0f;
        if (__builtin_amdgcn_ballot_w64(redo) != 0) {
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                mrow[rb] = -INFINITY;
                lrow[rb] = 0.f;
#pragma unroll
                for (int cb = 0; cb < 8; ++cb) oacc[rb][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            }
            for (int it2 = 0; it2 < n_plain; ++it2) {
                load_page(0, pid_at(it2));
                process(plain_t{}, adapt_t{}, 0, lpage_of(it2));
            }
        }
    }
    // masked pages of the chunk (at most two in all: T <= 16), each by the wavefront whose turn it is
    {
        const int t0 = plain_end > page0 ? plain_end : page0;
        for (int lp = t0 + ((wave - (t0 - page0)) & (ATT_WAVES - 1)); lp < page_end; lp += ATT_WAVES) {
            load_page(0, pt[lp]);
            process(masked_t{}, adapt_t{}, 0, lp);
        }
    }

#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) lrow[rb] = quad_sum(lrow[rb]);

    // merge the 4 wavefronts through LDS, one row block at a time
    const int64_t item = (int64_t)it * Hkv + kvh;
    float* po = part_o + item * rows * DH;
    float* pml = part_ml + item * rows * 2;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) s_o[wave][cb][lane][j] = oacc[rb][cb][j];
        if (lg == 0) { s_m[wave][lq] = mrow[rb]; s_l[wave][lq] = lrow[rb]; }
        __syncthreads();
        for (int e = threadIdx.x; e < 8 * 64; e += 256) {
            int l2 = e & 63, cb = e >> 6;
            int row = l2 & 15;
            float mw[ATT_WAVES], M = -INFINITY;
#pragma unroll
            for (int w = 0; w < ATT_WAVES; ++w) { mw[w] = s_m[w][row]; M = fmaxf(M, mw[w]); }
            float o4[4] = {0.f, 0.f, 0.f, 0.f}, L = 0.f;
#pragma unroll
            for (int w = 0; w < ATT_WAVES; ++w) {
                float f = mw[w] > -INFINITY ? exp2f(mw[w] - M) : 0.f;
                L += f * s_l[w][row];
#pragma unroll
                for (int j = 0; j < 4; ++j) o4[j] += f * s_o[w][cb][l2][j];
            }
            int r = (rb0 + rb) * 16 + row, c = cb * 16 + (l2 >> 4) * 4;
            *(float4*)(po + (int64_t)r * DH + c) = make_float4(o4[0], o4[1], o4[2], o4[3]);
            if (cb == 0 && (l2 >> 4) == 0) { pml[r * 2] = M; pml[r * 2 + 1] = L; }
        }
        __syncthreads();
    }
}

// one thread per (batch entry, kv head, row, 8 channels): merge chunks, normalise, write the bf16
// operand of the O projection: xp[k-step][m-block][lane][8] with k = head*128 + channel
__global__ void attn_reduce_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml, int B, int T,
                                   int G, int Hkv, int RBrows, const int2* __restrict__ entry_items,
                                   KvView kv, int layer, int mb_pad, int xf, uint4* __restrict__ xp)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int R = T * G;
    int64_t total = (int64_t)B * Hkv * R * (DH / 8);
    if (idx >= total) return;
    int c8 = (int)(idx % (DH / 8));
    int r = (int)((idx / (DH / 8)) % R);
    int kvh = (int)((idx / (DH / 8) / R) % Hkv);
    int b = (int)(idx / (DH / 8) / R / Hkv);
    const int2 mine = entry_items[b];                        // (first item, number of items) of this batch entry
    const int n_chunks = mine.y;
    auto slot = [&](int c) { return ((int64_t)(mine.x + c) * Hkv + kvh) * RBrows + r; };
    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, part_ml[slot(c) * 2]);
    float L = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < n_chunks; ++c) {
        float mc = part_ml[slot(c) * 2];
        float f = mc > -INFINITY ? exp2f(mc - M) : 0.f;      // branch-free: the loads of all chunks overlap
        L += f * part_ml[slot(c) * 2 + 1];
        const float4* src = (const float4*)(part_o + slot(c) * DH + c8 * 8);
        float4 a = src[0], d = src[1];
        o[0] += f * a.x; o[1] += f * a.y; o[2] += f * a.z; o[3] += f * a.w;
        o[4] += f * d.x; o[5] += f * d.y; o[6] += f * d.z; o[7] += f * d.w;
    }
    float inv = L > 0.f ? 1.0f / L : 0.f;
    if (kv.fp8) inv *= kv.v_scale[layer * Hkv + kvh];     // 8-bit cache: the values were accumulated as codes
    float res[8];
    for (int j = 0; j < 8; ++j) res[j] = o[j] * inv;
    xp_store8_rt(xp, xf, b * T + r / G, (kvh * G + r % G) * DH + c8 * 8, mb_pad, res);
}

// How R query rows per kv head are laid over workgroups: RG groups of NRB row blocks, NRB <= 4 and as equal as
// possible (tuning parameter attn_row_blocks = 1..4 caps NRB instead).  How the contexts are cut into work items is
// decided on the device (attn_plan_kernel); the host only gives the budget - the workgroups the chip holds at once
// times attn_rounds, per kv head and row group - and sizes the list: at most max(budget, B * ceil(longest context /
// 256 pages)) items, the host's bound on the longest context standing in for all of them.  attn_chunk_pages (a multiple
// of 4, at most 256) fixes the chunk length instead.
struct AttnPlan { int RB, RG, budget, forced, max_items; };
static AttnPlan attn_plan(int R, int B, int Hkv, int pages_bound)
{
    const int blocks = (int)cdiv(R, 16);
    const int forced_rb = tune("attn_row_blocks");
    AttnPlan p;
    if (forced_rb >= 1 && forced_rb <= 4) {
        p.RB = forced_rb < blocks ? forced_rb : blocks;
        p.RG = (int)cdiv(blocks, p.RB);
    } else {
        p.RG = (int)cdiv(blocks, 4);
        p.RB = (int)cdiv(blocks, p.RG);
    }
    const int64_t slots = 256 * (p.RB <= 2 ? 2 : 1);         // workgroups resident at once
    int rounds = tune("attn_rounds");
    if (rounds < 1) rounds = 1;
    p.budget = (int)std::max<int64_t>(1, slots * rounds / ((int64_t)Hkv * p.RG));
    const int cp = tune("attn_chunk_pages");
    p.forced = (cp >= ATT_WAVES && cp <= ATT_CP_MAX && cp % ATT_WAVES == 0) ? cp : 0;
    const int64_t by_length = (int64_t)B * cdiv(pages_bound, p.forced ? p.forced : ATT_CP_MAX);
    p.max_items = (int)(p.forced ? by_length : std::max<int64_t>(p.budget, by_length));
    return p;
}

// the most work items a forward pass over B entries of at most pages_bound pages may have: sizes the item list and the
// partial-result buffers
int attn_max_items(int R, int B, int Hkv, int pages_bound) { return attn_plan(R, B, Hkv, pages_bound).max_items; }

// rows of a partial tile for R query rows per kv head: enough for every layout above (the workspace is sized before
// the tuning parameters are final)
int attn_rows_padded(int R)
{
    const int blocks = (int)cdiv(R, 16);
    int most = blocks;
    for (int n = 1; n <= 4 && n <= blocks; ++n) most = std::max(most, (int)cdiv(blocks, n) * n);
    return most * 16;
}

size_t attn_item_bytes() { return sizeof(AttnItem); }

// once per forward pass, after the page reservation: the work list of all its attention launches
spec_status launch_attention_plan(int B, int T, int G, int Hkv, const KvView& kv, int pages_bound, void* items, void* entry_items, hipStream_t s)
{
    const AttnPlan pl = attn_plan(T * G, B, Hkv, pages_bound);
    int min_pages = tune("attn_min_pages");
    if (min_pages < ATT_WAVES) min_pages = ATT_WAVES;
    attn_plan_kernel<<<1, 256, 0, s>>>(B, T, kv, pl.budget, min_pages, pl.forced, pl.max_items, (AttnItem*)items, (int2*)entry_items);
    SPEC_LAUNCH_CHECK("attn_plan_kernel");
    return SPEC_OK;
}

spec_status launch_attention_bf16(const float* q, int B, int T, int G, int Hq, int Hkv, const KvView& kv, int layer_pool, int layer,
                                  int pages_bound, const void* items, const void* entry_items, float* part_o, float* part_ml,
                                  int mb_pad, int xf_out, bf16_t* xp_out, hipStream_t s)
{
    int R = T * G;
    if (R > 256) { set_error("attention: (k+1) * (query heads per kv head) = %d rows exceeds 256", R); return SPEC_EUNSUPPORTED; }
    const int rows = attn_rows_padded(R);
    const AttnPlan pl = attn_plan(R, B, Hkv, pages_bound);
    const int RG = pl.RG;
    float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
    int IP = 1;                                   // items folded into blockIdx.x so that it spans a multiple of 8
    while ((Hkv * IP) % 8 != 0) IP *= 2;
    dim3 grid((unsigned)(Hkv * IP), (unsigned)(RG * cdiv(pl.max_items, IP)));
    const AttnItem* it = (const AttnItem*)items;
#define SPEC_ATTN_LAUNCH(NRBV) do { \
        if (kv.fp8) attn_partial_kernel<NRBV, true><<<grid, 256, 0, s>>>(q, T, G, Hq, it, pl.max_items, kv, layer_pool, layer, scale_log2, RG, rows, Hkv, IP, part_o, part_ml); \
        else attn_partial_kernel<NRBV, false><<<grid, 256, 0, s>>>(q, T, G, Hq, it, pl.max_items, kv, layer_pool, layer, scale_log2, RG, rows, Hkv, IP, part_o, part_ml); \
    } while (0)
    switch (pl.RB) {
    case 1: SPEC_ATTN_LAUNCH(1); break;
    case 2: SPEC_ATTN_LAUNCH(2); break;
    case 3: SPEC_ATTN_LAUNCH(3); break;
    default: SPEC_ATTN_LAUNCH(4); break;
    }
#undef SPEC_ATTN_LAUNCH
    SPEC_LAUNCH_CHECK("attn_partial_kernel");
    prof_mark(PC_ATTN, s);
    int64_t total = (int64_t)B * Hkv * R * (DH / 8);
    attn_reduce_kernel<<<(unsigned)cdiv(total, 256), 256, 0, s>>>(part_o, part_ml, B, T, G, Hkv, rows, (const int2*)entry_items, kv,
                                                                  layer, mb_pad, xf_out, (uint4*)xp_out);
    SPEC_LAUNCH_CHECK("attn_reduce_kernel");
    prof_mark(PC_ATTN_REDUCE, s);
    return SPEC_OK;
}

}  // namespace specv
