// bf16 MFMA GEMM for the verify step's projections:  out[m][n] = sum_k x[m][k] * W[n][k],
// fp32 accumulation, M = B*(k+1) rows (a few dozen to a few hundred), N and K in the thousands.
// At these shapes the weights are streamed once from HBM and everything else is noise, so the
// kernel is organised around the weight stream:
//
//   * W is re-tiled once (at model creation) into MFMA operand order: for every block of 32
//     output columns and every 16-wide k-step, the 64 lanes' 16-byte operands are contiguous
//     (1 KiB).  A wavefront owns one 32-column block and reads its stream with perfectly
//     coalesced 16-byte loads straight into registers; no LDS round trip for the weights.
//     The fragments are ordered [k-slab][column block][k-step in slab]: all wavefronts of a
//     launch move through K together, so at any moment the chip reads one contiguous region
//     (spread evenly over the HBM channels) instead of thousands of streams a power of two apart.
//   * the activations are written by the producing kernel in the same operand order, as hi + lo
//     bf16 pairs ([k-step][32-row block][hi|lo][lane][8], see operand.h), staged through LDS in
//     slabs of KS k-steps (double buffered, one barrier per slab) and shared by the 4 wavefronts
//     of the workgroup; each weight fragment feeds two MFMAs per row block (hi and lo).
//   * v_mfma_f32_32x32x16_bf16: A = activation fragment (rows m), B = weight fragment
//     (columns n), so a lane ends up with one output column and 16 rows: stores are
//     128-byte row segments.
//   * K is split across workgroups (grid.y) when N alone gives too few workgroups to keep
//     256 CUs streaming; partial sums go to separate fp32 slices that the consumer adds up
//     in a fixed order (deterministic).
#include <type_traits>

#include "common.h"
#include "operand.h"

namespace specv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int GEMM_KS = 4;          // k-steps (of 16) per LDS slab
constexpr int GEMM_WD = 4;          // slabs of weight fragments each wavefront keeps in flight
constexpr int GEMM_KUNIT = GEMM_KS * GEMM_WD;
constexpr int GEMM_XCDS = 8;        // accelerator dies, each with its own L2; workgroup i of a launch runs on die i % 8   // k-steps per split are a multiple of this
constexpr int GEMM_THREADS = 256;
constexpr int GEMM_EPI_PLAIN = 0, GEMM_EPI_SWIGLU = 1;

size_t bf16_packed_elems(int N, int K) { return (size_t)cdiv(N, 32) * 32 * (size_t)K; }

// ------------------------------------------------------------------ weight re-tiling
struct PackParts { const bf16_t* ptr[4]; int row_end[4]; int n; int interleave; int to_f16; };

// bf16 pair -> fp16 pair.  Exact for magnitudes from 2^-14 up to 65504 (bf16 has fewer mantissa bits than fp16);
// below 2^-14 the fp16 grid has steps of 2^-24 (absolute error at most 2^-25, nothing for a weight matrix);
// beyond 65504 the value saturates.
__device__ inline unsigned int bf16x2_to_f16x2(unsigned int w)
{
    return pack_f16x2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}

__global__ void pack_w_kernel(PackParts parts, int N, int K, int k_steps, int64_t total, uint4* __restrict__ out)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte operand per thread
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    int64_t frag = idx >> 6;
    // frag = (slab * n_blocks + nb) * KS + kk
    int kk = (int)(frag % GEMM_KS);
    int n_blocks = (N + 31) / 32;
    int nb = (int)((frag / GEMM_KS) % n_blocks);
    int ks = (int)(frag / GEMM_KS / n_blocks) * GEMM_KS + kk;
    int n = nb * 32 + (lane & 31);
    int k0 = ks * 16 + (lane >> 5) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (parts.interleave) {
        // two equal parts (gate, up): column block 2j holds rows 32j.. of part 0, block 2j+1 the same rows of part 1
        int row = (nb >> 1) * 32 + (lane & 31);
        if (row < parts.row_end[0]) v = *(const uint4*)(parts.ptr[nb & 1] + (int64_t)row * K + k0);
    } else if (n < N) {
        int start = 0;
        for (int p = 0; p < parts.n; ++p) {
            if (n < parts.row_end[p]) {
                v = *(const uint4*)(parts.ptr[p] + (int64_t)(n - start) * K + k0);
                break;
            }
            start = parts.row_end[p];
        }
    }
    if (parts.to_f16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
    out[idx] = v;
}

spec_status bf16_pack_matrix(const bf16_t* const* dev_parts, const int* part_rows, int n_parts, int K, bf16_t* dev_out,
                             PackedW* out, bool interleave, bool to_f16, hipStream_t s)
{
    if (n_parts < 1 || n_parts > 4 || K % (16 * GEMM_KUNIT)) { set_error("bf16_pack_matrix: bad shape"); return SPEC_EINVAL; }
    PackParts pp;
    pp.n = n_parts;
    pp.interleave = interleave ? 1 : 0;
    pp.to_f16 = to_f16 ? 1 : 0;
    if (interleave && (n_parts != 2 || part_rows[0] != part_rows[1] || part_rows[0] % 32)) { set_error("bf16_pack_matrix: interleaving needs two equal parts of a multiple of 32 rows"); return SPEC_EINVAL; }
    int N = 0;
    for (int i = 0; i < n_parts; ++i) {
        if (((uintptr_t)dev_parts[i] & 15) != 0) { set_error("bf16 weights must be 16-byte aligned"); return SPEC_EINVAL; }
        N += part_rows[i];
        pp.ptr[i] = dev_parts[i];
        pp.row_end[i] = N;
    }
    out->data = dev_out;
    out->N = N;
    out->K = K;
    out->n_blocks = (int)cdiv(N, 32);
    out->k_steps = K / 16;
    out->f16 = to_f16 ? 1 : 0;
    int64_t total = (int64_t)out->n_blocks * out->k_steps * 64;
    pack_w_kernel<<<(unsigned)cdiv(total, 256), 256, 0, s>>>(pp, N, K, out->k_steps, total, (uint4*)dev_out);
    SPEC_LAUNCH_CHECK("pack_w_kernel");
    return SPEC_OK;
}

// 8-bit weights (E4M3 codes, one fp32 scale per output row): the same tiling with two k-steps per 16-byte word,
// [k_steps / KS][n_blocks][KS / 2][64 lanes][2 fragments of 8 codes], and the scales in tiled column order.
struct PackParts8 { const unsigned char* ptr[4]; const float* scale[4]; int row_end[4]; int n; int interleave; };

__device__ inline bool pack8_source(const PackParts8& parts, int nb, int col, int N, int* part, int* row)
{
    if (parts.interleave) {
        *part = nb & 1;
        *row = (nb >> 1) * 32 + col;
        return *row < parts.row_end[0];
    }
    const int n = nb * 32 + col;
    if (n >= N) return false;
    int start = 0;
    for (int p = 0; p < parts.n; ++p) {
        if (n < parts.row_end[p]) { *part = p; *row = n - start; return true; }
        start = parts.row_end[p];
    }
    return false;
}

__global__ void pack_w8_kernel(PackParts8 parts, int N, int K, int64_t total, uint4* __restrict__ out, float* __restrict__ scale_out)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // one 16-byte word (two fragments) per thread
    const int n_blocks = (N + 31) / 32;
    if (idx < (int64_t)n_blocks * 32) {                                // the scales, tiled column order; padding columns 0
        int part, row;
        scale_out[idx] = pack8_source(parts, (int)(idx >> 5), (int)(idx & 31), N, &part, &row) ? parts.scale[part][row] : 0.f;
    }
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const int64_t frag2 = idx >> 6;                                    // (slab * n_blocks + nb) * (KS / 2) + pair
    const int pair = (int)(frag2 % (GEMM_KS / 2));
    const int nb = (int)((frag2 / (GEMM_KS / 2)) % n_blocks);
    const int ks = (int)(frag2 / (GEMM_KS / 2) / n_blocks) * GEMM_KS + 2 * pair;
    const int k0 = ks * 16 + (lane >> 5) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    int part, row;
    if (pack8_source(parts, nb, lane & 31, N, &part, &row)) {
        const unsigned char* src = parts.ptr[part] + (int64_t)row * K + k0;
        const uint2 a = *(const uint2*)src, b = *(const uint2*)(src + 16);
        v = make_uint4(a.x, a.y, b.x, b.y);
    }
    out[idx] = v;
}

size_t w8_packed_bytes(int N, int K) { return align_up((size_t)cdiv(N, 32) * 32 * ((size_t)K + sizeof(float)), 256); }

// dev_out: w8_packed_bytes(N, K) bytes: the tiled codes, then the tiled scales
spec_status w8_pack_matrix(const unsigned char* const* dev_parts, const float* const* dev_scales, const int* part_rows, int n_parts,
                           int K, void* dev_out, PackedW* out, bool interleave, bool x_f16, hipStream_t s)
{
    if (n_parts < 1 || n_parts > 4 || K % (16 * GEMM_KUNIT)) { set_error("w8_pack_matrix: bad shape"); return SPEC_EINVAL; }
    PackParts8 pp;
    pp.n = n_parts;
    pp.interleave = interleave ? 1 : 0;
    if (interleave && (n_parts != 2 || part_rows[0] != part_rows[1] || part_rows[0] % 32)) { set_error("w8_pack_matrix: interleaving needs two equal parts of a multiple of 32 rows"); return SPEC_EINVAL; }
    int N = 0;
    for (int i = 0; i < n_parts; ++i) {
        if (((uintptr_t)dev_parts[i] & 7) != 0 || ((uintptr_t)dev_scales[i] & 3) != 0) { set_error("8-bit weights must be 8-byte aligned"); return SPEC_EINVAL; }
        N += part_rows[i];
        pp.ptr[i] = dev_parts[i];
        pp.scale[i] = dev_scales[i];
        pp.row_end[i] = N;
    }
    out->data = (const bf16_t*)dev_out;
    out->N = N;
    out->K = K;
    out->n_blocks = (int)cdiv(N, 32);
    out->k_steps = K / 16;
    out->w8 = 1;
    out->f16 = x_f16 ? 1 : 0;           // the codes are the same either way; the kernel widens them to the activations' type
    out->scale = (const float*)((const char*)dev_out + (size_t)out->n_blocks * 32 * K);
    int64_t total = (int64_t)out->n_blocks * (out->k_steps / 2) * 64;
    pack_w8_kernel<<<(unsigned)cdiv(total, 256), 256, 0, s>>>(pp, N, K, total, (uint4*)dev_out, (float*)out->scale);
    SPEC_LAUNCH_CHECK("pack_w8_kernel");
    return SPEC_OK;
}

// ------------------------------------------------------------------ the GEMM
// s_waitcnt operand: at most n vector-memory operations outstanding, the other counters not waited for
constexpr int vmcnt_imm(int n) { return (n & 15) | 0x70 | 0xF00 | ((n >> 4) << 14); }

// Wp : [k_steps / KS][n_blocks][KS][64] u32x4_t   Xp : [k_steps][mb_pad][hi|lo][64] u32x4_t
// out: [splits][M][ldo] fp32 (slice stride = split_stride floats)
// MB row blocks (of 32) per workgroup tile; the 4 wavefronts are arranged WM along the rows x 4/WM
// along the columns.  A wavefront owns MB/WM row blocks and WM column blocks (the tile is always 128
// columns), so with WM = 2 every activation fragment read from LDS feeds two MFMAs and every weight
// fragment is read by two wavefronts (the second read hits the CU's L1): half the LDS traffic per MFMA.
// GROUPED (mixture of experts): blockIdx.z walks a device-side list of row tiles, tiles[0] = number of
// tiles, then (group, first row block) pairs; group g multiplies by the matrix at Wp + g * w_group_stride
// (all groups have the same shape).  Tiles past the list's end exit at once.
// Large row counts (MB = 6 or 8: 192 or 256 rows per tile) take NBW_T = 4 column blocks per wavefront, i.e. a 256-column
// tile: a wavefront then owns 3-4 x 4 accumulator blocks (192-256 accumulation registers, one workgroup per CU) and
// every fragment it fetches feeds 4 (weights: 6-8) MFMAs, which halves the LDS and vector-memory traffic per MFMA
// that bounds the 128 x 128 tile.  Its two LDS slabs (96-128 KiB) are dynamic shared memory.
// W8: the weights are E4M3 codes, two k-steps per 16-byte word (half the weight bytes and load instructions); a
// fragment is widened to bf16 in registers right before its MFMAs (exact) and the output column's scale is applied to
// the accumulators in the epilogue.
// XF: the activations' operand format (operand.h): XF_HILO = hi + lo bf16 pairs against bf16 weights, two MFMAs per
// weight fragment and row block; XF_F16 = one fp16 value against fp16 weights, one MFMA.  The fused SwiGLU epilogue
// writes its output in the same format (gate/up and down projection take the same one).
template <int MB, int WM, int WD, int EPI, bool GROUPED = false, int NBW_T = WM, bool W8 = false, int XF = XF_HILO>
__global__ __launch_bounds__(GEMM_THREADS, (MB >= 6 || (MB >= 3 && WM == 1 && NBW_T == 2)) ? 1 : 2) void gemm_bf16_kernel(
    const u32x4_t* __restrict__ Wp, const u32x4_t* __restrict__ Xp, float* __restrict__ out, int n_blocks, int k_steps,
    int ksteps_per_split, int mb_pad, int M, int N, int ldo, int64_t split_stride,
    const int32_t* __restrict__ tiles = nullptr, int64_t w_group_stride = 0, const float* __restrict__ wscale = nullptr)
{
    constexpr int KS = GEMM_KS;
    constexpr int KSW = W8 ? KS / 2 : KS;               // 16-byte words of one column block per lane and slab
    constexpr int MBW = MB / WM, NBW = NBW_T;
    constexpr int TILE_NB = (4 / WM) * NBW;             // 32-column blocks per workgroup tile
    constexpr bool BIG = MB >= 6;
    static_assert(MB % WM == 0, "row blocks must divide over the wavefronts");
    constexpr int SLAB = KS * MB * 64 * XF;             // u32x4_t per slab (XF operand words per lane and k-step)
    constexpr int XPT = SLAB / GEMM_THREADS;            // u32x4_t per thread per slab
    static_assert(SLAB % GEMM_THREADS == 0, "a slab must divide over the threads");
    // the fused SwiGLU epilogue re-uses the slabs as an fp32 transpose tile, which may be the larger of the two
    constexpr int EPI_WORDS = EPI != GEMM_EPI_SWIGLU ? 0 : (BIG ? (MB / WM) * 32 * 129 : WM == 1 ? 32 * 129 : MB * 32 * 65) / 4 + 1;
    constexpr int LDS_WORDS = 2 * SLAB > EPI_WORDS ? 2 * SLAB : EPI_WORDS;
    extern __shared__ u32x4_t lds_dyn[];
    __shared__ u32x4_t lds_static[BIG ? 1 : LDS_WORDS];
    u32x4_t* const lds = BIG ? lds_dyn : lds_static;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int mh = wave % WM, np = wave / WM;
    // Which tile this workgroup computes.  Workgroups go to the 8 XCDs (each with an L2 of its own) round robin in
    // launch order, so the launch index is re-mapped: XCD j takes a contiguous stretch of the tiles in the order
    // (row tile fastest, then column tile, then k-split).  The workgroups that share a weight tile then share an L2,
    // and an XCD reads the activations of one or two k-splits instead of all of them.
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if constexpr (!GROUPED) {
        const int nx = gridDim.x, ny = gridDim.y, nz = gridDim.z;
        const int total = nx * ny * nz, lin = bx + nx * (by + ny * bz);
        const int xcd = lin % GEMM_XCDS, slot = lin / GEMM_XCDS;
        const int v = xcd * (total / GEMM_XCDS) + (xcd < total % GEMM_XCDS ? xcd : total % GEMM_XCDS) + slot;
        bz = v % nz;
        bx = (v / nz) % nx;
        by = v / (nz * nx);
    }
    const int nb0 = bx * TILE_NB + np * NBW;
    const int ks0 = by * ksteps_per_split;
    int ks1 = ks0 + ksteps_per_split;
    if (ks1 > k_steps) ks1 = k_steps;
    const int n_slabs = (ks1 - ks0) / KS;
    int mblk0 = bz * MB;                        // first 32-row block of this tile
    if constexpr (GROUPED) {
        if (bz >= tiles[0]) return;
        Wp += (int64_t)tiles[1 + 2 * bz] * w_group_stride;
        if constexpr (W8) wscale += (int64_t)tiles[1 + 2 * bz] * w_group_stride * 4;   // a group's scales sit in its own region
        mblk0 = tiles[2 + 2 * bz];
    }

    // slab s of column block j of this wavefront: wptr[j] + s * wslab
    const u32x4_t* wptr[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
        wptr[j] = Wp + (((int64_t)(ks0 / KS) * n_blocks + (nb0 + j < n_blocks ? nb0 + j : 0)) * KSW) * 64 + lane;
    const int64_t wslab = (int64_t)n_blocks * KSW * 64;
    float wsc[NBW];                                     // 8-bit weights: this lane's column scales
#pragma unroll
    for (int j = 0; j < NBW; ++j) wsc[j] = 1.0f;
    const u32x4_t* xbase = Xp + ((int64_t)ks0 * mb_pad + (int64_t)mblk0) * (64 * XF);

    f32x16_t acc[MBW][NBW];
#pragma unroll
    for (int i = 0; i < MBW; ++i)
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // the weight stream runs WD slabs ahead of the MFMAs: a register ring, each entry refilled
    // right after its last use
    u32x4_t w[WD][KSW][NBW], xr[XPT];

    auto load_x = [&](int slab) {
#pragma unroll
        for (int j = 0; j < XPT; ++j) {
            int idx = threadIdx.x + GEMM_THREADS * j;
            int kl = idx / (MB * 64 * XF), rem = idx % (MB * 64 * XF);
            xr[j] = xbase[((int64_t)(slab * KS + kl) * mb_pad) * (64 * XF) + rem];
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int j = 0; j < XPT; ++j) lds[buf * SLAB + threadIdx.x + GEMM_THREADS * j] = xr[j];
    };
    // The 128-column tiles skip the registers: their activation slabs go from global memory straight into LDS
    // (global_load ... lds: no staging registers, no LDS store instructions).  Each instruction moves 64 x 16 bytes:
    // per-lane global addresses, LDS address = the wavefront-uniform base given here + 16 * lane.  (The 256-column
    // tile measured slightly faster with its stores spread under the MFMAs, and keeps them.)
    auto stage_x = [&](int slab, int tobuf) {
#pragma unroll
        for (int j = 0; j < XPT; ++j) {
            int idx = threadIdx.x + GEMM_THREADS * j;
            int kl = idx / (MB * 64 * XF), rem = idx % (MB * 64 * XF);
            const u32x4_t* src = xbase + ((int64_t)(slab * KS + kl) * mb_pad) * (64 * XF) + rem;
            u32x4_t* dst = lds + tobuf * SLAB + (idx - lane);
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                             (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
        }
    };
    int buf = 0;
    // No branch may sit between the loads and their use: the compiler can only count outstanding
    // loads (s_waitcnt vmcnt(n)) along straight-line code, and falls back to draining the whole
    // queue otherwise.  So every slab issues its prefetches unconditionally; past the end they
    // re-read the last slab (cache hits, results unused).
    auto slab_body = [&](auto slot_c, int s) {
        constexpr int SLOT = decltype(slot_c)::value;
        const int s_w = s + WD < n_slabs ? s + WD : n_slabs - 1;
        const int s_x = s + 1 < n_slabs ? s + 1 : n_slabs - 1;
        // the next slab's activations are the oldest loads of this slab: what is waited for at its end
        if constexpr (BIG) load_x(s_x); else stage_x(s_x, buf ^ 1);
        // keep these loads HERE: left alone, the scheduler sinks them to the end of the slab, next to the LDS
        // stores that consume them, and the whole round trip to L2 is then paid once per slab
        __builtin_amdgcn_sched_barrier(0);
        // LDS reads run one k-step ahead of the MFMAs that use them (two register sets): with one or two
        // wavefronts per SIMD nothing else would hide the LDS latency.  The scheduling barriers keep that order.
        u32x4_t a[2][MBW][XF];
        auto read_a = [&](int set, int kk) {
#pragma unroll
            for (int i = 0; i < MBW; ++i)
#pragma unroll
                for (int part = 0; part < XF; ++part)
                    a[set][i][part] = lds[buf * SLAB + ((kk * MB + mh * MBW + i) * XF + part) * 64 + lane];
        };
        read_a(0, 0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            if (kk + 1 < KS) read_a((kk + 1) & 1, kk + 1);
            if constexpr (BIG) {
                // a slab of the 256-row tile lasts longer than the trip to L2: the next slab's activations go to LDS
                // under the MFMAs of the last two k-steps instead of after them
                if (kk >= KS - 2) {
#pragma unroll
                    for (int j = (kk - (KS - 2)) * (XPT / 2); j < (kk - (KS - 2) + 1) * (XPT / 2); ++j)
                        lds[(buf ^ 1) * SLAB + threadIdx.x + GEMM_THREADS * j] = xr[j];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            u32x4_t wk[NBW];                             // this k-step's weight fragments in the activations' 16-bit type
#pragma unroll
            for (int j = 0; j < NBW; ++j) {
                if constexpr (W8 && XF == XF_F16) {
                    const unsigned int wa = w[SLOT][kk >> 1][j][(kk & 1) * 2], wb = w[SLOT][kk >> 1][j][(kk & 1) * 2 + 1];
                    wk[j] = u32x4_t{__builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wa, 1.0f, false)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wa, 1.0f, true)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wb, 1.0f, false)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wb, 1.0f, true))};
                } else if constexpr (W8) {
                    const unsigned int wa = w[SLOT][kk >> 1][j][(kk & 1) * 2], wb = w[SLOT][kk >> 1][j][(kk & 1) * 2 + 1];
                    wk[j] = u32x4_t{__builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wa, 1.0f, false)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wa, 1.0f, true)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wb, 1.0f, false)),
                                    __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(wb, 1.0f, true))};
                } else {
                    wk[j] = w[SLOT][kk][j];
                }
            }
            // hi products of all blocks first, then the lo products: two MFMAs on one accumulator are never adjacent
#pragma unroll
            for (int part = 0; part < XF; ++part)
#pragma unroll
                for (int i = 0; i < MBW; ++i)
#pragma unroll
                    for (int j = 0; j < NBW; ++j) {
                        if constexpr (XF == XF_F16)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a[kk & 1][i][part]),
                                                                               __builtin_bit_cast(f16x8_t, wk[j]), acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[kk & 1][i][part]),
                                                                                __builtin_bit_cast(bf16x8_t, wk[j]), acc[i][j], 0, 0, 0);
                    }
            if (!W8 || (kk & 1)) {                       // (8-bit: a word serves two k-steps and is refilled after the second)
#pragma unroll
                for (int j = 0; j < NBW; ++j)
                    w[SLOT][W8 ? kk >> 1 : kk][j] = __builtin_nontemporal_load(wptr[j] + (int64_t)s_w * wslab + (W8 ? kk >> 1 : kk) * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // ... and the weight loads of this slab stay above the LDS stores, so that waiting for the (older)
        // activation loads does not drain the weight stream
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BIG) {
            __syncthreads();
        } else {
            // Wait for the transfers into LDS only: the slab's own weight reloads (KSW * NBW of them) were issued later
            // and stay in flight (__syncthreads would drain the whole queue).  No wavefront reads the other buffer
            // before this barrier, and all have finished reading this one when they pass the next.
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(KSW * NBW));
            __builtin_amdgcn_s_barrier();
        }
        buf ^= 1;
    };

    // n_slabs is a multiple of WD (K % (16 * GEMM_KUNIT) == 0 and split sizes are rounded to it)
    if (n_slabs > 0) {
        if constexpr (W8) {
            // Fetched with the first weight loads and known to have arrived (the wait below, then the empty asm that
            // ties the values to this point) on every path into the epilogue: a load the compiler may still count as
            // outstanding there makes it wait with vmcnt(0) before each of the 64 stores, which serialises them.
#pragma unroll
            for (int j = 0; j < NBW; ++j)
                if (nb0 + j < n_blocks) wsc[j] = wscale[(nb0 + j) * 32 + (lane & 31)];
        }
#pragma unroll
        for (int d = 0; d < WD; ++d) {
            const int sd = d < n_slabs ? d : n_slabs - 1;
#pragma unroll
            for (int i = 0; i < KSW; ++i)
#pragma unroll
                for (int j = 0; j < NBW; ++j) w[d][i][j] = __builtin_nontemporal_load(wptr[j] + (int64_t)sd * wslab + i * 64);
        }
        if constexpr (BIG) {
            load_x(0);
            store_x(0);
            __syncthreads();
        } else {
            stage_x(0, 0);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __builtin_amdgcn_s_barrier();
        }
        if constexpr (W8) {
#pragma unroll
            for (int j = 0; j < NBW; ++j) asm volatile("" : "+v"(wsc[j]));
        }
        for (int s = 0; s < n_slabs; s += WD) {
            slab_body(std::integral_constant<int, 0>{}, s);
            if constexpr (WD > 1) slab_body(std::integral_constant<int, 1>{}, s + 1);
            if constexpr (WD > 2) slab_body(std::integral_constant<int, 2>{}, s + 2);
            if constexpr (WD > 3) slab_body(std::integral_constant<int, 3>{}, s + 3);
        }
    }

    if constexpr (EPI == GEMM_EPI_SWIGLU && BIG) {
        // 256-column tile: a wavefront's four accumulator columns are (gate, up) of two groups of 32 hidden channels.
        // Same transpose through LDS as below, one half of the rows (the wavefronts with the same mh) at a time.
        static_assert(!BIG || NBW == 4, "the 256-column tile has four column blocks per wavefront");
        float* tile = (float*)lds;                              // [MBW*32 rows][129]
        uint4* xo = (uint4*)out;
#pragma unroll
        for (int half = 0; half < WM; ++half) {
            __syncthreads();
            if (mh == half) {
#pragma unroll
                for (int i = 0; i < MBW; ++i)
#pragma unroll
                    for (int cg = 0; cg < 2; ++cg)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            float g = acc[i][2 * cg][r], u = acc[i][2 * cg + 1][r];
                            if constexpr (W8) {
                                g *= wsc[2 * cg];
                                u *= wsc[2 * cg + 1];
                            }
                            int row = i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                            tile[row * 129 + (np * 2 + cg) * 32 + (lane & 31)] = g / (1.0f + __expf(-g)) * u;
                        }
            }
            __syncthreads();
            for (int e = threadIdx.x; e < MBW * 32 * 16; e += GEMM_THREADS) {
                int row = e >> 4, g8 = e & 15;
                int m = (mblk0 + half * MBW) * 32 + row, f = bx * 128 + g8 * 8;
                if (m >= M || f >= N / 2) continue;
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = tile[row * 129 + g8 * 8 + j];
                xp_store8_t<XF>(xo, m, f, mb_pad, v);
            }
        }
        return;
    } else if constexpr (EPI == GEMM_EPI_SWIGLU && WM == 1 && NBW == 1) {
        // 128-column tile of the 1 x 4 arrangement with one column block per wavefront: wavefronts 0 and 2 hold the gates,
        // 1 and 3 the ups of 2 x 32 hidden channels.  The raw accumulators go through LDS one row block at a time, and
        // silu(gate) * up is formed on the way out.
        float* tile = (float*)lds;                              // [32 rows][129]
        uint4* xo = (uint4*)out;
#pragma unroll
        for (int i = 0; i < MBW; ++i) {
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                tile[row * 129 + np * 32 + (lane & 31)] = W8 ? acc[i][0][r] * wsc[0] : acc[i][0][r];
            }
            __syncthreads();
            {
                const int e = threadIdx.x;                      // 32 rows x 8 groups of 8 hidden channels
                const int row = e >> 3, g8 = e & 7;
                const int m = (mblk0 + i) * 32 + row, f = bx * 64 + g8 * 8;
                if (m < M && f < N / 2) {
                    const float* src = tile + row * 129 + (g8 >> 2) * 64 + (g8 & 3) * 8;
                    float v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) { const float g = src[j], u = src[32 + j]; v[j] = g / (1.0f + __expf(-g)) * u; }
                    xp_store8_t<XF>(xo, m, f, mb_pad, v);
                }
            }
        }
        return;
    } else if constexpr (EPI == GEMM_EPI_SWIGLU && WM == 1) {
        // 256-column tile of the 1 x 4 arrangement (each wavefront: all MB row blocks, gate and up of 32 hidden channels):
        // the same transpose through LDS, one row block (32 rows x 128 channels) at a time.
        static_assert(EPI != GEMM_EPI_SWIGLU || WM != 1 || NBW == 2, "fused SwiGLU needs two column blocks per wavefront");
        float* tile = (float*)lds;                              // [32 rows][129]
        uint4* xo = (uint4*)out;
#pragma unroll
        for (int i = 0; i < MBW; ++i) {
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float g = acc[i][0][r], u = acc[i][NBW - 1][r];
                if constexpr (W8) {
                    g *= wsc[0];
                    u *= wsc[NBW - 1];
                }
                const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                tile[row * 129 + np * 32 + (lane & 31)] = g / (1.0f + __expf(-g)) * u;
            }
            __syncthreads();
            for (int e = threadIdx.x; e < 32 * 16; e += GEMM_THREADS) {
                const int row = e >> 4, g8 = e & 15;
                const int m = (mblk0 + i) * 32 + row, f = bx * 128 + g8 * 8;
                if (m >= M || f >= N / 2) continue;
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = tile[row * 129 + g8 * 8 + j];
                xp_store8_t<XF>(xo, m, f, mb_pad, v);
            }
        }
        return;
    } else if constexpr (EPI == GEMM_EPI_SWIGLU) {
        // The weights of the gate/up projection are tiled with gate and up column blocks interleaved,
        // so this wavefront's two accumulators hold gate and up of the same 32 hidden channels:
        // silu(gate) * up in registers, transposed through LDS (free after the main loop) into rows,
        // and written as hi + lo bf16 in the operand order the down projection reads.
        static_assert(EPI != GEMM_EPI_SWIGLU || NBW == 2, "fused SwiGLU needs two column blocks per wavefront");
        float* tile = (float*)lds;                              // [MB*32 rows][65]
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MBW; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float g = acc[i][0][r], u = acc[i][NBW - 1][r];
                if constexpr (W8) {
                    g *= wsc[0];
                    u *= wsc[NBW - 1];
                }
                int row = (mh * MBW + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                tile[row * 65 + np * 32 + (lane & 31)] = g / (1.0f + __expf(-g)) * u;
            }
        __syncthreads();
        uint4* xo = (uint4*)out;
        for (int e = threadIdx.x; e < MB * 32 * 8; e += GEMM_THREADS) {
            int row = e >> 3, g8 = e & 7;
            int m = mblk0 * 32 + row, f = bx * 64 + g8 * 8;
            if (m >= M || f >= N / 2) continue;
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = tile[row * 65 + g8 * 8 + j];
            xp_store8_t<XF>(xo, m, f, mb_pad, v);
        }
        return;
    }
    float* o = out + (int64_t)by * split_stride;
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
        const int n = (nb0 + j) * 32 + (lane & 31);
        if (nb0 + j >= n_blocks || n >= N) continue;
        const float sc = wsc[j];
#pragma unroll
        for (int i = 0; i < MBW; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = (mblk0 + mh * MBW + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m < M) o[(int64_t)m * ldo + n] = W8 ? acc[i][j][r] * sc : acc[i][j][r];
            }
    }
}

// Tile shapes.  Up to 4 row blocks (128 rows) a launch has one kind of tile: MB = min(row blocks, gemm_max_mb) x 128
// columns.  From gemm_big_min_blocks row blocks on (0 = never) the 256-column tile with 8 or 6 row blocks is available
// too, and each GEMM takes it when it still fills the chip: at least gemm_big_min_tiles (200) tiles, or - K split, two or more tiles of
// rows - at least 192 workgroups of 32 or more k-steps each (a 256 x 256 tile with a short K spends its time in prologue
// and epilogue; with one tile of rows the extra split-K slices cost the consumers more than the GEMM gains; and a fused
// SwiGLU epilogue cannot split K at all).  Both kinds read the same activation buffer, so its rows are padded
// to a multiple of both tile heights: 8 blocks, or 12 where that pads less (then the big tile has 6 row blocks).
static int gemm_big_mb(int M)
{
    const int nb = (int)cdiv(M, 32), from = tune("gemm_big_min_blocks");
    if (from <= 0 || nb < from || nb < 5) return 0;
    return cdiv(nb, 12) * 12 < cdiv(nb, 8) * 8 ? 6 : 8;
}
int gemm_mb(int M) { int mb = (int)cdiv(M, 32), cap = tune("gemm_max_mb"); cap = cap < 1 ? 1 : (cap > 4 ? 4 : cap); return mb > cap ? cap : mb; }
int gemm_mb_pad(int M)
{
    const int nb = (int)cdiv(M, 32), big = gemm_big_mb(M);
    if (big) return (int)cdiv(nb, big == 6 ? 12 : 8) * (big == 6 ? 12 : 8);
    const int mb = gemm_mb(M);
    return (int)cdiv(nb, mb) * mb;
}

struct GemmShape { int mb, tile_nb, kunit, m_tiles, n_tiles; bool wide = false, one_block = false; };
static GemmShape gemm_shape(const PackedW& W, int M, bool fused_swiglu)
{
    GemmShape g;
    const int pad = gemm_mb_pad(M), big = gemm_big_mb(M);
    if (big) {
        const int64_t tiles = (int64_t)cdiv(W.n_blocks, 8) * (pad / big);
        int64_t splits = tune("gemm_wg_target") / tiles;
        if (splits > W.k_steps / 32) splits = W.k_steps / 32;
        if (splits < 1) splits = 1;
        if (tiles >= tune("gemm_big_min_tiles") || (!fused_swiglu && pad / big >= 2 && tiles * splits >= 192)) {
            g.mb = big; g.tile_nb = 8; g.kunit = GEMM_KS * 2;
            g.m_tiles = pad / big; g.n_tiles = (int)cdiv(W.n_blocks, 8);
            if (big == 8 && cdiv(M, 32) <= 6) g.mb = 6;                 // 129..192 rows: the one tile needs 6 row blocks only
            return g;
        }
    }
    g.mb = big ? 4 : gemm_mb(M);
    g.tile_nb = 4;
    // k-steps per split come in units of one pass of the weight ring: 2 slabs for the 2x2 arrangement (even row-block
    // counts), 4 for the others
    g.kunit = g.mb % 2 == 0 ? GEMM_KS * 2 : GEMM_KUNIT;
    g.m_tiles = pad / g.mb; g.n_tiles = (int)cdiv(W.n_blocks, 4);
    // One tile of 64 or 128 rows, plain epilogue, K unsplit because the columns alone give enough workgroups (the LM head): 256-column
    // tiles with the wavefronts 1 x 4 - no weight fragment fetched twice, the activation slab serves twice the columns.
    // (With K split to make up the workgroups the extra slices cost the consumers what the GEMM gains.)
    if ((g.mb == 4 || g.mb == 2) && g.m_tiles == 1 && !fused_swiglu && tune("gemm_wide4") > 0 && W.n_blocks % 8 == 0 && W.n_blocks / 8 >= tune("gemm_wide4")) {
        g.wide = true; g.tile_nb = 8; g.n_tiles = W.n_blocks / 8; g.kunit = GEMM_KS * 2;
        return g;
    }
    // 97..128 rows: two tiles of 64 rows x 256 columns (wavefronts 1 x 4) instead of one of 128 x 128 (2 x 2): the same
    // number of workgroups and K splits, the same MFMAs per workgroup and slab, but no weight fragment fetched twice and half
    // the activation slab per workgroup; the second row tile's weights come from L2 (the two are neighbours on one XCD).
    // The same holds for up to gemm_split_rows 128-row tiles (129..256 rows at 2); a 64-row tile that would hold padding
    // only is not launched.
    // 129..256 rows where K is not split (the fused gate/up projection): two tiles of 96 or 128 rows instead of three or four of
    // 64 - 2 x 112 workgroups fit the chip at once, 3 x 112 and 4 x 112 do not.
    // 97..128 rows with fp16 activations: one tile of 128 rows x 128 columns with the wavefronts 1 x 4, each its own column
    // block over all four row blocks.  Every weight fragment is then fetched by exactly one wavefront of one workgroup
    // (the pair of 64-row tiles fetches each twice: the second time as an L2 hit, but through the same L1 and memory
    // pipeline as the weight stream), at the price of one LDS read per MFMA, which the single fp16 MFMA per fragment leaves room for:
    // gate/up 56 -> 50 us, down 31 -> 26 us at the 8B shape.  With hi + lo operands the pair stays ahead.
    if (g.mb == 4 && g.m_tiles == 1 && W.f16 && tune("gemm_one_block") != 0 && W.n_blocks % 4 == 0) {
        g.one_block = true; g.tile_nb = 4; g.n_tiles = W.n_blocks / 4; g.kunit = GEMM_KS * 2;
        return g;
    }
    if (g.mb == 4 && g.m_tiles <= tune("gemm_split_rows") && W.n_blocks % 8 == 0) {
        const int nb = (int)cdiv(M, 32);
        if (fused_swiglu && nb >= 5 && tune("gemm_tiles_96") != 0) g.mb = nb <= 6 ? 3 : 4;
        else g.mb = 2;
        g.m_tiles = (int)cdiv(nb, g.mb); g.wide = true; g.tile_nb = 8; g.n_tiles = W.n_blocks / 8; g.kunit = GEMM_KS * 2;
        return g;
    }
    return g;
}

int gemm_pick_splits(const PackedW& W, int M, int forced)
{
    const GemmShape g = gemm_shape(W, M, false);
    const int unit = g.kunit;
    int max_splits = W.k_steps / (tune("gemm_min_ksteps") > unit ? tune("gemm_min_ksteps") : unit);
    if (max_splits < 1) max_splits = 1;
    int splits = forced > 0 ? forced : tune("gemm_wg_target") / (g.n_tiles * g.m_tiles);
    if (splits < 1) splits = 1;
    if (splits > max_splits) splits = max_splits;
    int kps = (int)cdiv(cdiv(W.k_steps, splits), unit) * unit;
    return (int)cdiv(W.k_steps, kps);
}

// out must hold splits * M * ldo floats; with swiglu (gate/up projection, splits == 1, an even number
// of row blocks) out is instead the hi + lo operand buffer of silu(gate) * up, [N/2] channels wide.
// Returns SPEC_EUNSUPPORTED (nothing launched) if swiglu is asked for a shape it cannot fuse.
bool gemm_can_fuse_swiglu(const PackedW& W, int M, int splits) { if (splits != 1) return false; const GemmShape g = gemm_shape(W, M, true); return g.mb % 2 == 0 || (g.wide && g.mb == 3) || g.one_block; }

spec_status launch_gemm_bf16(const PackedW& W, const bf16_t* Xp, int M, float* out, int ldo, int splits, bool swiglu, hipStream_t s)
{
    const GemmShape g = gemm_shape(W, M, swiglu);
    const int mb = g.mb, mb_pad = gemm_mb_pad(M);
    int kps = (int)cdiv(cdiv(W.k_steps, splits), g.kunit) * g.kunit;
    dim3 grid((unsigned)g.n_tiles, (unsigned)cdiv(W.k_steps, kps), (unsigned)g.m_tiles);
    int64_t stride = (int64_t)M * ldo;
    const u32x4_t* wp = (const u32x4_t*)W.data;
    const u32x4_t* xp = (const u32x4_t*)Xp;
    if (swiglu && !gemm_can_fuse_swiglu(W, M, splits)) { set_error("gemm: SwiGLU cannot be fused for this shape"); return SPEC_EUNSUPPORTED; }
#define SPEC_GEMM_LAUNCH_W(MBV, WMV, WDV, E, W8V, XFV) gemm_bf16_kernel<MBV, WMV, WDV, E, false, (MBV % 2 == 0 && WMV == 1) ? 2 : WMV, W8V, XFV><<<grid, GEMM_THREADS, 0, s>>>(wp, xp, out, W.n_blocks, W.k_steps, kps, mb_pad, M, W.N, ldo, stride, nullptr, 0, W.scale)
#define SPEC_GEMM_LAUNCH_1BW(E, W8V, XFV) gemm_bf16_kernel<4, 1, 2, E, false, 1, W8V, XFV><<<grid, GEMM_THREADS, 0, s>>>(wp, xp, out, W.n_blocks, W.k_steps, kps, mb_pad, M, W.N, ldo, stride, nullptr, 0, W.scale)
#define SPEC_GEMM_LAUNCH_96W(E, W8V, XFV) gemm_bf16_kernel<3, 1, 2, E, false, 2, W8V, XFV><<<grid, GEMM_THREADS, 0, s>>>(wp, xp, out, W.n_blocks, W.k_steps, kps, mb_pad, M, W.N, ldo, stride, nullptr, 0, W.scale)
    // the four combinations of 8-bit or 16-bit weights and hi + lo or fp16 activations
#define SPEC_GEMM_BY_TYPE(CALL, ...) do { \
        if (W.w8) { if (W.f16) CALL(__VA_ARGS__, true, XF_F16); else CALL(__VA_ARGS__, true, XF_HILO); } \
        else { if (W.f16) CALL(__VA_ARGS__, false, XF_F16); else CALL(__VA_ARGS__, false, XF_HILO); } } while (0)
#define SPEC_GEMM_LAUNCH_96(E) SPEC_GEMM_BY_TYPE(SPEC_GEMM_LAUNCH_96W, E)
#define SPEC_GEMM_LAUNCH(MBV, WMV, WDV, E) SPEC_GEMM_BY_TYPE(SPEC_GEMM_LAUNCH_W, MBV, WMV, WDV, E)
    // the 256-column tile: two LDS slabs of MB * 8 KiB as dynamic shared memory (beyond the 64 KiB a kernel gets by default)
#define SPEC_GEMM_LAUNCH_BIG_W(MBV, E, W8V, XFV) do { \
        auto kern = gemm_bf16_kernel<MBV, 2, 1, E, false, 4, W8V, XFV>; \
        constexpr int slab_bytes = 2 * GEMM_KS * MBV * 64 * XFV * 16, epi_bytes = E == GEMM_EPI_SWIGLU ? (MBV / 2) * 32 * 129 * 4 + 16 : 0; \
        constexpr int lds_bytes = slab_bytes > epi_bytes ? slab_bytes : epi_bytes; \
        static bool raised = false; \
        if (!raised) { \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes); \
            if (e != hipSuccess) { set_error("gemm: cannot reserve %d bytes of LDS: %s", lds_bytes, hipGetErrorString(e)); return SPEC_EHIP; } \
            raised = true; \
        } \
        kern<<<grid, GEMM_THREADS, lds_bytes, s>>>(wp, xp, out, W.n_blocks, W.k_steps, kps, mb_pad, M, W.N, ldo, stride, nullptr, 0, W.scale); \
    } while (0)
#define SPEC_GEMM_LAUNCH_BIG(MBV, E) SPEC_GEMM_BY_TYPE(SPEC_GEMM_LAUNCH_BIG_W, MBV, E)
    switch (mb) {
        case 1: SPEC_GEMM_LAUNCH(1, 1, GEMM_WD, GEMM_EPI_PLAIN); break;
        case 2:
            if (g.wide && swiglu) SPEC_GEMM_LAUNCH(2, 1, 2, GEMM_EPI_SWIGLU);
            else if (g.wide) SPEC_GEMM_LAUNCH(2, 1, 2, GEMM_EPI_PLAIN);
            else if (swiglu) SPEC_GEMM_LAUNCH(2, 2, 2, GEMM_EPI_SWIGLU);
            else SPEC_GEMM_LAUNCH(2, 2, 2, GEMM_EPI_PLAIN);
            break;
        case 3:
            if (g.wide && swiglu) SPEC_GEMM_LAUNCH_96(GEMM_EPI_SWIGLU);
            else if (g.wide) SPEC_GEMM_LAUNCH_96(GEMM_EPI_PLAIN);
            else SPEC_GEMM_LAUNCH(3, 1, GEMM_WD, GEMM_EPI_PLAIN);
            break;
        case 6: if (swiglu) SPEC_GEMM_LAUNCH_BIG(6, GEMM_EPI_SWIGLU); else SPEC_GEMM_LAUNCH_BIG(6, GEMM_EPI_PLAIN); break;
        case 8: if (swiglu) SPEC_GEMM_LAUNCH_BIG(8, GEMM_EPI_SWIGLU); else SPEC_GEMM_LAUNCH_BIG(8, GEMM_EPI_PLAIN); break;
        default:
            if (g.one_block) {                               // fp16 activations only
                if (W.w8) { if (swiglu) SPEC_GEMM_LAUNCH_1BW(GEMM_EPI_SWIGLU, true, XF_F16); else SPEC_GEMM_LAUNCH_1BW(GEMM_EPI_PLAIN, true, XF_F16); }
                else { if (swiglu) SPEC_GEMM_LAUNCH_1BW(GEMM_EPI_SWIGLU, false, XF_F16); else SPEC_GEMM_LAUNCH_1BW(GEMM_EPI_PLAIN, false, XF_F16); }
            }
            else if (g.wide && swiglu) SPEC_GEMM_LAUNCH(4, 1, 2, GEMM_EPI_SWIGLU);
            else if (g.wide) SPEC_GEMM_LAUNCH(4, 1, 2, GEMM_EPI_PLAIN);
            else if (swiglu) SPEC_GEMM_LAUNCH(4, 2, 2, GEMM_EPI_SWIGLU);
            else SPEC_GEMM_LAUNCH(4, 2, 2, GEMM_EPI_PLAIN);
            break;
    }
#undef SPEC_GEMM_LAUNCH_BIG
#undef SPEC_GEMM_BY_TYPE
#undef SPEC_GEMM_LAUNCH_96
#undef SPEC_GEMM_LAUNCH_96W
#undef SPEC_GEMM_LAUNCH_1BW
#undef SPEC_GEMM_LAUNCH_BIG_W
#undef SPEC_GEMM_LAUNCH
#undef SPEC_GEMM_LAUNCH_W
    SPEC_LAUNCH_CHECK("gemm_bf16_kernel");
    return SPEC_OK;
}

// Grouped GEMM over a device-side tile list (see the kernel): 64-row tiles, group g uses the matrix g *
// group_stride elements after W0; Xp and the output cover rows_pad rows (a multiple of 64).  With swiglu
// the output is the hi + lo operand buffer of silu(gate) * up (rows_pad / 32 row blocks per k-step).
spec_status launch_gemm_bf16_grouped(const PackedW& W0, int64_t group_stride, const bf16_t* Xp, int rows_pad, int max_tiles,
                                     const int32_t* tiles, float* out, int ldo, bool swiglu, hipStream_t s)
{
    if (rows_pad % 64 || max_tiles < 1 || W0.k_steps % GEMM_KUNIT) { set_error("grouped gemm: bad shape"); return SPEC_EINVAL; }
    dim3 grid((unsigned)cdiv(W0.n_blocks, 4), 1, (unsigned)max_tiles);
    const u32x4_t* wp = (const u32x4_t*)W0.data;
    const u32x4_t* xp = (const u32x4_t*)Xp;
    // distance between the groups' matrices in 16-byte words (group_stride: bf16 elements, or bytes of a whole 8-bit region,
    // codes and scales, so that the scales of group g sit g * stride behind those of group 0 as well)
    const int64_t stride16 = W0.w8 ? group_stride / 16 : group_stride / 8;
    // Two tile shapes of 64 rows: 128 columns with the wavefronts 2 x 2, or 256 columns with the wavefronts 1 x 4 (each
    // its own two column blocks: no weight fragment is fetched twice and the activation slab serves twice the columns,
    // which is what the expert GEMMs - few rows, all weights touched - are bound by).
    const bool wide = tune("moe_wide_tiles") != 0 && W0.n_blocks % 8 == 0;
    if (wide) grid.x = (unsigned)cdiv(W0.n_blocks, 8);
#define SPEC_GROUPED_LAUNCH(WMV, E, W8V, XFV) gemm_bf16_kernel<2, WMV, 2, E, true, 2, W8V, XFV><<<grid, GEMM_THREADS, 0, s>>>( \
        wp, xp, out, W0.n_blocks, W0.k_steps, W0.k_steps, rows_pad / 32, rows_pad, W0.N, ldo, 0, tiles, stride16, W0.scale)
#define SPEC_GROUPED_BY_TYPE(WMV, E) do { \
        if (W0.w8) { if (W0.f16) SPEC_GROUPED_LAUNCH(WMV, E, true, XF_F16); else SPEC_GROUPED_LAUNCH(WMV, E, true, XF_HILO); } \
        else { if (W0.f16) SPEC_GROUPED_LAUNCH(WMV, E, false, XF_F16); else SPEC_GROUPED_LAUNCH(WMV, E, false, XF_HILO); } } while (0)
#define SPEC_GROUPED_LAUNCH_E(E) do { if (wide) SPEC_GROUPED_BY_TYPE(1, E); else SPEC_GROUPED_BY_TYPE(2, E); } while (0)
    if (swiglu) SPEC_GROUPED_LAUNCH_E(GEMM_EPI_SWIGLU); else SPEC_GROUPED_LAUNCH_E(GEMM_EPI_PLAIN);
#undef SPEC_GROUPED_LAUNCH_E
#undef SPEC_GROUPED_BY_TYPE
#undef SPEC_GROUPED_LAUNCH
    SPEC_LAUNCH_CHECK("gemm_bf16_kernel (grouped)");
    return SPEC_OK;
}

}  // namespace specv
