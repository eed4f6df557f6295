// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <map>
#include <string>
#include <vector>

#include "spec_verify.h"

namespace specv {

void set_error(const char* fmt, ...);
int tune(const char* name);

// per-kernel-class timing with HIP events (spec_profile_begin / spec_profile_end); prof_mark(c, s)
// is called after the launches of class c and costs one branch when profiling is off
enum ProfClass {
    PC_OTHER = 0, PC_EMBED_NORM, PC_GEMM_QKV, PC_QKV_ROPE, PC_ATTN, PC_ATTN_REDUCE, PC_GEMM_O, PC_RESID_NORM,
    PC_GEMM_GU, PC_SWIGLU, PC_GEMM_DOWN, PC_GEMM_HEAD, PC_SAMPLE_STATS, PC_SAMPLE_DRAW, PC_KV_RESERVE, PC_KV_COMMIT,
    PC_DRAFT_SAMPLE, PC_KV_TRUNCATE, PC_MOE_ROUTE, PC_MOE_GATHER, PC_NGRAM, PC_COUNT
};
extern bool g_prof_on;
void prof_record(int cls, hipStream_t s);
static inline void prof_mark(int cls, hipStream_t s) { if (g_prof_on) prof_record(cls, s); }

#define SPEC_HIP_TRY(expr)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            specv::set_error("%s failed: %s", #expr, hipGetErrorString(e_));                \
            return SPEC_EHIP;                                                               \
        }                                                                                   \
    } while (0)

#define SPEC_LAUNCH_CHECK(name)                                                             \
    do {                                                                                    \
        hipError_t e_ = hipGetLastError();                                                  \
        if (e_ != hipSuccess) {                                                             \
            specv::set_error("launch of %s failed: %s", name, hipGetErrorString(e_));       \
            return SPEC_EHIP;                                                               \
        }                                                                                   \
    } while (0)

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

typedef uint16_t bf16_t;   // raw bfloat16 bits in host-side signatures

// ---- device-resident KV bookkeeping, shared by all kernels that touch the cache ----
struct KvView {
    void* pool;                // base of the pool
    const int32_t* entry_seq;  // [B] the step's batch entries as sequence ids, -1 where the caller's id was out of range or a
                               // duplicate (written by the page reservation that opens every forward pass)
    int32_t* error;            // sticky error bits of the cache (reported by spec_kv_get_state)
    const int32_t* ctx_len;    // [max_seqs]
    const int32_t* n_held;     // [max_seqs] pages held
    const int32_t* page_table; // [max_seqs, max_pages]
    int32_t max_pages;         // per sequence
    int64_t n_pages;           // pool pages
    int32_t n_kv_heads, head_dim;
    int32_t alias_mod;
    int32_t elem_bytes;
    int32_t fp8;               // 1: blocks hold E4M3 codes of x / scale
    const float* k_scale;      // [n_layers * n_kv_heads], fp8 only
    const float* v_scale;
};

// ---- packed bf16 matrix for the MFMA GEMM (see gemm_bf16.hip for the tiling) ----
struct PackedW {
    const bf16_t* data = nullptr;  // [k_steps / 8][n_blocks][8][64 lanes][8]
    int32_t N = 0, K = 0;          // logical sizes
    int32_t n_blocks = 0;          // ceil(N / 32)
    int32_t k_steps = 0;           // K / 16
    int32_t w8 = 0;                // 1: E4M3 codes, two k-steps per 16-byte word; scale = per-column factors, tiled order
    int32_t f16 = 0;               // 1: the activations come as one fp16 per value and the weights are fp16 (converted once;
                                   //    8-bit codes are widened to fp16); 0: hi + lo bf16 pairs against bf16 weights
    const float* scale = nullptr;
};

}  // namespace specv

// rows of the output head (and entries of a logits row)
inline int head_rows(const spec_model_desc& d) { return d.head_vocab > 0 ? d.head_vocab : d.vocab; }

struct spec_model {
    spec_model_desc desc;
    int device = 0;
    std::vector<const void*> w;            // canonical pointers, borrowed
    // bf16 path: packed matrices in one arena
    void* arena = nullptr;
    size_t arena_bytes = 0;
    std::vector<specv::PackedW> wqkv, wo, wgu, wd;   // mixture of experts: wgu / wd describe expert 0, the
    std::vector<specv::PackedW> router;              // others follow at moe_gu_stride / moe_d_stride elements
    int64_t moe_gu_stride = 0, moe_d_stride = 0;
    specv::PackedW head, wfuse, wfc;
    bool moe() const { return desc.n_experts > 0; }
    int per_layer() const { return moe() ? 10 : 9; }
    const void* embed() const { return w[0]; }
    const void* layer_w(int l, int i) const { return w[1 + per_layer() * l + i]; }   // i: 0 attn_norm .. 8 wd, 9 router
    const void* final_norm() const { return w[1 + per_layer() * desc.n_layers]; }
    const void* head_w() const { return desc.tied_head ? w[0] : w[2 + per_layer() * desc.n_layers]; }
    // fuse_hidden: w_fuse, fuse_e_norm, fuse_h_norm follow the head; fuse_taps: then w_fc
    const void* fuse_w(int i) const { return w[2 + per_layer() * desc.n_layers + (desc.tied_head ? 0 : 1) + i]; }
    // 8-bit weights (dense, untied head): the scales follow everything else, 7 per layer in matrix order
    // (wq wk wv wo wg wu wd), then the head's
    const float* w_scale(int l, int i) const { return (const float*)w[3 + per_layer() * desc.n_layers + 7 * l + i]; }
    const float* head_scale() const { return (const float*)w[3 + per_layer() * desc.n_layers + 7 * desc.n_layers]; }
};

struct spec_kv {
    const spec_model* model = nullptr;
    int device = 0;
    int32_t max_seqs = 0, max_pages = 0, alias_mod = 0;
    int64_t n_pages = 0;
    void* pool = nullptr;
    const float *k_scale = nullptr, *v_scale = nullptr;   // 8-bit cache: borrowed device arrays [n_layers * n_kv_heads]
    // device state (one allocation)
    int32_t* d_state = nullptr;
    int32_t *d_ctx_len = nullptr, *d_n_held = nullptr, *d_page_table = nullptr, *d_free_stack = nullptr,
            *d_free_count = nullptr, *d_error = nullptr;
    // behind the bookkeeping (not part of a snapshot): scratch of the id check, and the checked ids of the current step
    int32_t *d_owner = nullptr, *d_entry_seq = nullptr, *d_entry_tmp = nullptr;
    int32_t* d_starved = nullptr;          // per sequence: its last reservation found no page (cleared by the commit that follows)
    size_t state_ints = 0;
    // host mirror, valid when !device_ahead
    std::vector<int32_t> h_ctx_len, h_n_held, h_page_table, h_free_stack;
    int64_t h_free_count = 0;
    bool device_ahead = false;
    // conservative bounds kept while the device is ahead of the mirror
    struct Bounds {
        int64_t max_ctx = 0;       // upper bound of the longest context
        int64_t base_pages = 0;    // pages in use at the last exact count
        int64_t added_ctx = 0;     // positions committed since (upper bound)
        int64_t touched = 0;       // batch entries stepped since (each may round up one more page)
        int64_t pages() const { return base_pages + (added_ctx + SPEC_PAGE_SIZE - 1) / SPEC_PAGE_SIZE + touched; }
    } ub;
    std::map<const void*, Bounds> snapshots;   // bounds saved with spec_kv_snapshot, by buffer
    void recount();                // exact bounds from the host mirror
    specv::KvView view() const;
};

namespace specv {

// ---- kv bookkeeping kernels (kvbook.hip) ----
spec_status launch_kv_reserve(spec_kv* kv, int B, int k, const int32_t* dev_seq_ids, hipStream_t s);
spec_status launch_kv_commit(spec_kv* kv, int B, int k, const int32_t* dev_seq_ids, const int32_t* dev_accept_len,
                             int32_t* dev_new_ctx_len, int32_t* dev_commit_slots, hipStream_t s);

spec_status launch_rollout_retire(int B, int k, int n_seqs, int32_t* slot_seq, int32_t* active, const int32_t* accept_len,
                                  int32_t* gen_len, const int32_t* target_len, const int32_t* queue, int queue_len,
                                  int32_t* queue_head, const int32_t* first_token, int32_t* tokens, int32_t* release_seq,
                                  int32_t* keep_len, int64_t* produced, hipStream_t s);
spec_status launch_rollout_pending(int B, int n_seqs, const int32_t* slot_seq_before, const int32_t* slot_seq, const int32_t* active,
                                   const int32_t* prev_token, const int32_t* first_token, int32_t* pending, hipStream_t s);
spec_status launch_rollout_pending_hidden(int B, int n_seqs, int d, const int32_t* slot_seq_before, const int32_t* slot_seq,
                                          const int32_t* active, const float* seq_hidden, float* pending_hidden, hipStream_t s);
spec_status launch_rollout_compact(int B, int k, int32_t* slot_seq, int32_t* active, int32_t* tokens, int32_t* n_live,
                                   int32_t* scratch, hipStream_t s);
spec_status launch_kv_truncate(spec_kv* kv, int B, const int32_t* dev_seq_ids, const int32_t* dev_len, int delta,
                               int32_t* dev_new_len, hipStream_t s);

// ---- fp32 generic path (forward_f32.hip) ----
size_t f32_workspace_bytes(const spec_model_desc& d, int B, int k);
spec_status f32_forward(spec_model* m, spec_kv* kv, int B, int k, const int32_t* dev_seq_ids,
                        const int32_t* dev_tokens, float* dev_logits, void* ws, hipStream_t s);

// ---- bf16 MFMA path (forward_bf16.hip, gemm_bf16.hip, attn_bf16.hip) ----
size_t bf16_packed_elems(int N, int K);
spec_status bf16_pack_matrix(const bf16_t* const* dev_parts, const int* part_rows, int n_parts, int K,
                             bf16_t* dev_out, PackedW* out, bool interleave, bool to_f16, hipStream_t s);
size_t w8_packed_bytes(int N, int K);
spec_status w8_pack_matrix(const unsigned char* const* dev_parts, const float* const* dev_scales, const int* part_rows, int n_parts,
                           int K, void* dev_out, PackedW* out, bool interleave, bool x_f16, hipStream_t s);
size_t bf16_workspace_bytes(const spec_model* m, const spec_kv* kv, int B, int k);
// hidden-state input: dev_hidden_in [M, d], or dev_features_in [M, fuse_taps * d] (one of them, models with fuse_hidden);
// outputs besides the logits: dev_hidden_out [M, d] and/or dev_taps_out [M, n_taps * d] after tap_layers[j] layers
struct Bf16Extras {
    const float* dev_hidden_in = nullptr;
    const float* dev_features_in = nullptr;
    float* dev_hidden_out = nullptr;
    int n_taps = 0;
    int tap_layers[SPEC_MAX_TAPS] = {0, 0, 0, 0};
    float* dev_taps_out = nullptr;
};
spec_status bf16_forward(spec_model* m, spec_kv* kv, int B, int k, const int32_t* dev_seq_ids,
                         const int32_t* dev_tokens, const Bf16Extras& io, float* dev_logits,
                         void* ws, size_t ws_bytes, hipStream_t s);

// in-block layouts of the cache, by storage type (host + device)
__host__ __device__ inline int64_t kv_block_offset(int dtype, int is_v, int t, int c, int head_dim)
{
    if (dtype == SPEC_F32) return (int64_t)t * head_dim + c;            // natural [t][c]
    if (dtype == SPEC_FP8_E4M3) {
        // one-byte elements, same MFMA operand order as bf16 with two fragments per 16-byte word:
        // K: [c/64][(c/8)%4][t][(c/32)%2][c%8]      V: [c/64][t/4][c%16][(c/32)%2][(c/16)%2][t%4]
        if (!is_v) return ((((int64_t)(c >> 6) * 4 + ((c >> 3) & 3)) * SPEC_PAGE_SIZE + t) * 2 + ((c >> 5) & 1)) * 8 + (c & 7);
        return (((((int64_t)(c >> 6) * 4 + (t >> 2)) * 16 + (c & 15)) * 2 + ((c >> 5) & 1)) * 2 + ((c >> 4) & 1)) * 4 + (t & 3);
    }
    if (!is_v)                                                           // K: [c/8][t][8]
        return ((int64_t)(c >> 3) * SPEC_PAGE_SIZE + t) * 8 + (c & 7);
    // V: [c/32][t/4][c%16][(c/16)%2][t%4]
    int cb = c >> 4, c1 = c & 15, g = t >> 2, j = t & 3;
    return ((((int64_t)(cb >> 1) * 4 + g) * 16 + c1) * 8) + (cb & 1) * 4 + j;
}

}  // namespace specv
