// Host side of the C ABI: handles, argument checks, cache bookkeeping mirror, dispatch to the
// fp32 or bf16 forward.  Every kernel lives in the other translation units.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>

#include "common.h"

namespace specv {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

static std::mutex g_tune_mutex;
static std::map<std::string, int>& tune_table()
{
    // launch parameters with their defaults; see gemm_bf16.hip / attn_bf16.hip for their meaning
    static std::map<std::string, int> t = {
        {"gemm_wg_target", 256},   // split K while a GEMM launches fewer workgroups than this
        {"fuse_swiglu", 1},        // 1: silu(gate) * up in the gate/up projection's epilogue (unsplit K, even row blocks)
        {"attn_row_blocks", 0},    // most 16-row blocks per attention workgroup (1..4; 0 = up to 4, groups as equal as possible)
        {"gemm_max_mb", 4},        // 32-row blocks per GEMM tile (1..4): smaller tiles = more workgroups, weights read once per tile
        {"gemm_split_rows", 2},     // GEMMs of up to this many 128-row tiles (97..256 rows at 2) run as 64-row x 256-column tiles instead (0 = never)
        {"gemm_big_min_tiles", 200}, // a GEMM with at least this many 256-column tiles takes them without further conditions
        {"gemm_tiles_96", 1},       // 129..256 rows, fused gate/up projection: two 96- or 128-row x 256-column tiles per column stripe instead of three or four 64-row ones
        {"gemm_wide4", 400},        // single-tile 128-row GEMMs with a plain epilogue take 128 x 256 tiles from this many such tiles on (0 = never)
        {"gemm_one_block", 1},      // 97..128 rows, fp16 activations: one 128 x 128 tile, wavefronts 1 x 4 with one column block each (0: as with hi + lo operands)
        {"moe_wide_tiles", 1},      // grouped expert GEMMs: 64 x 256 tiles, wavefronts 1 x 4 (0: 64 x 128, wavefronts 2 x 2)
        {"gemm_big_min_blocks", 5}, // from this many 32-row blocks on, a GEMM may take 192/256-row x 256-column tiles (0 = never)
        {"gemm_min_ksteps", 32},   // never split below this many 16-wide k-steps per workgroup
        {"splits_qkv", 0}, {"splits_o", 0}, {"splits_gu", 0}, {"splits_down", 0}, {"splits_head", 0},   // 0 = auto
        {"attn_chunk_pages", 0},   // KV pages per attention workgroup (a multiple of 4 up to 256; 0 = chosen on the device from the batch's contexts)
        {"attn_rounds", 1},        // the attention's work list is cut to fill the chip's resident workgroups this many times over (B=32, contexts 1k..8k: 3.41 ms of attention per step at 1, 3.54 at 2, 3.60 at 3)
        {"attn_min_pages", 16},    // shortest chunk the device-side choice may take (pages)
        // Which projections take one fp16 activation per value (one MFMA per weight fragment, weights tiled as fp16) instead of
        // hi + lo bf16 pairs (two MFMAs): bit 0 QKV, 1 attention output, 2 feed-forward (gate/up and down, experts included),
        // 3 output head.  Read at spec_model_create.  Default 12: the feed-forward and the head; the attention block's inputs
        // carry most of the logits error and stay hi + lo.
        {"gemm_f16_inputs", 12},
    };
    return t;
}

int tune(const char* name)
{
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    auto it = tune_table().find(name);
    return it == tune_table().end() ? 0 : it->second;
}

bool g_prof_on = false;
static std::vector<hipEvent_t> g_prof_events;
static std::vector<int> g_prof_class;
static size_t g_prof_used = 0;

void prof_record(int cls, hipStream_t s)
{
    if (g_prof_used >= g_prof_events.size()) return;           // out of events: the tail is not timed
    if (hipEventRecord(g_prof_events[g_prof_used], s) != hipSuccess) return;
    g_prof_class[g_prof_used++] = cls;
}

static const char* const PROF_NAMES[PC_COUNT] = {
    "other", "embed_norm", "gemm_qkv", "qkv_rope", "attn", "attn_reduce", "gemm_o", "resid_norm", "gemm_gu", "swiglu",
    "gemm_down", "gemm_head", "sample_stats", "sample_draw", "kv_reserve", "kv_commit", "draft_sample", "kv_truncate", "moe_route", "moe_gather", "ngram"};

}  // namespace specv

using namespace specv;

extern "C" int32_t spec_profile_class_count(void) { return PC_COUNT; }
extern "C" const char* spec_profile_class_name(int32_t c) { return c >= 0 && c < PC_COUNT ? PROF_NAMES[c] : nullptr; }

extern "C" spec_status spec_profile_begin(int32_t max_events)
{
    if (max_events < 2 || max_events > (1 << 22)) { set_error("spec_profile_begin: max_events out of range"); return SPEC_EINVAL; }
    while (g_prof_events.size() < (size_t)max_events) {
        hipEvent_t e;
        SPEC_HIP_TRY(hipEventCreate(&e));
        g_prof_events.push_back(e);
    }
    g_prof_class.assign(g_prof_events.size(), 0);
    g_prof_used = 0;
    g_prof_on = true;
    return SPEC_OK;
}

extern "C" spec_status spec_profile_end(double* host_ms, int64_t* host_counts, int32_t n)
{
    if (!g_prof_on) { set_error("spec_profile_end: profiling is not on"); return SPEC_ESTATE; }
    g_prof_on = false;
    if (!host_ms || !host_counts || n < PC_COUNT) { set_error("spec_profile_end: need %d slots", (int)PC_COUNT); return SPEC_EINVAL; }
    SPEC_HIP_TRY(hipDeviceSynchronize());
    for (int i = 0; i < n; ++i) { host_ms[i] = 0.0; host_counts[i] = 0; }
    for (size_t i = 1; i < g_prof_used; ++i) {
        float ms = 0.f;
        SPEC_HIP_TRY(hipEventElapsedTime(&ms, g_prof_events[i - 1], g_prof_events[i]));
        host_ms[g_prof_class[i]] += ms;
        host_counts[g_prof_class[i]] += 1;
    }
    return SPEC_OK;
}

extern "C" const char* spec_last_error(void) { return g_error; }

extern "C" spec_status spec_tune_set(const char* name, int32_t value)
{
    if (!name) { set_error("spec_tune_set: null name"); return SPEC_EINVAL; }
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    auto it = tune_table().find(name);
    if (it == tune_table().end()) { set_error("spec_tune_set: unknown parameter '%s'", name); return SPEC_EINVAL; }
    if (value < 0) { set_error("spec_tune_set: negative value"); return SPEC_EINVAL; }
    it->second = value;
    return SPEC_OK;
}

extern "C" int32_t spec_tune_get(const char* name)
{
    if (!name) return -1;
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    auto it = tune_table().find(name);
    return it == tune_table().end() ? -1 : it->second;
}

// ------------------------------------------------------------------------------------------ model

extern "C" int32_t spec_model_weight_count(const spec_model_desc* d)
{
    if (!d || d->n_layers < 0) return -1;
    return 1 + (9 + (d->n_experts > 0 ? 1 : 0)) * d->n_layers + 1 + (d->tied_head ? 0 : 1) + (d->fuse_hidden ? 3 : 0) + (d->fuse_taps ? 1 : 0) +
           (d->w_dtype == SPEC_FP8_E4M3 ? 7 * d->n_layers + 1 : 0);
}

static spec_status check_desc(const spec_model_desc& d)
{
    if (d.n_layers < 1 || d.d_model < 1 || d.n_q_heads < 1 || d.n_kv_heads < 1 || d.head_dim < 2 || d.ffn_dim < 1 ||
        d.vocab < 1 || !(d.rope_theta > 0.f) || !(d.rms_eps >= 0.f)) {
        set_error("spec_model_create: non-positive size in the description");
        return SPEC_EINVAL;
    }
    if (d.n_q_heads % d.n_kv_heads) { set_error("spec_model_create: n_q_heads must be a multiple of n_kv_heads"); return SPEC_EUNSUPPORTED; }
    if (d.dtype != SPEC_F32 && d.dtype != SPEC_BF16) { set_error("spec_model_create: unknown dtype"); return SPEC_EINVAL; }
    if (d.n_experts < 0 || d.top_k < 0 || d.expert_ffn_dim < 0) { set_error("spec_model_create: negative mixture-of-experts size"); return SPEC_EINVAL; }
    if (d.n_experts > 0) {
        if (d.dtype != SPEC_BF16) { set_error("spec_model_create: the fp32 path is dense only"); return SPEC_EUNSUPPORTED; }
        if (d.n_experts > 256 || d.top_k < 1 || d.top_k > 16 || d.top_k > d.n_experts || d.expert_ffn_dim < 1 || d.expert_ffn_dim % 256) {
            set_error("spec_model_create: mixture of experts needs n_experts <= 256, 1 <= top_k <= min(n_experts, 16), expert_ffn_dim %% 256 == 0");
            return SPEC_EUNSUPPORTED;
        }
    }
    if (d.kv_dtype != 0 && !(d.kv_dtype == SPEC_FP8_E4M3 && d.dtype == SPEC_BF16)) {
        set_error("spec_model_create: kv_dtype must be 0 or SPEC_FP8_E4M3 (bf16 models only)");
        return SPEC_EUNSUPPORTED;
    }
    if (d.w_dtype != 0 && !(d.w_dtype == SPEC_FP8_E4M3 && d.dtype == SPEC_BF16 && !d.fuse_hidden && !d.tied_head)) {
        set_error("spec_model_create: w_dtype must be 0 or SPEC_FP8_E4M3 (bf16, untied head, no hidden-state input)");
        return SPEC_EUNSUPPORTED;
    }
    if (d.fuse_hidden) {
        if (d.dtype != SPEC_BF16 || d.n_experts > 0 || d.ffn_dim < 2 * d.d_model) {
            set_error("spec_model_create: a model with hidden-state input must be bf16, dense, with ffn_dim >= 2 * d_model");
            return SPEC_EUNSUPPORTED;
        }
    }
    if (d.head_vocab < 0 || (d.head_vocab > 0 && d.tied_head)) {
        set_error("spec_model_create: head_vocab must be 0 or the row count of an untied head");
        return SPEC_EINVAL;
    }
    if (d.fuse_taps < 0 || d.fuse_taps > SPEC_MAX_TAPS || (d.fuse_taps && !d.fuse_hidden)) {
        set_error("spec_model_create: fuse_taps must be 0 .. %d and needs fuse_hidden", SPEC_MAX_TAPS);
        return SPEC_EINVAL;
    }
    if (d.dtype == SPEC_BF16) {
        if (d.head_dim != 128 || d.d_model % 256 || d.ffn_dim % 256) {
            set_error("spec_model_create: the bf16 path needs head_dim == 128 and d_model, ffn_dim multiples of 256");
            return SPEC_EUNSUPPORTED;
        }
        int rows = d.n_q_heads / d.n_kv_heads;
        if (rows * (SPEC_MAX_DRAFT + 1) > 256 && rows > 16) { set_error("spec_model_create: more than 16 query heads per kv head"); return SPEC_EUNSUPPORTED; }
    }
    return SPEC_OK;
}

extern "C" spec_status spec_model_create(const spec_model_desc* desc, const void* const* dev_weights, int32_t n_weights,
                                         spec_model** out)
{
    if (!desc || !dev_weights || !out) { set_error("spec_model_create: null pointer"); return SPEC_EINVAL; }
    spec_status st = check_desc(*desc);
    if (st != SPEC_OK) return st;
    if (n_weights != spec_model_weight_count(desc)) {
        set_error("spec_model_create: expected %d weight pointers, got %d", spec_model_weight_count(desc), n_weights);
        return SPEC_EINVAL;
    }
    for (int i = 0; i < n_weights; ++i)
        if (!dev_weights[i]) { set_error("spec_model_create: weight pointer %d is null", i); return SPEC_EINVAL; }
    spec_model* m = new (std::nothrow) spec_model();
    if (!m) { set_error("spec_model_create: out of host memory"); return SPEC_ENOMEM; }
    m->desc = *desc;
    m->w.assign(dev_weights, dev_weights + n_weights);
    SPEC_HIP_TRY(hipGetDevice(&m->device));

    if (desc->dtype == SPEC_BF16 && desc->w_dtype == SPEC_FP8_E4M3) {
        // 8-bit weights: codes and scales re-tiled into one arena, matrix by matrix
        const spec_model_desc& d = *desc;
        const int L = d.n_layers, D = d.d_model, F = d.ffn_dim;
        const int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim;
        const int E = d.n_experts, Fe = d.expert_ffn_dim;
        m->arena_bytes = (size_t)L * (w8_packed_bytes(nq + 2 * nkv, D) + w8_packed_bytes(D, nq)) + w8_packed_bytes(head_rows(d), D);
        if (E > 0)       // every expert's region (codes, then scales) on its own; the router stays a bf16 matrix
            m->arena_bytes += (size_t)L * ((size_t)E * (w8_packed_bytes(2 * Fe, D) + w8_packed_bytes(D, Fe)) + align_up(bf16_packed_elems(E, D) * sizeof(bf16_t), 256));
        else
            m->arena_bytes += (size_t)L * (w8_packed_bytes(2 * F, D) + w8_packed_bytes(D, F));
        hipError_t e = hipMalloc(&m->arena, m->arena_bytes);
        if (e != hipSuccess) {
            set_error("spec_model_create: hipMalloc of %zu bytes for the tiled weights failed: %s", m->arena_bytes, hipGetErrorString(e));
            delete m;
            return SPEC_ENOMEM;
        }
        char* at = (char*)m->arena;
        m->wqkv.resize(L); m->wo.resize(L); m->wgu.resize(L); m->wd.resize(L); m->router.resize(L);
        const int f16_mask = tune("gemm_f16_inputs");
        auto pack8 = [&](std::initializer_list<const void*> parts, std::initializer_list<const float*> scales, std::initializer_list<int> rows,
                         int K, PackedW* pw, bool x_f16, bool interleave = false) -> spec_status {
            std::vector<const unsigned char*> p;
            for (auto q : parts) p.push_back((const unsigned char*)q);
            std::vector<const float*> sc(scales);
            std::vector<int> r(rows);
            int N = 0;
            for (int x : r) N += x;
            spec_status s2 = w8_pack_matrix(p.data(), sc.data(), r.data(), (int)p.size(), K, at, pw, interleave, x_f16, nullptr);
            at += w8_packed_bytes(N, K);
            return s2;
        };
        for (int l = 0; l < L && st == SPEC_OK; ++l) {
            st = pack8({m->layer_w(l, 1), m->layer_w(l, 2), m->layer_w(l, 3)}, {m->w_scale(l, 0), m->w_scale(l, 1), m->w_scale(l, 2)}, {nq, nkv, nkv}, D, &m->wqkv[l], f16_mask & 1);
            if (st == SPEC_OK) st = pack8({m->layer_w(l, 4)}, {m->w_scale(l, 3)}, {D}, nq, &m->wo[l], f16_mask & 2);
            if (E > 0) {
                const unsigned char *wg = (const unsigned char*)m->layer_w(l, 6), *wu = (const unsigned char*)m->layer_w(l, 7),
                                    *wdn = (const unsigned char*)m->layer_w(l, 8);
                const float *sg = m->w_scale(l, 4), *su = m->w_scale(l, 5), *sd = m->w_scale(l, 6);
                m->moe_gu_stride = (int64_t)w8_packed_bytes(2 * Fe, D);       // bytes: see launch_gemm_bf16_grouped
                m->moe_d_stride = (int64_t)w8_packed_bytes(D, Fe);
                PackedW tmp;
                for (int e2 = 0; e2 < E && st == SPEC_OK; ++e2)
                    st = pack8({wg + (size_t)e2 * Fe * D, wu + (size_t)e2 * Fe * D}, {sg + (size_t)e2 * Fe, su + (size_t)e2 * Fe}, {Fe, Fe}, D,
                               e2 == 0 ? &m->wgu[l] : &tmp, f16_mask & 4, true);
                for (int e2 = 0; e2 < E && st == SPEC_OK; ++e2)
                    st = pack8({wdn + (size_t)e2 * D * Fe}, {sd + (size_t)e2 * D}, {D}, Fe, e2 == 0 ? &m->wd[l] : &tmp, f16_mask & 4);
                if (st == SPEC_OK) {
                    const bf16_t* rp = (const bf16_t*)m->layer_w(l, 9);
                    const int rows = E;
                    st = bf16_pack_matrix(&rp, &rows, 1, D, (bf16_t*)at, &m->router[l], false, false, nullptr);
                    at += align_up(bf16_packed_elems(E, D) * sizeof(bf16_t), 256);
                }
            } else {
                if (st == SPEC_OK) st = pack8({m->layer_w(l, 6), m->layer_w(l, 7)}, {m->w_scale(l, 4), m->w_scale(l, 5)}, {F, F}, D, &m->wgu[l], f16_mask & 4, true);
                if (st == SPEC_OK) st = pack8({m->layer_w(l, 8)}, {m->w_scale(l, 6)}, {D}, F, &m->wd[l], f16_mask & 4);
            }
        }
        if (st == SPEC_OK) st = pack8({m->head_w()}, {m->head_scale()}, {head_rows(d)}, D, &m->head, f16_mask & 8);
        if (st == SPEC_OK && hipDeviceSynchronize() != hipSuccess) { set_error("spec_model_create: weight tiling failed on the device"); st = SPEC_EHIP; }
        if (st != SPEC_OK) { (void)hipFree(m->arena); delete m; return st; }
    } else if (desc->dtype == SPEC_BF16) {
        const spec_model_desc& d = *desc;
        int L = d.n_layers, D = d.d_model, F = d.ffn_dim;
        int nq = d.n_q_heads * d.head_dim, nkv = d.n_kv_heads * d.head_dim;
        const int E = d.n_experts, Fe = d.expert_ffn_dim;
        size_t elems = 0;
        elems += (size_t)L * (bf16_packed_elems(nq + 2 * nkv, D) + bf16_packed_elems(D, nq));
        if (E > 0) elems += (size_t)L * ((size_t)E * (bf16_packed_elems(2 * Fe, D) + bf16_packed_elems(D, Fe)) + bf16_packed_elems(E, D));
        else elems += (size_t)L * (bf16_packed_elems(2 * F, D) + bf16_packed_elems(D, F));
        elems += bf16_packed_elems(head_rows(d), D);
        if (d.fuse_hidden) elems += bf16_packed_elems(D, 2 * D);
        if (d.fuse_taps) elems += bf16_packed_elems(D, d.fuse_taps * D);
        m->arena_bytes = elems * sizeof(bf16_t);
        hipError_t e = hipMalloc(&m->arena, m->arena_bytes);
        if (e != hipSuccess) {
            set_error("spec_model_create: hipMalloc of %zu bytes for the tiled weights failed: %s", m->arena_bytes, hipGetErrorString(e));
            delete m;
            return SPEC_ENOMEM;
        }
        bf16_t* at = (bf16_t*)m->arena;
        m->wqkv.resize(L); m->wo.resize(L); m->wgu.resize(L); m->wd.resize(L); m->router.resize(L);
        const int f16_mask = tune("gemm_f16_inputs");
        auto pack = [&](std::initializer_list<const void*> parts, std::initializer_list<int> rows, int K, PackedW* pw, bool to_f16, bool interleave = false) -> spec_status {
            std::vector<const bf16_t*> p;
            for (auto q : parts) p.push_back((const bf16_t*)q);
            std::vector<int> r(rows);
            int N = 0;
            for (int x : r) N += x;
            spec_status s2 = bf16_pack_matrix(p.data(), r.data(), (int)p.size(), K, at, pw, interleave, to_f16, nullptr);
            at += bf16_packed_elems(N, K);
            return s2;
        };
        for (int l = 0; l < L && st == SPEC_OK; ++l) {
            st = pack({m->layer_w(l, 1), m->layer_w(l, 2), m->layer_w(l, 3)}, {nq, nkv, nkv}, D, &m->wqkv[l], f16_mask & 1);
            if (st == SPEC_OK) st = pack({m->layer_w(l, 4)}, {D}, nq, &m->wo[l], f16_mask & 2);
            if (E > 0) {
                // every expert re-tiled on its own, all experts of a matrix back to back (equal sizes)
                const bf16_t *wg = (const bf16_t*)m->layer_w(l, 6), *wu = (const bf16_t*)m->layer_w(l, 7), *wdn = (const bf16_t*)m->layer_w(l, 8);
                m->moe_gu_stride = (int64_t)bf16_packed_elems(2 * Fe, D);
                m->moe_d_stride = (int64_t)bf16_packed_elems(D, Fe);
                PackedW tmp;
                for (int e = 0; e < E && st == SPEC_OK; ++e)
                    st = pack({wg + (size_t)e * Fe * D, wu + (size_t)e * Fe * D}, {Fe, Fe}, D, e == 0 ? &m->wgu[l] : &tmp, f16_mask & 4, true);
                for (int e = 0; e < E && st == SPEC_OK; ++e)
                    st = pack({wdn + (size_t)e * D * Fe}, {D}, Fe, e == 0 ? &m->wd[l] : &tmp, f16_mask & 4);
                if (st == SPEC_OK) st = pack({m->layer_w(l, 9)}, {E}, D, &m->router[l], false);
            } else {
                if (st == SPEC_OK) st = pack({m->layer_w(l, 6), m->layer_w(l, 7)}, {F, F}, D, &m->wgu[l], f16_mask & 4, true);
                if (st == SPEC_OK) st = pack({m->layer_w(l, 8)}, {D}, F, &m->wd[l], f16_mask & 4);
            }
        }
        if (st == SPEC_OK) st = pack({m->head_w()}, {head_rows(d)}, D, &m->head, f16_mask & 8);
        if (st == SPEC_OK && d.fuse_hidden) st = pack({m->fuse_w(0)}, {D}, 2 * D, &m->wfuse, false);
        if (st == SPEC_OK && d.fuse_taps) st = pack({m->fuse_w(3)}, {D}, d.fuse_taps * D, &m->wfc, false);
        if (st == SPEC_OK && hipDeviceSynchronize() != hipSuccess) { set_error("spec_model_create: weight tiling failed on the device"); st = SPEC_EHIP; }
        if (st != SPEC_OK) { (void)hipFree(m->arena); delete m; return st; }
    }
    *out = m;
    return SPEC_OK;
}

extern "C" spec_status spec_model_destroy(spec_model* m)
{
    if (!m) return SPEC_OK;
    if (m->arena) (void)hipFree(m->arena);
    delete m;
    return SPEC_OK;
}

// ------------------------------------------------------------------------------------------ cache

static int elem_bytes(int dtype) { return dtype == SPEC_F32 ? 4 : dtype == SPEC_FP8_E4M3 ? 1 : 2; }
// storage type of the cache's blocks
static int kv_storage(const spec_model_desc& d) { return d.kv_dtype == SPEC_FP8_E4M3 ? SPEC_FP8_E4M3 : d.dtype; }

void spec_kv::recount()
{
    ub = Bounds();
    for (int s = 0; s < max_seqs; ++s) {
        if (h_ctx_len[s] > ub.max_ctx) ub.max_ctx = h_ctx_len[s];
        ub.base_pages += h_n_held[s];
    }
}

specv::KvView spec_kv::view() const
{
    KvView v;
    v.pool = pool;
    v.entry_seq = d_entry_seq;
    v.error = d_error;
    v.ctx_len = d_ctx_len;
    v.n_held = d_n_held;
    v.page_table = d_page_table;
    v.max_pages = max_pages;
    v.n_pages = n_pages;
    v.n_kv_heads = model->desc.n_kv_heads;
    v.head_dim = model->desc.head_dim;
    v.alias_mod = alias_mod;
    v.elem_bytes = elem_bytes(kv_storage(model->desc));
    v.fp8 = model->desc.kv_dtype == SPEC_FP8_E4M3;
    v.k_scale = k_scale;
    v.v_scale = v_scale;
    return v;
}

extern "C" int64_t spec_kv_pool_bytes(const spec_model* m, int64_t n_pages, int32_t alias)
{
    if (!m || n_pages < 1 || alias < 0) return -1;
    int pools = alias > 0 ? (alias < m->desc.n_layers ? alias : m->desc.n_layers) : m->desc.n_layers;
    return (int64_t)pools * n_pages * 2 * m->desc.n_kv_heads * SPEC_PAGE_SIZE * m->desc.head_dim * elem_bytes(kv_storage(m->desc));
}

extern "C" spec_status spec_kv_alloc(const spec_model* m, int32_t max_seqs, int32_t max_ctx_len, int64_t n_pages,
                                     void* dev_pool, int32_t alias, spec_kv** out)
{
    if (!m || !dev_pool || !out) { set_error("spec_kv_alloc: null pointer"); return SPEC_EINVAL; }
    if (max_seqs < 1 || max_ctx_len < 1 || n_pages < 1 || n_pages > (1 << 27) || alias < 0) {
        set_error("spec_kv_alloc: size out of range");
        return SPEC_EINVAL;
    }
    spec_kv* kv = new (std::nothrow) spec_kv();
    if (!kv) { set_error("spec_kv_alloc: out of host memory"); return SPEC_ENOMEM; }
    kv->model = m;
    kv->device = m->device;
    kv->max_seqs = max_seqs;
    kv->max_pages = (int32_t)cdiv(max_ctx_len, SPEC_PAGE_SIZE);
    kv->alias_mod = alias;
    kv->n_pages = n_pages;
    kv->pool = dev_pool;
    kv->state_ints = (size_t)max_seqs * 2 + (size_t)max_seqs * kv->max_pages + (size_t)n_pages + 2;
    hipError_t e = hipMalloc((void**)&kv->d_state, (kv->state_ints + 4 * (size_t)max_seqs) * sizeof(int32_t));
    if (e != hipSuccess) { set_error("spec_kv_alloc: hipMalloc failed: %s", hipGetErrorString(e)); delete kv; return SPEC_ENOMEM; }
    int32_t* p = kv->d_state;
    kv->d_ctx_len = p; p += max_seqs;
    kv->d_n_held = p; p += max_seqs;
    kv->d_page_table = p; p += (size_t)max_seqs * kv->max_pages;
    kv->d_free_stack = p; p += n_pages;
    kv->d_free_count = p; p += 1;
    kv->d_error = p; p += 1;
    kv->d_owner = p; p += max_seqs;
    kv->d_entry_seq = p; p += max_seqs;
    kv->d_entry_tmp = p; p += max_seqs;
    kv->d_starved = p;
    kv->h_ctx_len.assign(max_seqs, 0);
    kv->h_n_held.assign(max_seqs, 0);
    kv->h_page_table.assign((size_t)max_seqs * kv->max_pages, -1);
    kv->h_free_stack.resize(n_pages);
    for (int64_t i = 0; i < n_pages; ++i) kv->h_free_stack[i] = (int32_t)(n_pages - 1 - i);   // top of stack = page 0
    kv->h_free_count = n_pages;
    kv->device_ahead = false;
    // upload
    std::vector<int32_t> img(kv->state_ints + 4 * (size_t)max_seqs, 0);
    std::fill(img.begin() + kv->state_ints, img.begin() + kv->state_ints + max_seqs, 0x7fffffff);       // d_owner
    std::fill(img.begin() + kv->state_ints + max_seqs, img.begin() + kv->state_ints + 3 * (size_t)max_seqs, -1);   // entry ids; d_starved stays 0
    std::fill(img.begin() + 2 * max_seqs, img.begin() + 2 * max_seqs + (size_t)max_seqs * kv->max_pages, -1);
    std::copy(kv->h_free_stack.begin(), kv->h_free_stack.end(), img.begin() + 2 * max_seqs + (size_t)max_seqs * kv->max_pages);
    img[kv->state_ints - 2] = (int32_t)n_pages;
    e = hipMemcpy(kv->d_state, img.data(), img.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) { set_error("spec_kv_alloc: upload failed: %s", hipGetErrorString(e)); (void)hipFree(kv->d_state); delete kv; return SPEC_EHIP; }
    *out = kv;
    return SPEC_OK;
}

extern "C" spec_status spec_kv_free(spec_kv* kv)
{
    if (!kv) return SPEC_OK;
    if (kv->d_state) (void)hipFree(kv->d_state);
    delete kv;
    return SPEC_OK;
}

extern "C" spec_status spec_kv_set_scales(spec_kv* kv, const float* dev_k_scale, const float* dev_v_scale)
{
    if (!kv || !dev_k_scale || !dev_v_scale) { set_error("spec_kv_set_scales: null pointer"); return SPEC_EINVAL; }
    if (kv->model->desc.kv_dtype != SPEC_FP8_E4M3) { set_error("spec_kv_set_scales: not an 8-bit cache"); return SPEC_EINVAL; }
    kv->k_scale = dev_k_scale;
    kv->v_scale = dev_v_scale;
    return SPEC_OK;
}

extern "C" int32_t spec_kv_max_pages_per_seq(const spec_kv* kv) { return kv ? kv->max_pages : -1; }

extern "C" int64_t spec_kv_block_offset(const spec_kv* kv, int32_t is_v, int32_t t, int32_t c)
{
    if (!kv || t < 0 || t >= SPEC_PAGE_SIZE || c < 0 || c >= kv->model->desc.head_dim || (is_v != 0 && is_v != 1)) return -1;
    return kv_block_offset(kv_storage(kv->model->desc), is_v, t, c, kv->model->desc.head_dim);
}

extern "C" int64_t spec_kv_block_base(const spec_kv* kv, int32_t layer, int64_t page, int32_t is_v, int32_t h)
{
    if (!kv) return -1;
    const spec_model_desc& d = kv->model->desc;
    if (layer < 0 || layer >= d.n_layers || page < 0 || page >= kv->n_pages || (is_v != 0 && is_v != 1) || h < 0 || h >= d.n_kv_heads) return -1;
    int lp = kv->alias_mod > 0 ? layer % kv->alias_mod : layer;
    return ((((int64_t)lp * kv->n_pages + page) * 2 + is_v) * d.n_kv_heads + h) * SPEC_PAGE_SIZE * d.head_dim;
}

// bring the host mirror up to date with the device (synchronises)
static spec_status kv_download(spec_kv* kv, int32_t* err_bits)
{
    SPEC_HIP_TRY(hipDeviceSynchronize());
    std::vector<int32_t> img(kv->state_ints);
    SPEC_HIP_TRY(hipMemcpy(img.data(), kv->d_state, img.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    size_t S = kv->max_seqs, PT = (size_t)kv->max_seqs * kv->max_pages;
    std::copy(img.begin(), img.begin() + S, kv->h_ctx_len.begin());
    std::copy(img.begin() + S, img.begin() + 2 * S, kv->h_n_held.begin());
    std::copy(img.begin() + 2 * S, img.begin() + 2 * S + PT, kv->h_page_table.begin());
    std::copy(img.begin() + 2 * S + PT, img.begin() + 2 * S + PT + kv->n_pages, kv->h_free_stack.begin());
    kv->h_free_count = img[kv->state_ints - 2];
    if (err_bits) *err_bits = img[kv->state_ints - 1];
    if (img[kv->state_ints - 1] != 0) {
        int32_t zero = 0;
        SPEC_HIP_TRY(hipMemcpy(kv->d_error, &zero, sizeof(zero), hipMemcpyHostToDevice));
    }
    kv->device_ahead = false;
    kv->recount();
    return SPEC_OK;
}

extern "C" spec_status spec_kv_seq_assign(spec_kv* kv, int32_t seq, int32_t ctx_len, const int32_t* host_page_ids, int32_t n_ids)
{
    if (!kv) { set_error("spec_kv_seq_assign: null handle"); return SPEC_EINVAL; }
    if (seq < 0 || seq >= kv->max_seqs || ctx_len < 0) { set_error("spec_kv_seq_assign: seq or ctx_len out of range"); return SPEC_EINVAL; }
    int need = (int)cdiv(ctx_len, SPEC_PAGE_SIZE);
    if (n_ids != need || need > kv->max_pages || (need > 0 && !host_page_ids)) {
        set_error("spec_kv_seq_assign: %d page ids given, context of %d tokens needs %d (at most %d per sequence)", n_ids, ctx_len, need, kv->max_pages);
        return SPEC_EINVAL;
    }
    if (kv->device_ahead) {
        spec_status st = kv_download(kv, nullptr);
        if (st != SPEC_OK) return st;
    }
    // pages the sequence held so far go back to the stack (last page first)
    std::vector<int32_t> stack(kv->h_free_stack.begin(), kv->h_free_stack.begin() + kv->h_free_count);
    for (int j = kv->h_n_held[seq] - 1; j >= 0; --j) stack.push_back(kv->h_page_table[(size_t)seq * kv->max_pages + j]);
    for (int j = 0; j < need; ++j) {
        int32_t p = host_page_ids[j];
        auto it = std::find(stack.begin(), stack.end(), p);
        if (p < 0 || p >= kv->n_pages || it == stack.end()) { set_error("spec_kv_seq_assign: page %d is out of range or in use", p); return SPEC_EINVAL; }
        stack.erase(it);
    }
    for (int j = 0; j < kv->max_pages; ++j) kv->h_page_table[(size_t)seq * kv->max_pages + j] = j < need ? host_page_ids[j] : -1;
    kv->h_ctx_len[seq] = ctx_len;
    kv->h_n_held[seq] = need;
    std::copy(stack.begin(), stack.end(), kv->h_free_stack.begin());
    kv->h_free_count = (int64_t)stack.size();
    // upload the touched parts
    size_t S = kv->max_seqs;
    SPEC_HIP_TRY(hipMemcpy(kv->d_ctx_len + seq, &kv->h_ctx_len[seq], sizeof(int32_t), hipMemcpyHostToDevice));
    SPEC_HIP_TRY(hipMemcpy(kv->d_n_held + seq, &kv->h_n_held[seq], sizeof(int32_t), hipMemcpyHostToDevice));
    SPEC_HIP_TRY(hipMemcpy(kv->d_page_table + (size_t)seq * kv->max_pages, &kv->h_page_table[(size_t)seq * kv->max_pages],
                           kv->max_pages * sizeof(int32_t), hipMemcpyHostToDevice));
    SPEC_HIP_TRY(hipMemcpy(kv->d_free_stack, kv->h_free_stack.data(), kv->n_pages * sizeof(int32_t), hipMemcpyHostToDevice));
    int32_t fc = (int32_t)kv->h_free_count;
    SPEC_HIP_TRY(hipMemcpy(kv->d_free_count, &fc, sizeof(int32_t), hipMemcpyHostToDevice));
    (void)S;
    kv->recount();
    return SPEC_OK;
}

extern "C" spec_status spec_kv_get_state(spec_kv* kv, int32_t* host_ctx_len, int32_t* host_n_pages, int32_t* host_page_table,
                                         int32_t* host_free_stack, int64_t* host_n_free)
{
    if (!kv) { set_error("spec_kv_get_state: null handle"); return SPEC_EINVAL; }
    int32_t err = 0;
    spec_status st = kv_download(kv, &err);
    if (st != SPEC_OK) return st;
    if (host_ctx_len) std::copy(kv->h_ctx_len.begin(), kv->h_ctx_len.end(), host_ctx_len);
    if (host_n_pages) std::copy(kv->h_n_held.begin(), kv->h_n_held.end(), host_n_pages);
    if (host_page_table) std::copy(kv->h_page_table.begin(), kv->h_page_table.end(), host_page_table);
    if (host_free_stack) std::copy(kv->h_free_stack.begin(), kv->h_free_stack.end(), host_free_stack);
    if (host_n_free) *host_n_free = kv->h_free_count;
    if (err & 1) { set_error("a step ran out of KV pages; its sequences were left without new pages"); return SPEC_ENOMEM; }
    if (err & 2) { set_error("a step was given a sequence id out of range, or the same id twice: those batch entries were left out"); return SPEC_EINVAL; }
    if (err & 8) { set_error("a step met contexts longer than the bound its launch was sized for (a graph replayed from a longer cache state?): its logits are not valid"); return SPEC_ESTATE; }
    if (err & 4) { set_error("a sequence outgrew max_ctx_len"); return SPEC_EINVAL; }
    return SPEC_OK;
}

// ------------------------------------------------------------------------------------------ the step

extern "C" size_t spec_verify_workspace_bytes(const spec_model* m, const spec_kv* kv, int32_t B, int32_t k)
{
    if (!m || !kv || kv->model != m || B < 1 || k < 0 || k > SPEC_MAX_DRAFT) return 0;
    return m->desc.dtype == SPEC_F32 ? f32_workspace_bytes(m->desc, B, k) : bf16_workspace_bytes(m, kv, B, k);
}

static spec_status verify_forward_any(spec_model* m, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                      const int32_t* dev_tokens, const Bf16Extras& io, float* dev_logits,
                                      void* ws, size_t ws_bytes, void* stream)
{
    const float* dev_hidden_in = io.dev_hidden_in ? io.dev_hidden_in : io.dev_features_in;
    float* dev_hidden_out = io.dev_hidden_out ? io.dev_hidden_out : io.dev_taps_out;
    if (!m || !kv || !dev_seq_ids || !dev_tokens || !dev_logits || !ws) { set_error("spec_verify_forward: null pointer"); return SPEC_EINVAL; }
    if (kv->model != m) { set_error("spec_verify_forward: the cache belongs to another model"); return SPEC_EINVAL; }
    if ((m->desc.fuse_hidden != 0) != (dev_hidden_in != nullptr)) {
        set_error("spec_verify_forward: hidden-state input %s", m->desc.fuse_hidden ? "is required by this model (spec_verify_forward_hidden)" : "given to a model that takes none");
        return SPEC_EINVAL;
    }
    if (dev_hidden_out && m->desc.dtype != SPEC_BF16) { set_error("spec_verify_forward_hidden: hidden-state output needs a bf16 model"); return SPEC_EUNSUPPORTED; }
    if (B < 1 || B > kv->max_seqs || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_verify_forward: B or k out of range"); return SPEC_EINVAL; }
    if (m->desc.kv_dtype == SPEC_FP8_E4M3 && !(kv->k_scale && kv->v_scale)) { set_error("spec_verify_forward: the 8-bit cache has no scales yet (spec_kv_set_scales)"); return SPEC_ESTATE; }
    if (ws_bytes < spec_verify_workspace_bytes(m, kv, B, k)) { set_error("spec_verify_forward: workspace too small (%zu < %zu)", ws_bytes, spec_verify_workspace_bytes(m, kv, B, k)); return SPEC_EINVAL; }
    if (((uintptr_t)ws & 255) != 0) { set_error("spec_verify_forward: workspace must be 256-byte aligned"); return SPEC_EINVAL; }
    // page budget: every batch entry may need ceil((k+1)/P)+1 more pages than it holds at most
    int64_t grow = (int64_t)B * (cdiv(k + 1, SPEC_PAGE_SIZE) + 1);
    if (kv->ub.pages() + grow > kv->n_pages || kv->ub.max_ctx + k + 1 > (int64_t)kv->max_pages * SPEC_PAGE_SIZE) {
        if (kv->device_ahead) {                           // bounds may be stale: refresh them exactly once
            // ... which reads the device state back and synchronises: not under stream capture (it would end the recording)
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing((hipStream_t)stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
                set_error("spec_verify_forward: the host's bounds on the cache state no longer show that %d more positions fit, and the exact state cannot be read while the stream is being captured: call spec_kv_get_state before recording", k + 1);
                return SPEC_ESTATE;
            }
            spec_status st = kv_download(kv, nullptr);
            if (st != SPEC_OK) return st;
        }
        int64_t exact_grow = 0;                           // worst case over any B sequences: take the B largest needs
        std::vector<int64_t> needs;
        for (int s = 0; s < kv->max_seqs; ++s)
            needs.push_back(cdiv((int64_t)kv->h_ctx_len[s] + k + 1, SPEC_PAGE_SIZE) - kv->h_n_held[s]);
        std::sort(needs.begin(), needs.end(), [](int64_t a, int64_t b) { return a > b; });
        for (int i = 0; i < B; ++i) exact_grow += needs[i] > 0 ? needs[i] : 0;
        if (exact_grow > kv->h_free_count) { set_error("spec_verify_forward: the page pool cannot hold %d more positions for %d sequences", k + 1, B); return SPEC_ENOMEM; }
        if (kv->ub.max_ctx + k + 1 > (int64_t)kv->max_pages * SPEC_PAGE_SIZE) { set_error("spec_verify_forward: a sequence would outgrow max_ctx_len"); return SPEC_EINVAL; }
    }
    hipStream_t s = (hipStream_t)stream;
    prof_mark(PC_OTHER, s);
    spec_status st = launch_kv_reserve(kv, B, k, dev_seq_ids, s);
    if (st != SPEC_OK) return st;
    prof_mark(PC_KV_RESERVE, s);
    kv->device_ahead = true;
    st = m->desc.dtype == SPEC_F32 ? f32_forward(m, kv, B, k, dev_seq_ids, dev_tokens, dev_logits, ws, s)
                                   : bf16_forward(m, kv, B, k, dev_seq_ids, dev_tokens, io, dev_logits, ws, ws_bytes, s);
    return st;
}

extern "C" spec_status spec_verify_forward_hidden(spec_model* m, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                                  const int32_t* dev_tokens, const float* dev_hidden_in, float* dev_logits,
                                                  float* dev_hidden_out, void* ws, size_t ws_bytes, void* stream)
{
    Bf16Extras io;
    io.dev_hidden_in = dev_hidden_in;
    io.dev_hidden_out = dev_hidden_out;
    return verify_forward_any(m, kv, B, k, dev_seq_ids, dev_tokens, io, dev_logits, ws, ws_bytes, stream);
}

extern "C" spec_status spec_verify_forward_taps(spec_model* m, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                                const int32_t* dev_tokens, float* dev_logits, int32_t n_taps,
                                                const int32_t* host_tap_layers, float* dev_taps_out, void* ws, size_t ws_bytes,
                                                void* stream)
{
    if (!m || !host_tap_layers || !dev_taps_out) { set_error("spec_verify_forward_taps: null pointer"); return SPEC_EINVAL; }
    if (n_taps < 1 || n_taps > SPEC_MAX_TAPS) { set_error("spec_verify_forward_taps: n_taps must be 1 .. %d", SPEC_MAX_TAPS); return SPEC_EINVAL; }
    Bf16Extras io;
    io.n_taps = n_taps;
    for (int j = 0; j < n_taps; ++j) {
        if (host_tap_layers[j] < 1 || host_tap_layers[j] > m->desc.n_layers) {
            set_error("spec_verify_forward_taps: tap %d asks for the state after %d layers; the model has %d", j, host_tap_layers[j], m->desc.n_layers);
            return SPEC_EINVAL;
        }
        io.tap_layers[j] = host_tap_layers[j];
    }
    io.dev_taps_out = dev_taps_out;
    return verify_forward_any(m, kv, B, k, dev_seq_ids, dev_tokens, io, dev_logits, ws, ws_bytes, stream);
}

extern "C" spec_status spec_verify_forward_features(spec_model* m, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                                    const int32_t* dev_tokens, const float* dev_features_in, float* dev_logits,
                                                    float* dev_hidden_out, void* ws, size_t ws_bytes, void* stream)
{
    if (!m || !dev_features_in) { set_error("spec_verify_forward_features: null pointer"); return SPEC_EINVAL; }
    if (!m->desc.fuse_taps) { set_error("spec_verify_forward_features: the model was not created with fuse_taps"); return SPEC_EINVAL; }
    Bf16Extras io;
    io.dev_features_in = dev_features_in;
    io.dev_hidden_out = dev_hidden_out;
    return verify_forward_any(m, kv, B, k, dev_seq_ids, dev_tokens, io, dev_logits, ws, ws_bytes, stream);
}

extern "C" spec_status spec_verify_forward(spec_model* m, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                           const int32_t* dev_tokens, float* dev_logits, void* ws, size_t ws_bytes, void* stream)
{
    return spec_verify_forward_hidden(m, kv, B, k, dev_seq_ids, dev_tokens, nullptr, dev_logits, nullptr, ws, ws_bytes, stream);
}

extern "C" spec_status spec_commit_kv(spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids, const int32_t* dev_accept_len,
                                      int32_t* dev_new_ctx_len, int32_t* dev_commit_slots, void* stream)
{
    if (!kv || !dev_seq_ids || !dev_accept_len) { set_error("spec_commit_kv: null pointer"); return SPEC_EINVAL; }
    if (B < 1 || B > kv->max_seqs || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_commit_kv: B or k out of range"); return SPEC_EINVAL; }
    prof_mark(PC_OTHER, (hipStream_t)stream);
    spec_status st = launch_kv_commit(kv, B, k, dev_seq_ids, dev_accept_len, dev_new_ctx_len, dev_commit_slots, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_KV_COMMIT, (hipStream_t)stream);
    kv->device_ahead = true;
    kv->ub.max_ctx += k + 1;
    kv->ub.added_ctx += (int64_t)B * (k + 1);
    kv->ub.touched = std::min<int64_t>(kv->max_seqs, kv->ub.touched + B);
    return SPEC_OK;
}

extern "C" spec_status spec_kv_truncate(spec_kv* kv, int32_t B, const int32_t* dev_seq_ids, const int32_t* dev_len, int32_t delta,
                                        int32_t* dev_new_len, void* stream)
{
    if (!kv || !dev_seq_ids || !dev_len) { set_error("spec_kv_truncate: null pointer"); return SPEC_EINVAL; }
    if (B < 1 || B > kv->max_seqs) { set_error("spec_kv_truncate: B out of range"); return SPEC_EINVAL; }
    prof_mark(PC_OTHER, (hipStream_t)stream);
    spec_status st = launch_kv_truncate(kv, B, dev_seq_ids, dev_len, delta, dev_new_len, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_KV_TRUNCATE, (hipStream_t)stream);
    kv->device_ahead = true;            // lengths only shrink: the conservative bounds stay valid
    return SPEC_OK;
}

extern "C" spec_status spec_rollout_retire(int32_t B, int32_t k, int32_t n_seqs, int32_t* dev_slot_seq, int32_t* dev_active,
                                           const int32_t* dev_accept_len, int32_t* dev_gen_len, const int32_t* dev_target_len,
                                           const int32_t* dev_queue, int32_t queue_len, int32_t* dev_queue_head,
                                           const int32_t* dev_first_token, int32_t* dev_tokens, int32_t* dev_release_seq,
                                           int32_t* dev_keep_len, int64_t* dev_produced, void* stream)
{
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT || n_seqs < 1 || queue_len < 0) { set_error("spec_rollout_retire: size out of range"); return SPEC_EINVAL; }
    if (!dev_slot_seq || !dev_active || !dev_accept_len || !dev_gen_len || !dev_target_len || !dev_queue_head || !dev_first_token ||
        !dev_tokens || !dev_release_seq || !dev_keep_len || !dev_produced || (queue_len > 0 && !dev_queue)) {
        set_error("spec_rollout_retire: null pointer");
        return SPEC_EINVAL;
    }
    spec_status st = launch_rollout_retire(B, k, n_seqs, dev_slot_seq, dev_active, dev_accept_len, dev_gen_len, dev_target_len, dev_queue,
                                           queue_len, dev_queue_head, dev_first_token, dev_tokens, dev_release_seq, dev_keep_len,
                                           dev_produced, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_OTHER, (hipStream_t)stream);
    return SPEC_OK;
}

extern "C" spec_status spec_rollout_compact(int32_t B, int32_t k, int32_t* dev_slot_seq, int32_t* dev_active, int32_t* dev_tokens,
                                            int32_t* dev_n_live, int32_t* dev_scratch, void* stream)
{
    if (B < 1 || k < 0 || k > SPEC_MAX_DRAFT) { set_error("spec_rollout_compact: B or k out of range"); return SPEC_EINVAL; }
    if (!dev_slot_seq || !dev_active || !dev_tokens || !dev_n_live || !dev_scratch) { set_error("spec_rollout_compact: null pointer"); return SPEC_EINVAL; }
    spec_status st = launch_rollout_compact(B, k, dev_slot_seq, dev_active, dev_tokens, dev_n_live, dev_scratch, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_OTHER, (hipStream_t)stream);
    return SPEC_OK;
}

extern "C" spec_status spec_rollout_pending(int32_t B, int32_t n_seqs, const int32_t* dev_slot_seq_before, const int32_t* dev_slot_seq,
                                            const int32_t* dev_active, const int32_t* dev_prev_token, const int32_t* dev_first_token,
                                            int32_t* dev_pending, void* stream)
{
    if (B < 1 || n_seqs < 1) { set_error("spec_rollout_pending: B or n_seqs out of range"); return SPEC_EINVAL; }
    if (!dev_slot_seq_before || !dev_slot_seq || !dev_active || !dev_prev_token || !dev_first_token || !dev_pending) {
        set_error("spec_rollout_pending: null pointer");
        return SPEC_EINVAL;
    }
    spec_status st = launch_rollout_pending(B, n_seqs, dev_slot_seq_before, dev_slot_seq, dev_active, dev_prev_token, dev_first_token,
                                            dev_pending, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_OTHER, (hipStream_t)stream);
    return SPEC_OK;
}

extern "C" spec_status spec_rollout_pending_hidden(int32_t B, int32_t n_seqs, int32_t d, const int32_t* dev_slot_seq_before,
                                                   const int32_t* dev_slot_seq, const int32_t* dev_active, const float* dev_seq_hidden,
                                                   float* dev_pending_hidden, void* stream)
{
    if (B < 1 || n_seqs < 1 || d < 1) { set_error("spec_rollout_pending_hidden: B, n_seqs or d out of range"); return SPEC_EINVAL; }
    if (!dev_slot_seq_before || !dev_slot_seq || !dev_active || !dev_seq_hidden || !dev_pending_hidden) {
        set_error("spec_rollout_pending_hidden: null pointer");
        return SPEC_EINVAL;
    }
    spec_status st = launch_rollout_pending_hidden(B, n_seqs, d, dev_slot_seq_before, dev_slot_seq, dev_active, dev_seq_hidden,
                                                   dev_pending_hidden, (hipStream_t)stream);
    if (st != SPEC_OK) return st;
    prof_mark(PC_OTHER, (hipStream_t)stream);
    return SPEC_OK;
}

extern "C" size_t spec_kv_state_bytes(const spec_kv* kv) { return kv ? kv->state_ints * sizeof(int32_t) : 0; }

extern "C" spec_status spec_kv_snapshot(spec_kv* kv, void* dev_buf, void* stream)
{
    if (!kv || !dev_buf) { set_error("spec_kv_snapshot: null pointer"); return SPEC_EINVAL; }
    SPEC_HIP_TRY(hipMemcpyAsync(dev_buf, kv->d_state, kv->state_ints * sizeof(int32_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
    kv->snapshots[dev_buf] = kv->ub;
    return SPEC_OK;
}

extern "C" spec_status spec_kv_restore(spec_kv* kv, const void* dev_buf, void* stream)
{
    if (!kv || !dev_buf) { set_error("spec_kv_restore: null pointer"); return SPEC_EINVAL; }
    auto it = kv->snapshots.find(dev_buf);
    if (it == kv->snapshots.end()) { set_error("spec_kv_restore: this buffer holds no snapshot of this cache"); return SPEC_ESTATE; }
    SPEC_HIP_TRY(hipMemcpyAsync(kv->d_state, dev_buf, kv->state_ints * sizeof(int32_t), hipMemcpyDeviceToDevice, (hipStream_t)stream));
    kv->ub = it->second;
    kv->device_ahead = true;
    return SPEC_OK;
}

// ------------------------------------------------------------------------------------------ graphs

struct spec_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

extern "C" spec_status spec_graph_capture_begin(void* stream)
{
    if (!stream) { set_error("spec_graph_capture_begin: capture needs a stream of its own, not the default stream"); return SPEC_EINVAL; }
    if (g_prof_on) { set_error("spec_graph_capture_begin: switch event profiling off first"); return SPEC_ESTATE; }
    SPEC_HIP_TRY(hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal));
    return SPEC_OK;
}

extern "C" spec_status spec_graph_capture_end(void* stream, spec_graph** out)
{
    if (!stream || !out) { set_error("spec_graph_capture_end: null pointer"); return SPEC_EINVAL; }
    hipGraph_t g = nullptr;
    SPEC_HIP_TRY(hipStreamEndCapture((hipStream_t)stream, &g));
    spec_graph* sg = new (std::nothrow) spec_graph();
    if (!sg) { (void)hipGraphDestroy(g); set_error("spec_graph_capture_end: out of host memory"); return SPEC_ENOMEM; }
    sg->graph = g;
    hipError_t e = hipGraphInstantiate(&sg->exec, g, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        set_error("spec_graph_capture_end: hipGraphInstantiate failed: %s", hipGetErrorString(e));
        (void)hipGraphDestroy(g);
        delete sg;
        return SPEC_EHIP;
    }
    *out = sg;
    return SPEC_OK;
}

extern "C" spec_status spec_graph_launch(spec_graph* graph, void* stream)
{
    if (!graph || !graph->exec) { set_error("spec_graph_launch: null graph"); return SPEC_EINVAL; }
    SPEC_HIP_TRY(hipGraphLaunch(graph->exec, (hipStream_t)stream));
    return SPEC_OK;
}

extern "C" spec_status spec_graph_destroy(spec_graph* graph)
{
    if (!graph) return SPEC_OK;
    if (graph->exec) (void)hipGraphExecDestroy(graph->exec);
    if (graph->graph) (void)hipGraphDestroy(graph->graph);
    delete graph;
    return SPEC_OK;
}
