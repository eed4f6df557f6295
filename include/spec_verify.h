/*
 * spec_verify.h - C ABI of the MI355X (gfx950) speculative-decoding verify step.
 *
 * The operation (paper: Introduction, paragraph introducing speculative decoding; Section 2.1,
 * "lossless acceleration"; Section 2.2, acceptance length): a draft proposes k tokens per
 * sequence, the target model scores all k+1 positions of every sequence in ONE decode-phase
 * forward pass against its KV cache, a rejection procedure that preserves the target's output
 * distribution keeps the longest valid draft prefix and draws one more token, and the cache keeps
 * only what was accepted.  One "step" is
 *     spec_verify_forward -> spec_reject_sample -> spec_commit_kv
 * enqueued on one HIP stream; none of the three synchronises with the host or allocates.
 *
 * General rules
 *   - Every function returns SPEC_OK (0) or a negative spec_status; nothing throws, aborts or
 *     exits.  spec_last_error() gives a thread-local message for the last failure.
 *   - Pointers named dev_* are device memory owned by the caller (e.g. torch.empty on the GPU);
 *     they are only borrowed until the enqueued work has run.  Pointers named host_* are host memory.
 *   - Opaque handles (spec_model, spec_kv) are owned by the library; release them with the
 *     matching destroy/free.  Handles are bound to the device that was current at creation.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Arguments are validated on the host before anything is launched.
 */
#ifndef SPEC_VERIFY_H
#define SPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPEC_OK = 0,
    SPEC_EINVAL = -1,        /* bad argument (null pointer, size out of range, workspace too small) */
    SPEC_ENOMEM = -2,        /* page pool exhausted or device allocation failed */
    SPEC_EHIP = -3,          /* a HIP call failed; message holds hipGetErrorString */
    SPEC_ESTATE = -4,        /* call not valid in the handle's current state */
    SPEC_EUNSUPPORTED = -5   /* shape or type outside what the kernels cover */
} spec_status;

enum { SPEC_F32 = 0, SPEC_BF16 = 1, SPEC_FP8_E4M3 = 2 /* KV cache only */ };
enum { SPEC_MAX_DRAFT = 15 };          /* largest k */
enum { SPEC_PAGE_SIZE = 16 };          /* tokens per KV page */

const char* spec_last_error(void);

/* ---------------------------------------------------------------- model ------------------------------------ */

/* Plain data, copied by spec_model_create.  Pre-norm decoder: RMSNorm, grouped-query attention
 * with rotary embedding (pair j with j + head_dim/2, angle pos * rope_theta^(-2j/head_dim)), SwiGLU
 * feed-forward, dense or a routed mixture of experts (the 235B-A22B-class target of Section 3.1):
 * router probabilities softmax(h Wr^T) over all experts, the top_k most probable experts (ties to the
 * lower index), their probabilities renormalised to sum to one, output = weighted sum of those
 * experts' SwiGLU feed-forwards of width expert_ffn_dim.
 * fuse_hidden = 1 describes a draft model that takes the verifier's hidden states as a second input (the paper's
 * drafting paths, Section 2.3: EAGLE-3 and native multi-token-prediction heads both consume target hidden states;
 * the combination is the multi-token-prediction one): the first layer's input is
 *     w_fuse . [ RMSNorm(embedding of the token) * fuse_e_norm ; RMSNorm(hidden state) * fuse_h_norm ],
 * the hidden state being that of the position before the token (spec_verify_forward_hidden).
 * kv_dtype = SPEC_FP8_E4M3 (bf16 models only; 0 = the cache stores `dtype`): an 8-bit cache, the FP8 serving the
 * paper's projections assume (Section 4, simulator set-up).  Keys (after rotation) and values are stored as OCP
 * E4M3 codes (1-4-3 bits, bias 7, no infinities, largest magnitude 448) of x / scale, rounded to nearest even and
 * saturated, with one fp32 scale per (layer, kv head) for keys and one for values (spec_kv_set_scales); attention
 * reads code * scale.  As with the other storage types the k+1 new positions are encoded before any row attends
 * to them.
 * w_dtype = SPEC_FP8_E4M3 (bf16, untied head, no hidden-state input): the matrices wq .. wd and head are
 * E4M3 codes [out_features, in_features], one byte each, with one fp32 scale per output row (W[n][k] = code * scale[n];
 * stacked expert matrices: one scale per expert and output row, [E, Fe] for wg and wu, [E, d] for wd);
 * embed, the norm gains and the router stay `dtype`.  The kernels widen the codes to bf16 in registers (exact) and apply the
 * scale to the accumulated output, so the arithmetic is that of the bf16 path on the dequantised matrix. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
    float rope_theta, rms_eps;
    int32_t dtype;             /* SPEC_F32 or SPEC_BF16: storage type of weights and of the KV cache */
    int32_t tied_head;         /* 1: output head = embedding matrix */
    int32_t n_experts, top_k, expert_ffn_dim;   /* 0, 0, 0: dense feed-forward of width ffn_dim */
    int32_t fuse_hidden;       /* 1: a draft model whose input also takes hidden states (bf16, dense, ffn_dim >= 2 d_model) */
    int32_t kv_dtype;          /* 0: the cache stores `dtype`; SPEC_FP8_E4M3: 8-bit cache with scales (bf16 models) */
    int32_t w_dtype;           /* 0: the matrices are `dtype`; SPEC_FP8_E4M3: 8-bit matrices with one scale per output row */
    int32_t fuse_taps;         /* 0, or 1..SPEC_MAX_TAPS with fuse_hidden: the hidden-state input can also come as that many
                                  hidden states side by side (spec_verify_forward_features), projected by w_fc */
    int32_t head_vocab;        /* 0: the output head has `vocab` rows; else its number of rows (untied heads only): a draft
                                  model that proposes from a subset of the vocabulary (spec_draft_sample_mapped); the
                                  embedding still has `vocab` rows and the logits are [B, k+1, head_vocab] */
} spec_model_desc;

typedef struct spec_model spec_model;
typedef struct spec_kv spec_kv;
typedef struct spec_graph spec_graph;

/* Number of weight pointers spec_model_create expects:
 * 1 + (9 + (n_experts ? 1 : 0))*n_layers + 1 + (tied_head ? 0 : 1) + (fuse_hidden ? 3 : 0) + (fuse_taps ? 1 : 0)
 * + (w_dtype == SPEC_FP8_E4M3 ? 7*n_layers + 1 : 0). */
int32_t spec_model_weight_count(const spec_model_desc* desc);

/*
 * dev_weights[i], all in `dtype`, row-major [out_features, in_features], in this order:
 *   embed [vocab, d_model];
 *   per layer: attn_norm [d], wq [Hq*dh, d], wk [Hkv*dh, d], wv [Hkv*dh, d], wo [d, Hq*dh],
 *              ffn_norm [d], wg [ffn, d], wu [ffn, d], wd [d, ffn];
 *              with n_experts > 0 instead: wg [E, Fe, d], wu [E, Fe, d], wd [E, d, Fe] (the experts stacked,
 *              Fe = expert_ffn_dim), then router [E, d];
 *   final_norm [d]; head [vocab, d] ([head_vocab, d] if that is set) unless tied_head;
 *   with fuse_hidden: w_fuse [d, 2d] (columns 0..d-1 meet the embedding half), fuse_e_norm [d], fuse_h_norm [d];
 *   with fuse_taps = n: w_fc [d, n*d] (columns j*d .. (j+1)*d-1 meet the j-th hidden state);
 *   with w_dtype = SPEC_FP8_E4M3, after all of the above: the fp32 scales [out_features] of wq, wk, wv, wo, wg, wu, wd
 *   of layer 0, then of layer 1, ..., then of head (the matrices themselves then hold codes, 8-byte aligned).
 * SPEC_F32: the pointers are borrowed for the model's lifetime (kernels read them in place).
 * SPEC_BF16: the matrices are re-tiled once into a library-owned device buffer laid out for the
 * MFMA kernels (one hipMalloc of about the model's size); afterwards only embed and the norm
 * gains are still read from the caller's buffers.  BF16 needs head_dim == 128,
 * d_model % 256 == 0, ffn_dim % 256 == 0 (expert_ffn_dim % 256 == 0, n_experts <= 256,
 * 1 <= top_k <= min(n_experts, 16) for a mixture) and n_q_heads % n_kv_heads == 0, else
 * SPEC_EUNSUPPORTED; the fp32 path is dense only.
 * Synchronises the device.  (Paper: the target model of Section 2.1; its shape is the caller's.)
 */
spec_status spec_model_create(const spec_model_desc* desc, const void* const* dev_weights, int32_t n_weights,
                              spec_model** out);
spec_status spec_model_destroy(spec_model* model);

/* ---------------------------------------------------------------- KV cache --------------------------------- */

/*
 * Paged KV cache (the cache the decode-phase verification of Section 2.2 runs against; paging and
 * layout are this library's).  The pool is caller-owned device memory of spec_kv_pool_bytes():
 *   pool[layer_pool][page][K=0|V=1][kv_head] -> one block of SPEC_PAGE_SIZE * head_dim elements (of the cache's
 *   storage type: `dtype`, or one byte each with kv_dtype = SPEC_FP8_E4M3),
 * layer_pool = layer if layer_alias_mod == 0, else layer % layer_alias_mod (several layers share a
 * pool region: a way to run a cache larger than memory through the real access pattern; each
 * layer writes its new entries before it reads, cached context then is per region, not per layer).
 * Inside a block, element (token t of the page, channel c) sits at spec_kv_block_offset().
 * Page ids are 0 .. n_pages-1; slot = page * SPEC_PAGE_SIZE + t.
 *
 * Bookkeeping lives on the device (context length and page list per sequence, a stack of free
 * pages) so that a step needs no host round trip.  A fresh cache's stack pops 0, 1, 2, ...
 */
int64_t spec_kv_pool_bytes(const spec_model* model, int64_t n_pages, int32_t layer_alias_mod);
spec_status spec_kv_alloc(const spec_model* model, int32_t max_seqs, int32_t max_ctx_len, int64_t n_pages,
                          void* dev_pool, int32_t layer_alias_mod, spec_kv** out);
spec_status spec_kv_free(spec_kv* kv);

/*
 * 8-bit cache only: the scales, dev_k_scale and dev_v_scale [n_layers * n_kv_heads] fp32 in device memory (> 0),
 * borrowed until spec_kv_free.  Must be called before the first forward pass on this cache (SPEC_ESTATE otherwise);
 * SPEC_EINVAL for a cache that is not 8-bit.  The caller's page contents are codes under these scales.
 */
spec_status spec_kv_set_scales(spec_kv* kv, const float* dev_k_scale, const float* dev_v_scale);

/* Element offset (in elements) of (t, c) inside a K (is_v = 0) or V (is_v = 1) block; -1 on bad input. */
int64_t spec_kv_block_offset(const spec_kv* kv, int32_t is_v, int32_t t, int32_t c);
/* Element offset of the block of (layer, page, is_v, kv_head) from the start of the pool; -1 on bad input. */
int64_t spec_kv_block_base(const spec_kv* kv, int32_t layer, int64_t page, int32_t is_v, int32_t kv_head);

/*
 * Host call: install sequence `seq` (0 <= seq < max_seqs) with cached length ctx_len on the given
 * pages (exactly ceil(ctx_len / SPEC_PAGE_SIZE) distinct free page ids, possibly fragmented).  The
 * caller fills the pages' contents itself.  Synchronises the device if steps have run since the
 * last host call.  SPEC_EINVAL for pages in use or out of range.
 */
spec_status spec_kv_seq_assign(spec_kv* kv, int32_t seq, int32_t ctx_len, const int32_t* host_page_ids,
                               int32_t n_page_ids);

/*
 * Host call (synchronises): copy the bookkeeping out.  Any pointer may be NULL.
 *   host_ctx_len [max_seqs]; host_n_pages [max_seqs] pages held; host_page_table
 *   [max_seqs * spec_kv_max_pages_per_seq()] (-1 padded); host_free_stack [n_pages] bottom to top,
 *   *host_n_free entries valid.  Returns SPEC_ENOMEM if a step ran out of pages since the last
 *   call (the affected sequences were left untouched by that step), clearing the flag.
 */
spec_status spec_kv_get_state(spec_kv* kv, int32_t* host_ctx_len, int32_t* host_n_pages,
                              int32_t* host_page_table, int32_t* host_free_stack, int64_t* host_n_free);
int32_t spec_kv_max_pages_per_seq(const spec_kv* kv);

/*
 * Roll the bookkeeping back without a host round trip (re-running a step from the same state,
 * abandoning a speculative branch).  spec_kv_snapshot copies context lengths, page lists and
 * the free stack into dev_buf (spec_kv_state_bytes() bytes, caller-owned); spec_kv_restore
 * copies them back.  Page contents are not saved: positions beyond the restored lengths are
 * dead anyway.  Both are asynchronous on `stream`; a buffer that was never the target of
 * spec_kv_snapshot on this cache gives SPEC_ESTATE.
 */
size_t spec_kv_state_bytes(const spec_kv* kv);
spec_status spec_kv_snapshot(spec_kv* kv, void* dev_buf, void* stream);
spec_status spec_kv_restore(spec_kv* kv, const void* dev_buf, void* stream);

/* ---------------------------------------------------------------- the step ---------------------------------- */

/*
 * Verify forward (Section 2.1-2.2: the target scores all drafted positions in one decode pass).
 * Batch entry b is sequence dev_seq_ids[b] (distinct ids); its input row i (0..k) is token
 * dev_tokens[b*(k+1)+i] at position ctx_len+i: row 0 is the last emitted token (not cached yet),
 * rows 1..k are the drafts.  The call reserves pages for positions ctx..ctx+k, writes their K/V
 * there, and writes dev_logits[b][i][:] (fp32, [B, k+1, vocab]) = the target's logits for the token
 * following row i, which sees cache positions 0..ctx+i.  ctx_len is not changed (spec_commit_kv does).
 * dev_workspace: at least spec_verify_workspace_bytes(model, kv, B, k) bytes (0 = bad arguments), 256-byte
 * aligned; contents need not be preserved between calls.  Query the size again after spec_tune_set.
 * Errors: SPEC_EINVAL (null, B < 1, k < 0, k > SPEC_MAX_DRAFT, workspace too small, kv of another
 * model), SPEC_ENOMEM (the pool cannot hold k+1 more positions for every batch entry),
 * SPEC_EHIP.  Asynchronous on `stream`, with one exception: when the host's bounds on the cache state (kept
 * without reading the device) no longer show that the new positions fit, the call reads the exact state back once,
 * which synchronises; under stream capture it returns SPEC_ESTATE instead, with nothing launched (call
 * spec_kv_get_state before recording, so that the bounds are exact).
 *
 * spec_verify_forward_hidden is the same pass with the hidden states exposed (bf16 models): dev_hidden_out
 * [B, k+1, d_model] fp32 (may be NULL) receives the residual stream after the last layer, before the final norm -
 * what a hidden-state-consuming draft model is fed; dev_hidden_in [B, k+1, d_model] fp32 is required for a model
 * created with fuse_hidden (row i: the hidden state of the position before input row i) and must be NULL otherwise.
 */
size_t spec_verify_workspace_bytes(const spec_model* model, const spec_kv* kv, int32_t B, int32_t k);
spec_status spec_verify_forward(spec_model* model, spec_kv* kv, int32_t B, int32_t k,
                                const int32_t* dev_seq_ids, const int32_t* dev_tokens, float* dev_logits,
                                void* dev_workspace, size_t workspace_bytes, void* stream);
spec_status spec_verify_forward_hidden(spec_model* model, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                       const int32_t* dev_tokens, const float* dev_hidden_in, float* dev_logits,
                                       float* dev_hidden_out, void* dev_workspace, size_t workspace_bytes, void* stream);

/*
 * Multi-layer features (the EAGLE-3 drafting path of Section 2.3: the draft is fed the target's state at several
 * depths instead of the last one only).
 *
 * spec_verify_forward_taps: the verify forward of a bf16 model without hidden-state input that also writes
 * dev_taps_out [B, k+1, n_taps * d_model] fp32: columns j*d .. (j+1)*d-1 of row (b, i) = the residual stream after
 * host_tap_layers[j] layers (1 .. n_layers; n_layers is what spec_verify_forward_hidden returns; repeats allowed),
 * 1 <= n_taps <= SPEC_MAX_TAPS.  The array of layers is read during the call only.
 *
 * spec_verify_forward_features: the pass of a draft model created with fuse_taps = n whose hidden-state input comes
 * as features, dev_features_in [B, k+1, n * d_model] fp32 (row i: the target's taps of the position before input
 * row i, as spec_verify_forward_taps wrote them): the hidden state the fusion sees is w_fc . features (no norm before
 * it).  Everything else as spec_verify_forward_hidden, which the same model still takes for passes that chain its own
 * d_model-wide state.  spec_next_step_hidden and spec_rollout_pending_hidden carry features when given d = n * d_model.
 * Errors as spec_verify_forward; SPEC_EINVAL for a tap out of range or a model of the wrong kind.
 */
#define SPEC_MAX_TAPS 4
spec_status spec_verify_forward_taps(spec_model* model, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                     const int32_t* dev_tokens, float* dev_logits, int32_t n_taps,
                                     const int32_t* host_tap_layers, float* dev_taps_out, void* dev_workspace,
                                     size_t workspace_bytes, void* stream);
spec_status spec_verify_forward_features(spec_model* model, spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                                         const int32_t* dev_tokens, const float* dev_features_in, float* dev_logits,
                                         float* dev_hidden_out, void* dev_workspace, size_t workspace_bytes, void* stream);

/*
 * Lossless rejection sampling (the rejection procedure of Section 2.1; acceptance length as in
 * Section 2.2).  p_i = softmax(dev_logits[b][i][:] / temperature).  For i = 0..k-1 in order: draft
 * x = dev_draft_tokens[b][i] is kept iff u * q(x) < p_i(x) (u in [0,1), compared in fp64), where
 * q = dev_q[b][i][:] are the probabilities the draft was sampled from; stop at the first failure.
 * With n kept: if n < k the next token is drawn from norm(max(0, p_n - q_n)) (from p_n if that
 * residual is identically zero), else from p_k (bonus).  The draw is an exponential race,
 * argmax_v w_v / (-ln u_v), ties to the lowest v.  Every quantity a decision hangs on - logit / temperature,
 * the softmax, the accept test, the residual and the race keys - is computed in fp64.
 * Random numbers: Philox4x32-10, key = (seed low word, seed high word), counter =
 * (c0, i, b, step*4 + stream); accept: stream 0, c0 = 0, u = (word0 >> 8) * 2^-24;
 * vocabulary entry v: stream 1, c0 = v >> 2, word v & 3, u_v = ((word >> 9) + 0.5) * 2^-23.
 * Outputs: dev_accept_len[b] = n; dev_out_tokens[b][0..k] = the n kept drafts, the drawn token,
 * then -1.  dev_dbg [B, k, 3] fp32, may be NULL: P, Q, u of every accept test evaluated (NaN elsewhere).
 * Needs B >= 1, 0 <= k <= SPEC_MAX_DRAFT, V >= 1, temperature > 0, step < 2^30; draft tokens
 * outside [0, V) are treated as rejected.  dev_q and dev_draft_tokens may be NULL when k == 0.
 * dev_q == NULL with k > 0 means one-hot draft distributions (a deterministic drafter such as an n-gram
 * table, Section 3.1): q_i(x_i) = 1, so x_i is kept with probability p_i(x_i) and the residual is p_i with
 * entry x_i removed; no [B, k, V] array is read.
 * dev_workspace: at least spec_sample_workspace_bytes(B, k) bytes.  Asynchronous on `stream`.
 */
size_t spec_sample_workspace_bytes(int32_t B, int32_t k);
spec_status spec_reject_sample(int32_t B, int32_t k, int32_t V, const float* dev_logits, const float* dev_q,
                               const int32_t* dev_draft_tokens, float temperature, uint64_t seed, uint64_t step,
                               int32_t* dev_accept_len, int32_t* dev_out_tokens, float* dev_dbg,
                               void* dev_workspace, size_t workspace_bytes, void* stream);

/*
 * spec_reject_sample for callers that cannot allocate device memory or carry a workspace along: code recorded under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic, random
 * streams and outputs as spec_reject_sample, minus the workspace: the row statistics and per-range race results live
 * in a buffer that is part of the loaded library (1.5 MiB of device memory per GPU, held until the process ends).
 * The call allocates and frees nothing.  Limit: B * (k + 1) <= 4096 logits rows, SPEC_EINVAL beyond (use
 * spec_reject_sample then).
 * All calls on one GPU share that buffer: calls whose work may overlap on one GPU (different streams, or graphs
 * replayed concurrently) race on it; calls on one stream, or otherwise ordered, are safe, and nothing needs
 * clearing between them (every entry is written before it is read).  The buffer's address is looked
 * up on the first call on each GPU (that first call should not itself be under capture).  Asynchronous on `stream`.
 */
spec_status spec_reject_sample_static(int32_t B, int32_t k, int32_t V, const float* dev_logits, const float* dev_q,
                                      const int32_t* dev_draft_tokens, float temperature, uint64_t seed, uint64_t step,
                                      int32_t* dev_accept_len, int32_t* dev_out_tokens, float* dev_dbg, void* stream);

/*
 * KV commit (keeps the accepted prefix; the paper leaves the cache handling to the serving engine).
 * For batch entry b with n = dev_accept_len[b] (values outside 0..k are clamped): positions
 * ctx..ctx+n stay, the new context length is ctx+n+1 (the drawn token is the next step's row 0 and
 * has no entry yet); pages wholly beyond the new length return to the free stack, a sequence's
 * last page first, batch entries in order.  k must be the k of the preceding spec_verify_forward.
 * Outputs (either may be NULL): dev_new_ctx_len [B]; dev_commit_slots [B, k+1] = pool slot of each
 * kept position, -1 for dropped ones.  A batch entry the step left out - its sequence id out of range or named
 * twice, or (only possible when a recorded step is replayed over a cache state with fewer free pages than the host
 * had checked) no page left for its new positions - is not committed: its sequence stays as it was, and it gets
 * dev_new_ctx_len[b] = -1 and slots of -1; spec_kv_get_state then reports SPEC_EINVAL or SPEC_ENOMEM.
 * Asynchronous on `stream`.
 */
spec_status spec_commit_kv(spec_kv* kv, int32_t B, int32_t k, const int32_t* dev_seq_ids,
                           const int32_t* dev_accept_len, int32_t* dev_new_ctx_len, int32_t* dev_commit_slots,
                           void* stream);

/* ---------------------------------------------------------------- draft side ---------------------------------- */

/*
 * The draft model's proposal for one draft position (Section 2.1: the draft proposes several tokens, which
 * the target then verifies; Section 3.1 uses a learned single-layer draft).  A draft model is an ordinary
 * spec_model with a cache of its own, run with spec_verify_forward one position at a time; this call turns
 * its logits into q = softmax(logits / temperature) and one token x ~ q:
 *   dev_logits: row b at dev_logits + b * logits_row_stride (fp32, V entries);
 *   dev_q:      row b written at dev_q + b * q_row_stride (so that the rows of all k positions can be laid out
 *               as the [B, k, V] array spec_reject_sample takes);
 *   x is written to dev_tokens_a[b * stride_a] and dev_tokens_b[b * stride_b] (either pointer may be NULL):
 *               typically the verify step's token array [B, k+1] and the draft's next input [B].
 * Draw: exponential race argmax_v q_v / (-ln u_v), ties to the lowest v, Philox4x32-10 with the key and
 * counter layout of spec_reject_sample on stream 2: counter = (v >> 2, row, b, step*4 + 2), word v & 3,
 * u_v = ((word >> 9) + 0.5) * 2^-23; `row` is the index of the draft position (0 .. SPEC_MAX_DRAFT).
 * dev_workspace: at least spec_draft_sample_workspace_bytes(B) bytes of device memory (contents irrelevant).
 * Errors: SPEC_EINVAL (sizes, strides below V, temperature <= 0, step >= 2^30, null, workspace too small).
 * Asynchronous on `stream`.
 */
size_t spec_draft_sample_workspace_bytes(int32_t B);
spec_status spec_draft_sample(int32_t B, int32_t V, const float* dev_logits, int64_t logits_row_stride,
                              float temperature, uint64_t seed, uint64_t step, int32_t row,
                              int32_t* dev_tokens_a, int32_t stride_a, int32_t* dev_tokens_b, int32_t stride_b,
                              float* dev_q, int64_t q_row_stride, void* dev_workspace, size_t workspace_bytes, void* stream);

/*
 * The same for a draft model whose head covers a subset of the target's vocabulary (the reduced draft vocabulary of the
 * EAGLE-3 design, Section 2.3: a head of the V_d most useful tokens is a quarter of the bytes and of the sampling work
 * of a 128k one).  dev_logits rows have V_d entries; dev_token_map [V_d] holds their ids in the target's vocabulary,
 * strictly increasing, all below V_full.  q = softmax over the V_d entries, written into rows of V_full entries
 * (q_row_stride >= V_full) at the mapped positions with zeros everywhere else - the [B, k, V_full] array
 * spec_reject_sample takes, which then resamples tokens outside the subset from the target's own probabilities; the
 * tokens written are target ids.  Draw and random numbers as spec_draft_sample, v counting draft entries.
 * Errors as spec_draft_sample.  The map's contents live on the device and are not validated by the call: an entry
 * outside [0, V_full) is skipped by the kernel (its probability is written nowhere, so the row of q then sums to
 * less than 1, and it is never drawn); repeated ids are not detected.
 */
spec_status spec_draft_sample_mapped(int32_t B, int32_t V_d, const float* dev_logits, int64_t logits_row_stride,
                                     float temperature, uint64_t seed, uint64_t step, int32_t row,
                                     int32_t* dev_tokens_a, int32_t stride_a, int32_t* dev_tokens_b, int32_t stride_b,
                                     float* dev_q, int64_t q_row_stride, const int32_t* dev_token_map, int32_t V_full,
                                     void* dev_workspace, size_t workspace_bytes, void* stream);

/*
 * Roll a cache back (the draft's cache after verification keeps only what the verifier kept): batch entry b
 * ends with min(current length, dev_len[b] + delta) cached positions; a negative target is clamped to 0 and
 * flagged like other bookkeeping errors (reported by the next spec_kv_get_state).  Pages wholly beyond the new
 * length return to the free stack, a sequence's last page first, batch entries in order.  dev_new_len [B]
 * (may be NULL) receives the lengths in force.  With dev_len = the target's dev_new_ctx_len and delta = -1
 * the draft is left one position behind the target, which the next step's first draft pass feeds together
 * with the newly emitted token.  Asynchronous on `stream`.
 */
spec_status spec_kv_truncate(spec_kv* kv, int32_t B, const int32_t* dev_seq_ids, const int32_t* dev_len, int32_t delta,
                             int32_t* dev_new_len, void* stream);

/*
 * Inputs of the next speculation step, on the device (so that consecutive steps of a rollout need no host round
 * trip): with n = dev_accept_len[b] of the step just sampled, dev_pending[b] = (dev_tokens[b][n], dev_out_tokens[b][n])
 * = the last input the target kept and the token it emitted - what a draft model that is one position behind
 * feeds first (dev_pending [B, 2], may be NULL) - and dev_tokens[b][0] = dev_out_tokens[b][n], the next step's
 * first input.  dev_tokens and dev_out_tokens are the [B, k+1] arrays of spec_verify_forward / spec_reject_sample.
 * Asynchronous on `stream`.
 */
spec_status spec_next_step_inputs(int32_t B, int32_t k, int32_t* dev_tokens, const int32_t* dev_out_tokens,
                                  const int32_t* dev_accept_len, int32_t* dev_pending, void* stream);

/* ---------------------------------------------------------------- tuning / introspection -------------------- */

/* Set a launch parameter by name (split factors and the like); unknown names give SPEC_EINVAL.
 * Results never depend on these beyond floating-point summation order. */
spec_status spec_tune_set(const char* name, int32_t value);
int32_t spec_tune_get(const char* name);

/*
 * Per-kernel-class timing with HIP events on the stream the kernels run on (for benchmarks; adds
 * one event per launch group while on).  spec_profile_begin creates up to max_events events once
 * and switches recording on; the step calls then bracket each class of launches; spec_profile_end
 * synchronises the device, switches recording off and fills host_ms[c] / host_counts[c]
 * (c < spec_profile_class_count(), n = array length) with the summed milliseconds and the number
 * of timed segments of class c.  Not thread-safe; meant for one stream at a time.
 */
int32_t spec_profile_class_count(void);
const char* spec_profile_class_name(int32_t c);
spec_status spec_profile_begin(int32_t max_events);
spec_status spec_profile_end(double* host_ms, int64_t* host_counts, int32_t n);

/*
 * Hidden states for the next step's two pending tokens of a hidden-state-consuming draft model (see
 * spec_next_step_inputs: the last input the verifier kept, and the token it emitted): the verifier's hidden states
 * of the positions before them.  With n = dev_accept_len[b] clamped to [0, k] and H = dev_target_hidden
 * [B, k+1, d] (spec_verify_forward_hidden of the step just sampled), dev_pending_hidden [B, 2, d] becomes
 *   row 0 = H[b][n-1] if n >= 1, else its own old row 1 (the state that was paired with the old emitted token),
 *   row 1 = H[b][n].
 * fp32, plain copies.  Asynchronous on `stream`.
 */
spec_status spec_next_step_hidden(int32_t B, int32_t k, int32_t d, const float* dev_target_hidden,
                                  const int32_t* dev_accept_len, float* dev_pending_hidden, void* stream);

/*
 * Model-free n-gram drafting (the paper's n-gram baseline: Section 3.1 set-up, Section 3.2 and Table 2; the paper
 * gives no algorithm - this is prompt-lookup drafting): the drafts of a step are copied from the sequence's own
 * token history, from behind the most recent earlier occurrence of its current ending.
 *
 * dev_hist [n_rows, hist_stride] int32 (device) holds one history per row, dev_hist_len [n_rows] its length L; the
 * last token h[L-1] is the one the verifier emitted last.  Batch entry b uses row dev_seq_ids[b] (row b if
 * dev_seq_ids is NULL).  For n = n_max down to n_min (1 <= n_min <= n_max <= 16) the ending h[L-n..L-1] is searched
 * at start positions j with j + n <= L - 1 (a token follows the occurrence; it may overlap the ending); the longest
 * n with an occurrence wins, among its occurrences the largest j.  Output, for the [B, k+1] token array of
 * spec_verify_forward: dev_tokens[b][0] = h[L-1]; dev_tokens[b][1..c] = h[j+n .. j+n+c-1] with
 * c = min(k, L - (j+n)); the slots c+1..k repeat the last drafted token; dev_n_drafted[b] = c (may be NULL).
 * Without an occurrence c = 0 and every slot holds h[L-1].  A row index outside [0, n_rows) or an empty history
 * gives c = -1 and zeros.  Such drafts are point masses: verify them with spec_reject_sample(dev_q = NULL).
 * Integer work, bit-exact.  Asynchronous on `stream`; nothing is allocated.
 */
spec_status spec_ngram_draft(int32_t B, int32_t k, int32_t n_max, int32_t n_min, const int32_t* dev_hist,
                             int64_t hist_stride, int32_t n_rows, const int32_t* dev_hist_len, const int32_t* dev_seq_ids,
                             int32_t* dev_tokens, int32_t* dev_n_drafted, void* stream);

/*
 * After a verify step the accepted drafts and the emitted token join the history: row r of batch entry b gets
 * dev_out_tokens[b][0..n], n = dev_accept_len[b] clamped to [0, k], appended at dev_hist_len[r], which advances.
 * A history that reaches hist_stride tokens keeps what fits (its length saturates).  Rows outside [0, n_rows) are
 * skipped.  Two batch entries must not name the same row.  Asynchronous on `stream`.
 */
spec_status spec_ngram_append(int32_t B, int32_t k, int32_t* dev_hist, int64_t hist_stride, int32_t n_rows,
                              int32_t* dev_hist_len, const int32_t* dev_seq_ids, const int32_t* dev_out_tokens,
                              const int32_t* dev_accept_len, void* stream);

/*
 * Slot bookkeeping of a continuous rollout, on the device (the paper's rollouts have long-tailed response lengths,
 * Section 2.2 / Section 4: batch slots drain unevenly while the decode phase keeps running; the paper describes no
 * mechanism - this is continuous batching over already prefilled sequences).  Call after spec_commit_kv and
 * spec_next_step_inputs of a step.  For batch slot b, in batch order:
 *   live slot (dev_active[b] != 0), sequence s = dev_slot_seq[b], n = dev_accept_len[b] clamped to [0, k]:
 *     made = min(n + 1, dev_target_len[s] - dev_gen_len[s]) response tokens count (those behind the end of the
 *     response are dropped); dev_gen_len[s] += made.  If the response is complete the sequence is retired
 *     (dev_keep_len[b] = 0): the next waiting sequence dev_queue[*dev_queue_head] takes the slot
 *     (dev_slot_seq[b], *dev_queue_head advance; dev_tokens[b][0] = dev_first_token[new sequence]), or, with the
 *     queue (queue_len entries) exhausted, the slot goes idle (dev_active[b] = 0, the sequence id stays).
 *     Otherwise dev_keep_len[b] = 2^30 (keep everything).
 *   idle slot: counts nothing; dev_keep_len[b] = 0 (whatever later steps cached for it is dropped again).
 * dev_release_seq[b] receives the sequence the slot held on entry: hand (dev_release_seq, dev_keep_len, delta 0) to
 * spec_kv_truncate of every cache involved to release the retired sequences' pages.  *dev_produced (int64, device)
 * is increased by the tokens counted.  Waiting sequences must already hold their prompt's cache
 * (spec_kv_seq_assign) - prefill is outside this library.  Sequence ids index dev_gen_len, dev_target_len and
 * dev_first_token (n_seqs entries each); a slot whose sequence id is out of range is treated as idle.
 * dev_tokens is the [B, k+1] input array of the next spec_verify_forward.  Asynchronous on `stream`.
 */
spec_status spec_rollout_retire(int32_t B, int32_t k, int32_t n_seqs, int32_t* dev_slot_seq, int32_t* dev_active,
                                const int32_t* dev_accept_len, int32_t* dev_gen_len, const int32_t* dev_target_len,
                                const int32_t* dev_queue, int32_t queue_len, int32_t* dev_queue_head,
                                const int32_t* dev_first_token, int32_t* dev_tokens, int32_t* dev_release_seq,
                                int32_t* dev_keep_len, int64_t* dev_produced, void* stream);

/*
 * Compaction of the batch slots of a continuous rollout: the live slots (dev_active[b] != 0) move to the front in
 * their order, the idle ones follow in theirs; dev_slot_seq [B], dev_active [B] and the rows of dev_tokens
 * [B, k+1] travel together.  *dev_n_live (device) receives the number of live slots: a step over the first
 * n_live slots then covers every live sequence, and costs what a batch of that size costs - the answer to the
 * under-used tail of a long-tailed rollout (Section 4 of the paper discusses it; the mechanism is this library's).
 * The caller reads n_live back when it chooses to resize the batch.  dev_scratch: B * (k + 3) int32 of device
 * memory, contents irrelevant.  Asynchronous on `stream`.
 */
spec_status spec_rollout_compact(int32_t B, int32_t k, int32_t* dev_slot_seq, int32_t* dev_active, int32_t* dev_tokens,
                                 int32_t* dev_n_live, int32_t* dev_scratch, void* stream);

/*
 * Continuous rollout with a draft model (the paper's drafting paths, Section 2.3, run inside the rollout loop of
 * Section 2.2): besides the verifier's inputs every slot carries the pair of tokens its draft model has not cached yet,
 * dev_pending [B, 2] = (last input the verifier has cached, last emitted token) (spec_next_step_inputs).  For every
 * live slot whose sequence changed in spec_rollout_retire - dev_slot_seq_before [B] is a copy of dev_slot_seq taken
 * before that call - the pair becomes the new sequence's own: (dev_prev_token[s], dev_first_token[s]), the last token
 * of its prompt (cached by the verifier, not by the draft model, whose cache is one position behind) and its first
 * input token.  Other slots are left alone.  Sequence ids index dev_prev_token and dev_first_token (n_seqs entries
 * each).  Asynchronous on `stream`.
 */
spec_status spec_rollout_pending(int32_t B, int32_t n_seqs, const int32_t* dev_slot_seq_before, const int32_t* dev_slot_seq,
                                 const int32_t* dev_active, const int32_t* dev_prev_token, const int32_t* dev_first_token,
                                 int32_t* dev_pending, void* stream);

/*
 * The same for a draft model that takes the verifier's hidden states (Section 2.3; spec_verify_forward_hidden,
 * spec_next_step_hidden): every slot also carries the hidden states of the positions before its two pending tokens,
 * dev_pending_hidden [B, 2, d] fp32.  A waiting sequence brings its own, dev_seq_hidden [n_seqs, 2, d] fp32, left by
 * whatever prefilled it (the verifier's hidden state of the position before its last prompt token, and of that token's
 * own position); the live slots whose sequence changed in spec_rollout_retire get them, the others are left alone.
 * Call it with the same dev_slot_seq_before as spec_rollout_pending.  Plain copies.  Asynchronous on `stream`.
 */
spec_status spec_rollout_pending_hidden(int32_t B, int32_t n_seqs, int32_t d, const int32_t* dev_slot_seq_before,
                                        const int32_t* dev_slot_seq, const int32_t* dev_active, const float* dev_seq_hidden,
                                        float* dev_pending_hidden, void* stream);

/*
 * Replay of a recorded sequence of step calls (for callers whose steps are short enough that launching ~350 small
 * kernels per step costs more than running them).  Between spec_graph_capture_begin and spec_graph_capture_end every
 * call of this library on `stream` (which must not be the default stream) is recorded instead of executed; the
 * result replays with spec_graph_launch.  The step calls allocate nothing and use no memset, so they record cleanly;
 * what is baked in: all pointer and scalar arguments (the random-counter `step` included - record several steps with
 * their own `step` values into one graph), the split factors in force, and the number of attention chunks launched,
 * which follows the longest context the cache's host-side bound knew at recording time: replay only from a cache
 * state whose contexts are no longer than that (e.g. after spec_kv_restore of the state it was recorded from; the
 * restore itself may be part of the recording).  Event profiling must be off while recording.  The host-side
 * bounds of the caches are advanced while recording as if the calls had run once.
 */
spec_status spec_graph_capture_begin(void* stream);
spec_status spec_graph_capture_end(void* stream, spec_graph** out);
spec_status spec_graph_launch(spec_graph* graph, void* stream);
spec_status spec_graph_destroy(spec_graph* graph);

/*
 * Calibration kernels of known size (for benchmarks: the measured HBM ceiling, and the reference
 * that hardware traffic counters are scaled by).  spec_calib_read streams `bytes` (multiple of 16,
 * 16-byte aligned) from dev_src and discards them (dev_sink4: 4 writable bytes);
 * spec_calib_copy copies dev_src to dev_dst.  `workgroups` of 256 lanes walk the buffer with a grid
 * stride.  Asynchronous on `stream`.
 */
spec_status spec_calib_read(const void* dev_src, size_t bytes, void* dev_sink4, int32_t workgroups, void* stream);
spec_status spec_calib_copy(void* dev_dst, const void* dev_src, size_t bytes, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_VERIFY_H */
