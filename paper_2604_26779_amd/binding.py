"""ctypes binding of libspecverify.so: same names as the C ABI (include/spec_verify.h), argument
marshalling only.  Device buffers are torch tensors (their ``data_ptr()`` is what crosses the
boundary); no step of the verify path runs in Python or in torch.

The library must have been built (``python -m paper_2604_26779_amd.build`` or
``__graft_entry__.build()``); loading fails loudly otherwise, there is no fallback.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecverify.so")

SPEC_OK, SPEC_EINVAL, SPEC_ENOMEM, SPEC_EHIP, SPEC_ESTATE, SPEC_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
SPEC_F32, SPEC_BF16, SPEC_FP8_E4M3 = 0, 1, 2
SPEC_MAX_DRAFT = 15
SPEC_PAGE_SIZE = 16

EXPORTS = [
    "spec_last_error", "spec_model_weight_count", "spec_model_create", "spec_model_destroy", "spec_kv_pool_bytes",
    "spec_kv_alloc", "spec_kv_free", "spec_kv_set_scales", "spec_kv_block_offset", "spec_kv_block_base", "spec_kv_seq_assign",
    "spec_kv_get_state", "spec_kv_max_pages_per_seq", "spec_kv_state_bytes", "spec_kv_snapshot", "spec_kv_restore",
    "spec_verify_workspace_bytes", "spec_verify_forward", "spec_verify_forward_hidden", "spec_verify_forward_taps", "spec_verify_forward_features", "spec_next_step_hidden", "spec_sample_workspace_bytes", "spec_reject_sample", "spec_reject_sample_static",
    "spec_commit_kv", "spec_draft_sample", "spec_draft_sample_mapped", "spec_draft_sample_workspace_bytes", "spec_kv_truncate", "spec_next_step_inputs", "spec_ngram_draft", "spec_ngram_append", "spec_rollout_retire", "spec_rollout_compact", "spec_rollout_pending", "spec_rollout_pending_hidden", "spec_tune_set", "spec_tune_get", "spec_profile_class_count", "spec_profile_class_name",
    "spec_profile_begin", "spec_profile_end", "spec_graph_capture_begin", "spec_graph_capture_end", "spec_graph_launch",
    "spec_graph_destroy", "spec_calib_read", "spec_calib_copy",
]


class SpecError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("spec_status %d: %s" % (status, message))
        self.status = status


class spec_model_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                              "ffn_dim", "vocab")] + \
               [("rope_theta", ctypes.c_float), ("rms_eps", ctypes.c_float), ("dtype", ctypes.c_int32),
                ("tied_head", ctypes.c_int32), ("n_experts", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("expert_ffn_dim", ctypes.c_int32), ("fuse_hidden", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("w_dtype", ctypes.c_int32),
                ("fuse_taps", ctypes.c_int32), ("head_vocab", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libspecverify.so is not built: run `python -m paper_2604_26779_amd.build` "
                              "(there is no CPU or PyTorch fallback for the verify step)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, sz, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64,
                                      ctypes.c_size_t, ctypes.c_float)
        sig = {
            "spec_last_error": (ctypes.c_char_p, []),
            "spec_model_weight_count": (i32, [vp]),
            "spec_model_create": (i32, [vp, vp, i32, vp]),
            "spec_model_destroy": (i32, [vp]),
            "spec_kv_pool_bytes": (i64, [vp, i64, i32]),
            "spec_kv_alloc": (i32, [vp, i32, i32, i64, vp, i32, vp]),
            "spec_kv_free": (i32, [vp]),
            "spec_kv_set_scales": (i32, [vp, vp, vp]),
            "spec_kv_block_offset": (i64, [vp, i32, i32, i32]),
            "spec_kv_block_base": (i64, [vp, i32, i64, i32, i32]),
            "spec_kv_seq_assign": (i32, [vp, i32, i32, vp, i32]),
            "spec_kv_get_state": (i32, [vp, vp, vp, vp, vp, vp]),
            "spec_kv_max_pages_per_seq": (i32, [vp]),
            "spec_kv_state_bytes": (sz, [vp]),
            "spec_kv_snapshot": (i32, [vp, vp, vp]),
            "spec_kv_restore": (i32, [vp, vp, vp]),
            "spec_verify_workspace_bytes": (sz, [vp, vp, i32, i32]),
            "spec_verify_forward": (i32, [vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]),
            "spec_verify_forward_hidden": (i32, [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]),
            "spec_verify_forward_taps": (i32, [vp, vp, i32, i32, vp, vp, vp, i32, vp, vp, vp, sz, vp]),
            "spec_verify_forward_features": (i32, [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]),
            "spec_next_step_hidden": (i32, [i32, i32, i32, vp, vp, vp, vp]),
            "spec_sample_workspace_bytes": (sz, [i32, i32]),
            "spec_reject_sample": (i32, [i32, i32, i32, vp, vp, vp, f32, u64, u64, vp, vp, vp, vp, sz, vp]),
            "spec_reject_sample_static": (i32, [i32, i32, i32, vp, vp, vp, f32, u64, u64, vp, vp, vp, vp]),
            "spec_commit_kv": (i32, [vp, i32, i32, vp, vp, vp, vp, vp]),
            "spec_draft_sample": (i32, [i32, i32, vp, i64, f32, u64, u64, i32, vp, i32, vp, i32, vp, i64, vp, sz, vp]),
            "spec_draft_sample_mapped": (i32, [i32, i32, vp, i64, f32, u64, u64, i32, vp, i32, vp, i32, vp, i64, vp, i32, vp, sz, vp]),
            "spec_draft_sample_workspace_bytes": (sz, [i32]),
            "spec_kv_truncate": (i32, [vp, i32, vp, vp, i32, vp, vp]),
            "spec_next_step_inputs": (i32, [i32, i32, vp, vp, vp, vp, vp]),
            "spec_ngram_draft": (i32, [i32, i32, i32, i32, vp, i64, i32, vp, vp, vp, vp, vp]),
            "spec_ngram_append": (i32, [i32, i32, vp, i64, i32, vp, vp, vp, vp, vp]),
            "spec_rollout_retire": (i32, [i32, i32, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]),
            "spec_rollout_compact": (i32, [i32, i32, vp, vp, vp, vp, vp, vp]),
            "spec_rollout_pending": (i32, [i32, i32, vp, vp, vp, vp, vp, vp, vp]),
            "spec_rollout_pending_hidden": (i32, [i32, i32, i32, vp, vp, vp, vp, vp, vp]),
            "spec_tune_set": (i32, [ctypes.c_char_p, i32]),
            "spec_tune_get": (i32, [ctypes.c_char_p]),
            "spec_profile_class_count": (i32, []),
            "spec_profile_class_name": (ctypes.c_char_p, [i32]),
            "spec_profile_begin": (i32, [i32]),
            "spec_profile_end": (i32, [vp, vp, i32]),
            "spec_graph_capture_begin": (i32, [vp]),
            "spec_graph_capture_end": (i32, [vp, vp]),
            "spec_graph_launch": (i32, [vp, vp]),
            "spec_graph_destroy": (i32, [vp]),
            "spec_calib_read": (i32, [vp, sz, vp, i32, vp]),
            "spec_calib_copy": (i32, [vp, vp, sz, i32, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def spec_last_error():
    return lib().spec_last_error().decode()


def _check(status):
    if status != SPEC_OK:
        raise SpecError(status, spec_last_error())


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    return int(t)


def _addr(t):
    """Address of a tensor's first element (views into larger arrays allowed), or a raw address."""
    if t is None:
        return None
    return t.data_ptr() if isinstance(t, torch.Tensor) else int(t)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def make_desc(cfg):
    d = spec_model_desc()
    for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab"):
        setattr(d, n, int(cfg[n]))
    d.rope_theta, d.rms_eps = float(cfg["rope_theta"]), float(cfg["rms_eps"])
    d.dtype = {"f32": SPEC_F32, "bf16": SPEC_BF16}[cfg["dtype"]]
    d.tied_head = int(cfg.get("tied_head", 0))
    d.n_experts, d.top_k, d.expert_ffn_dim = (int(cfg.get(n, 0)) for n in ("n_experts", "top_k", "expert_ffn_dim"))
    d.fuse_hidden = int(cfg.get("fuse_hidden", 0))
    d.fuse_taps = int(cfg.get("fuse_taps", 0))
    d.head_vocab = int(cfg.get("head_vocab", 0))
    d.kv_dtype = {None: 0, "fp8_e4m3": SPEC_FP8_E4M3}[cfg.get("kv_dtype")]
    d.w_dtype = {None: 0, "fp8_e4m3": SPEC_FP8_E4M3}[cfg.get("w_dtype")]
    return d


def spec_model_weight_count(cfg):
    d = make_desc(cfg)
    return lib().spec_model_weight_count(ctypes.byref(d))


def spec_model_create(cfg, weights):
    """weights: device tensors in the header's canonical order.  Returns an opaque handle."""
    d = make_desc(cfg)
    arr = (ctypes.c_void_p * len(weights))(*[_ptr(w) for w in weights])
    out = ctypes.c_void_p()
    _check(lib().spec_model_create(ctypes.byref(d), arr, len(weights), ctypes.byref(out)))
    return out


def spec_model_destroy(model):
    _check(lib().spec_model_destroy(model))


def spec_kv_pool_bytes(model, n_pages, layer_alias_mod=0):
    return lib().spec_kv_pool_bytes(model, n_pages, layer_alias_mod)


def spec_kv_alloc(model, max_seqs, max_ctx_len, n_pages, pool, layer_alias_mod=0):
    out = ctypes.c_void_p()
    _check(lib().spec_kv_alloc(model, max_seqs, max_ctx_len, n_pages, _ptr(pool), layer_alias_mod, ctypes.byref(out)))
    return out


def spec_kv_set_scales(kv, k_scale, v_scale):
    """k_scale, v_scale: fp32 device tensors [n_layers * n_kv_heads]; the caller keeps them alive."""
    _check(lib().spec_kv_set_scales(kv, _ptr(k_scale), _ptr(v_scale)))


def spec_kv_free(kv):
    _check(lib().spec_kv_free(kv))


def spec_kv_block_offset(kv, is_v, t, c):
    return lib().spec_kv_block_offset(kv, is_v, t, c)


def spec_kv_block_base(kv, layer, page, is_v, kv_head):
    return lib().spec_kv_block_base(kv, layer, page, is_v, kv_head)


def spec_kv_seq_assign(kv, seq, ctx_len, page_ids):
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    _check(lib().spec_kv_seq_assign(kv, seq, ctx_len, ids.ctypes.data, len(ids)))


def spec_kv_max_pages_per_seq(kv):
    return lib().spec_kv_max_pages_per_seq(kv)


def spec_kv_get_state(kv, max_seqs, n_pages):
    """Returns dict(ctx_len, n_pages, page_table [max_seqs, max_pages], free_stack (valid part))."""
    mp = spec_kv_max_pages_per_seq(kv)
    ctx = np.zeros(max_seqs, dtype=np.int32)
    held = np.zeros(max_seqs, dtype=np.int32)
    table = np.zeros((max_seqs, mp), dtype=np.int32)
    stack = np.zeros(n_pages, dtype=np.int32)
    nfree = ctypes.c_int64()
    _check(lib().spec_kv_get_state(kv, ctx.ctypes.data, held.ctypes.data, table.ctypes.data, stack.ctypes.data,
                                   ctypes.byref(nfree)))
    return dict(ctx_len=ctx, n_pages=held, page_table=table, free_stack=stack[:nfree.value].copy())


def spec_kv_state_bytes(kv):
    return lib().spec_kv_state_bytes(kv)


def spec_kv_snapshot(kv, buf, stream=None):
    _check(lib().spec_kv_snapshot(kv, _ptr(buf), _stream(stream)))


def spec_kv_restore(kv, buf, stream=None):
    _check(lib().spec_kv_restore(kv, _ptr(buf), _stream(stream)))


def spec_verify_workspace_bytes(model, kv, B, k):
    return lib().spec_verify_workspace_bytes(model, kv, B, k)


def spec_verify_forward(model, kv, B, k, seq_ids, tokens, logits, workspace, stream=None):
    _check(lib().spec_verify_forward(model, kv, B, k, _ptr(seq_ids), _ptr(tokens), _ptr(logits), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))


def spec_verify_forward_hidden(model, kv, B, k, seq_ids, tokens, hidden_in, logits, hidden_out, workspace, stream=None):
    """hidden_in / hidden_out: [B, k+1, d] fp32 device tensors or None."""
    _check(lib().spec_verify_forward_hidden(model, kv, B, k, _ptr(seq_ids), _ptr(tokens), _ptr(hidden_in), _ptr(logits),
                                            _ptr(hidden_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream)))


def spec_verify_forward_taps(model, kv, B, k, seq_ids, tokens, logits, tap_layers, taps_out, workspace, stream=None):
    """tap_layers: host sequence of layer counts; taps_out [B, k+1, len(tap_layers) * d] fp32 device tensor."""
    layers = (ctypes.c_int32 * len(tap_layers))(*[int(l) for l in tap_layers])
    _check(lib().spec_verify_forward_taps(model, kv, B, k, _ptr(seq_ids), _ptr(tokens), _ptr(logits), len(tap_layers),
                                          ctypes.cast(layers, ctypes.c_void_p), _ptr(taps_out), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)))


def spec_verify_forward_features(model, kv, B, k, seq_ids, tokens, features_in, logits, hidden_out, workspace, stream=None):
    """features_in [B, k+1, fuse_taps * d], hidden_out [B, k+1, d] or None: fp32 device tensors."""
    _check(lib().spec_verify_forward_features(model, kv, B, k, _ptr(seq_ids), _ptr(tokens), _ptr(features_in), _ptr(logits),
                                              _ptr(hidden_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                              _stream(stream)))


def spec_next_step_hidden(B, k, d, target_hidden, accept_len, pending_hidden, stream=None):
    _check(lib().spec_next_step_hidden(B, k, int(d), _ptr(target_hidden), _ptr(accept_len), _ptr(pending_hidden), _stream(stream)))


def spec_sample_workspace_bytes(B, k):
    return lib().spec_sample_workspace_bytes(B, k)


def spec_reject_sample(B, k, V, logits, q, draft_tokens, temperature, seed, step, accept_len, out_tokens, dbg,
                       workspace, stream=None):
    _check(lib().spec_reject_sample(B, k, V, _ptr(logits), _ptr(q), _ptr(draft_tokens), float(temperature),
                                    int(seed), int(step), _ptr(accept_len), _ptr(out_tokens), _ptr(dbg),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def spec_reject_sample_static(B, k, V, logits, q, draft_tokens, temperature, seed, step, accept_len, out_tokens, dbg, stream=None):
    _check(lib().spec_reject_sample_static(B, k, V, _ptr(logits), _ptr(q), _ptr(draft_tokens), float(temperature),
                                           int(seed), int(step), _ptr(accept_len), _ptr(out_tokens), _ptr(dbg), _stream(stream)))


def spec_commit_kv(kv, B, k, seq_ids, accept_len, new_ctx_len, commit_slots, stream=None):
    _check(lib().spec_commit_kv(kv, B, k, _ptr(seq_ids), _ptr(accept_len), _ptr(new_ctx_len), _ptr(commit_slots),
                                _stream(stream)))


def spec_draft_sample_workspace_bytes(B):
    return int(lib().spec_draft_sample_workspace_bytes(int(B)))


_draft_ws = {}


def spec_draft_sample(B, V, logits, logits_row_stride, temperature, seed, step, row, tokens_a, stride_a, tokens_b, stride_b,
                      q, q_row_stride, stream=None, workspace=None):
    """logits, tokens_a, tokens_b, q: device tensors or raw addresses (ints) of the first row / element.
    workspace: uint8 device tensor of spec_draft_sample_workspace_bytes(B) bytes (one per batch size is kept here if none is given)."""
    if workspace is None:
        if B not in _draft_ws:
            _draft_ws[B] = torch.empty(spec_draft_sample_workspace_bytes(B), dtype=torch.uint8, device="cuda")
        workspace = _draft_ws[B]
    _check(lib().spec_draft_sample(B, V, _addr(logits), int(logits_row_stride), float(temperature), int(seed), int(step),
                                   int(row), _addr(tokens_a), int(stride_a), _addr(tokens_b), int(stride_b), _addr(q),
                                   int(q_row_stride), _ptr(workspace), workspace.numel(), _stream(stream)))


def spec_draft_sample_mapped(B, V_d, logits, logits_row_stride, temperature, seed, step, row, tokens_a, stride_a, tokens_b, stride_b,
                             q, q_row_stride, token_map, V_full, stream=None, workspace=None):
    """As spec_draft_sample for a draft head over a subset of the vocabulary: token_map [V_d] int32 device tensor of
    target ids, q rows V_full wide."""
    if workspace is None:
        if B not in _draft_ws:
            _draft_ws[B] = torch.empty(spec_draft_sample_workspace_bytes(B), dtype=torch.uint8, device="cuda")
        workspace = _draft_ws[B]
    _check(lib().spec_draft_sample_mapped(B, V_d, _addr(logits), int(logits_row_stride), float(temperature), int(seed), int(step),
                                          int(row), _addr(tokens_a), int(stride_a), _addr(tokens_b), int(stride_b), _addr(q),
                                          int(q_row_stride), _ptr(token_map), int(V_full), _ptr(workspace), workspace.numel(),
                                          _stream(stream)))


def spec_kv_truncate(kv, B, seq_ids, lengths, delta, new_len, stream=None):
    _check(lib().spec_kv_truncate(kv, B, _ptr(seq_ids), _ptr(lengths), int(delta), _ptr(new_len), _stream(stream)))


def spec_next_step_inputs(B, k, tokens, out_tokens, accept_len, pending, stream=None):
    _check(lib().spec_next_step_inputs(B, k, _ptr(tokens), _ptr(out_tokens), _ptr(accept_len), _ptr(pending), _stream(stream)))


def spec_ngram_draft(B, k, n_max, n_min, hist, hist_len, seq_ids, tokens, n_drafted, stream=None):
    """hist [n_rows, cap] int32, hist_len [n_rows], tokens [B, k+1] (out), n_drafted [B] or None."""
    _check(lib().spec_ngram_draft(B, k, int(n_max), int(n_min), _ptr(hist), int(hist.shape[1]), int(hist.shape[0]), _ptr(hist_len),
                                  _ptr(seq_ids), _ptr(tokens), _ptr(n_drafted), _stream(stream)))


def spec_ngram_append(B, k, hist, hist_len, seq_ids, out_tokens, accept_len, stream=None):
    _check(lib().spec_ngram_append(B, k, _ptr(hist), int(hist.shape[1]), int(hist.shape[0]), _ptr(hist_len), _ptr(seq_ids),
                                   _ptr(out_tokens), _ptr(accept_len), _stream(stream)))


def spec_rollout_retire(B, k, slot_seq, active, accept_len, gen_len, target_len, queue, queue_head, first_token, tokens,
                        release_seq, keep_len, produced, stream=None):
    """All arguments device tensors (int32; produced int64 [1]); queue may be empty (None)."""
    _check(lib().spec_rollout_retire(B, k, int(gen_len.shape[0]), _ptr(slot_seq), _ptr(active), _ptr(accept_len), _ptr(gen_len),
                                     _ptr(target_len), _ptr(queue), 0 if queue is None else int(queue.shape[0]), _ptr(queue_head),
                                     _ptr(first_token), _ptr(tokens), _ptr(release_seq), _ptr(keep_len), _ptr(produced),
                                     _stream(stream)))


def spec_rollout_pending(B, slot_seq_before, slot_seq, active, prev_token, first_token, pending, stream=None):
    _check(lib().spec_rollout_pending(B, int(prev_token.shape[0]), _ptr(slot_seq_before), _ptr(slot_seq), _ptr(active),
                                      _ptr(prev_token), _ptr(first_token), _ptr(pending), _stream(stream)))


def spec_rollout_pending_hidden(B, slot_seq_before, slot_seq, active, seq_hidden, pending_hidden, stream=None):
    """seq_hidden [n_seqs, 2, d], pending_hidden [B, 2, d]: contiguous fp32 device tensors."""
    assert seq_hidden.is_contiguous() and pending_hidden.is_contiguous() and seq_hidden.shape[1:] == pending_hidden.shape[1:]
    _check(lib().spec_rollout_pending_hidden(B, int(seq_hidden.shape[0]), int(seq_hidden.shape[2]), _ptr(slot_seq_before), _ptr(slot_seq),
                                             _ptr(active), _ptr(seq_hidden), _ptr(pending_hidden), _stream(stream)))


def spec_rollout_compact(B, k, slot_seq, active, tokens, n_live, scratch, stream=None):
    """scratch: int32 device tensor of at least B * (k + 3) elements."""
    assert scratch.numel() >= B * (k + 3)
    _check(lib().spec_rollout_compact(B, k, _ptr(slot_seq), _ptr(active), _ptr(tokens), _ptr(n_live), _ptr(scratch), _stream(stream)))


def spec_tune_set(name, value):
    _check(lib().spec_tune_set(name.encode(), int(value)))


def spec_tune_get(name):
    return lib().spec_tune_get(name.encode())


def spec_profile_class_count():
    return lib().spec_profile_class_count()


def spec_profile_class_name(c):
    name = lib().spec_profile_class_name(c)
    return name.decode() if name else None


def spec_profile_begin(max_events):
    _check(lib().spec_profile_begin(int(max_events)))


def spec_profile_end():
    """Returns {class name: (milliseconds, timed segments)}."""
    n = spec_profile_class_count()
    ms = np.zeros(n, dtype=np.float64)
    cnt = np.zeros(n, dtype=np.int64)
    _check(lib().spec_profile_end(ms.ctypes.data, cnt.ctypes.data, n))
    return {spec_profile_class_name(c): (float(ms[c]), int(cnt[c])) for c in range(n)}


def spec_graph_capture_begin(stream=None):
    _check(lib().spec_graph_capture_begin(_stream(stream)))


def spec_graph_capture_end(stream=None):
    out = ctypes.c_void_p()
    _check(lib().spec_graph_capture_end(_stream(stream), ctypes.byref(out)))
    return out


def spec_graph_launch(graph, stream=None):
    _check(lib().spec_graph_launch(graph, _stream(stream)))


def spec_graph_destroy(graph):
    _check(lib().spec_graph_destroy(graph))


def spec_calib_read(src, nbytes, sink, workgroups, stream=None):
    _check(lib().spec_calib_read(_ptr(src), int(nbytes), _ptr(sink), int(workgroups), _stream(stream)))


def spec_calib_copy(dst, src, nbytes, workgroups, stream=None):
    _check(lib().spec_calib_copy(_ptr(dst), _ptr(src), int(nbytes), int(workgroups), _stream(stream)))
