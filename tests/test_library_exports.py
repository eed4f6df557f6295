"""CPU checks of the boundary: the shared library loads, exports every function the header
declares, and rejects bad arguments on the host before any device work (no GPU needed)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sv():
    from paper_2604_26779_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "spec_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_function_is_exported(sv):
    declared = _declared_functions()
    assert len(declared) >= 20
    lib = sv.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(sv.EXPORTS) == declared          # the binding covers the header, name for name
    for name in declared:
        assert callable(getattr(sv, name)), name


def test_host_side_argument_checks_need_no_gpu(sv):
    assert sv.spec_tune_get("attn_chunk_pages") == 0
    with pytest.raises(sv.SpecError) as e:
        sv.spec_tune_set("no_such_parameter", 1)
    assert e.value.status == sv.SPEC_EINVAL and "no_such_parameter" in str(e.value)
    sv.spec_tune_set("splits_o", 4)
    assert sv.spec_tune_get("splits_o") == 4
    sv.spec_tune_set("splits_o", 0)
    cfg = dict(n_layers=3, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=32, vocab=10,
               rope_theta=1e4, rms_eps=1e-5, dtype="f32", tied_head=0)
    assert sv.spec_model_weight_count(cfg) == 1 + 27 + 2
    assert sv.spec_model_weight_count(dict(cfg, tied_head=1)) == 1 + 27 + 1
    assert sv.spec_sample_workspace_bytes(4, 3) >= 4 * 4 * 8
    assert sv.spec_sample_workspace_bytes(0, 3) == 0
    # validated before any HIP call (the pointers are never dereferenced)
    assert sv.lib().spec_reject_sample(0, 1, 4, 1, 1, 1, 1.0, 0, 0, 1, 1, None, 1, 64, None) == sv.SPEC_EINVAL
    assert "out of range" in sv.spec_last_error()
    assert sv.lib().spec_commit_kv(None, 1, 1, None, None, None, None, None) == sv.SPEC_EINVAL
    assert sv.lib().spec_verify_forward(None, None, 1, 1, None, None, None, None, 0, None) == sv.SPEC_EINVAL
    assert sv.lib().spec_verify_workspace_bytes(None, None, 1, 1) == 0
    assert sv.lib().spec_kv_pool_bytes(None, 1, 0) == -1


def test_argument_checks_of_the_draft_side_calls(sv):
    L = sv.lib()
    ok = dict(B=2, V=10, logits=1, lstride=10, T=1.0, seed=0, step=0, row=0, ta=1, sa=1, tb=None, sb=0, q=1, qstride=10)

    def draft(**kw):
        a = dict(ok, **kw)
        return L.spec_draft_sample(a["B"], a["V"], a["logits"], a["lstride"], a["T"], a["seed"], a["step"], a["row"], a["ta"], a["sa"],
                                   a["tb"], a["sb"], a["q"], a["qstride"], a.get("ws", 1), a.get("ws_bytes", 1 << 20), None)
    assert sv.spec_draft_sample_workspace_bytes(2) > 0 and sv.spec_draft_sample_workspace_bytes(0) == 0
    for bad in (dict(B=0), dict(V=0), dict(row=-1), dict(row=16), dict(T=0.0), dict(step=1 << 30), dict(logits=None), dict(q=None),
                dict(ta=None), dict(lstride=9), dict(qstride=9), dict(sa=0), dict(ws=None), dict(ws_bytes=8)):
        assert draft(**bad) == sv.SPEC_EINVAL, bad
        assert "spec_draft_sample" in sv.spec_last_error()
    # the draw of a head over a subset of the vocabulary: the same checks, and a map and a full width that fit
    okm = dict(ok, V=6, lstride=6, tmap=1, vfull=10)

    def mapped(**kw):
        a = dict(okm, **kw)
        return L.spec_draft_sample_mapped(a["B"], a["V"], a["logits"], a["lstride"], a["T"], a["seed"], a["step"], a["row"], a["ta"], a["sa"],
                                          a["tb"], a["sb"], a["q"], a["qstride"], a["tmap"], a["vfull"], a.get("ws", 1), a.get("ws_bytes", 1 << 20), None)
    for bad in (dict(B=0), dict(V=0), dict(T=0.0), dict(logits=None), dict(q=None), dict(tmap=None), dict(vfull=5), dict(qstride=9),
                dict(lstride=5), dict(ws=None), dict(ws_bytes=8)):
        assert mapped(**bad) == sv.SPEC_EINVAL, bad
        assert "spec_draft_sample_mapped" in sv.spec_last_error()
    assert L.spec_kv_truncate(None, 1, None, None, -1, None, None) == sv.SPEC_EINVAL
    assert L.spec_next_step_inputs(0, 3, 1, 1, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_next_step_inputs(2, 16, 1, 1, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_next_step_inputs(2, 3, None, 1, 1, None, None) == sv.SPEC_EINVAL
    # mixture-of-experts descriptions are counted with their router; the fp32 path refuses them at creation
    moe = dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=256, vocab=10, rope_theta=1e4, rms_eps=1e-5,
               dtype="bf16", tied_head=0, n_experts=4, top_k=2, expert_ffn_dim=256)
    assert sv.spec_model_weight_count(moe) == 1 + 2 * 10 + 2


def test_argument_checks_of_the_rollout_side_calls(sv):
    """n-gram drafter, slot bookkeeping and hidden-state calls reject bad sizes and null pointers before any HIP call."""
    L = sv.lib()
    # spec_ngram_draft(B, k, n_max, n_min, hist, stride, n_rows, hist_len, seq_ids, tokens, n_drafted, stream)
    assert L.spec_ngram_draft(0, 3, 3, 1, 1, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_ngram_draft(2, 16, 3, 1, 1, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_ngram_draft(2, 3, 17, 1, 1, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL      # n_max > 16
    assert L.spec_ngram_draft(2, 3, 2, 3, 1, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL       # n_min > n_max
    assert L.spec_ngram_draft(2, 3, 3, 0, 1, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_ngram_draft(2, 3, 3, 1, None, 8, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL
    assert L.spec_ngram_draft(2, 3, 3, 1, 1, 0, 2, 1, None, 1, None, None) == sv.SPEC_EINVAL
    assert "spec_ngram_draft" in sv.spec_last_error()
    assert L.spec_ngram_append(2, 3, 1, 8, 2, 1, None, None, 1, None) == sv.SPEC_EINVAL
    assert L.spec_ngram_append(2, 3, 1, 8, 0, 1, None, 1, 1, None) == sv.SPEC_EINVAL
    # spec_rollout_retire(B, k, n_seqs, slot_seq, active, accept, gen, target, queue, queue_len, head, first, tokens, rel, keep, produced, stream)
    good = [2, 3, 4, 1, 1, 1, 1, 1, 1, 2, 1, 1, 1, 1, 1, 1, None]
    for pos, bad in ((0, 0), (1, 16), (2, 0), (9, -1), (3, None), (8, None), (15, None)):
        a = list(good)
        a[pos] = bad
        assert L.spec_rollout_retire(*a) == sv.SPEC_EINVAL, (pos, bad)
        assert "spec_rollout_retire" in sv.spec_last_error()
    assert L.spec_rollout_compact(0, 3, 1, 1, 1, 1, 1, None) == sv.SPEC_EINVAL
    assert L.spec_rollout_compact(2, 3, 1, 1, 1, None, 1, None) == sv.SPEC_EINVAL
    assert "spec_rollout_compact" in sv.spec_last_error()
    assert L.spec_next_step_hidden(0, 3, 8, 1, 1, 1, None) == sv.SPEC_EINVAL
    assert L.spec_next_step_hidden(2, 3, 0, 1, 1, 1, None) == sv.SPEC_EINVAL
    assert L.spec_next_step_hidden(2, 3, 8, None, 1, 1, None) == sv.SPEC_EINVAL
    assert L.spec_verify_forward_hidden(None, None, 1, 1, None, None, None, None, None, None, 0, None) == sv.SPEC_EINVAL
    # a model with hidden-state input: three more weights; bf16, dense and wide enough only
    fused = dict(n_layers=1, d_model=256, n_q_heads=2, n_kv_heads=2, head_dim=128, ffn_dim=512, vocab=10, rope_theta=1e4, rms_eps=1e-5,
                 dtype="bf16", tied_head=1, fuse_hidden=1)
    assert sv.spec_model_weight_count(fused) == 1 + 9 + 1 + 3
    assert sv.spec_model_weight_count(dict(fused, fuse_taps=3)) == 1 + 9 + 1 + 3 + 1
    # a head over a subset of the vocabulary is a matrix of its own
    assert sv.spec_model_weight_count(dict(fused, fuse_taps=3, tied_head=0, head_vocab=6)) == 1 + 9 + 1 + 1 + 3 + 1
