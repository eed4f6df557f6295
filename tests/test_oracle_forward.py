"""Pins for the forward-pass oracle (numpy fp64) against library routines, closed forms and invariants.

The decoder is the standard one (Section 2.1-2.2 of the paper only says the target verifies the
drafts in one decode-phase pass), so the pins are:
  * an independent composition out of PyTorch CPU fp64 library routines
    (scaled_dot_product_attention with an explicit mask, rms_norm, silu, embedding, complex
    multiplication for the rotary embedding);
  * one pass over k+1 positions == k+1 single-token decodes == the tail of one causal pass
    from an empty cache;
  * closed forms: zero output projections; zero queries give the mean of the visible values
    (pins the causal visibility count); the rotary score depends on the position difference only;
  * grouped-query attention == multi-head attention with repeated key/value heads.
"""
import copy

import numpy as np
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import forward as of

CFG = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=96, vocab=50,
           rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f64", tied_head=0)


def _weights(cfg, seed=1, std=0.2):
    w = si.make_weights(cfg, seed=seed, std=std)
    # non-trivial gains so that a dropped or misplaced gain shows
    g = torch.Generator().manual_seed(seed + 100)
    for name in w:
        if name.endswith("norm"):
            w[name] = 1.0 + 0.3 * torch.randn(w[name].shape, generator=g)
    return si.weights_for_oracle(cfg, w)


def _random_ctx(cfg, ctx_len, seed=2):
    return si.kv_for_oracle(si.make_logical_kv(dict(cfg, dtype="f32" if cfg["dtype"] == "f64" else cfg["dtype"]), ctx_len, seed=seed))


def _torch_reference(cfg, w, kv_ctx, tokens, ctx_len):
    """Same computation out of torch fp64 library calls, one sequence at a time."""
    T64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    Hq, Hkv, dh, d = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_model"]
    half = dh // 2
    inv_freq = cfg["rope_theta"] ** (-torch.arange(half, dtype=torch.float64) * 2 / dh)
    out = []
    for b in range(tokens.shape[0]):
        x = F.embedding(torch.from_numpy(tokens[b].astype(np.int64)), T64(w["embed"]))
        Tn = x.shape[0]
        pos = torch.arange(Tn, dtype=torch.float64) + float(ctx_len[b])
        rot = torch.polar(torch.ones(Tn, half, dtype=torch.float64), pos[:, None] * inv_freq[None, :])

        def rope(t):                                        # [Tn, H, dh] via complex multiply
            z = torch.complex(t[..., :half], t[..., half:]) * rot[:, None, :]
            return torch.cat([z.real, z.imag], dim=-1)
        for l in range(cfg["n_layers"]):
            lw = w["layers"][l]
            h = F.rms_norm(x, (d,), T64(lw["attn_norm"]), cfg["rms_eps"])
            q = rope(F.linear(h, T64(lw["wq"])).view(Tn, Hq, dh))
            kk = rope(F.linear(h, T64(lw["wk"])).view(Tn, Hkv, dh))
            vv = F.linear(h, T64(lw["wv"])).view(Tn, Hkv, dh)
            K = torch.cat([T64(kv_ctx[l][b][0]), kk]).repeat_interleave(Hq // Hkv, dim=1)
            V = torch.cat([T64(kv_ctx[l][b][1]), vv]).repeat_interleave(Hq // Hkv, dim=1)
            S = K.shape[0]
            mask = torch.arange(S)[None, :] <= (int(ctx_len[b]) + torch.arange(Tn))[:, None]
            o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], K.transpose(0, 1)[None],
                                               V.transpose(0, 1)[None], attn_mask=mask[None, None])
            x = x + F.linear(o[0].transpose(0, 1).reshape(Tn, Hq * dh), T64(lw["wo"]))
            h = F.rms_norm(x, (d,), T64(lw["ffn_norm"]), cfg["rms_eps"])
            x = x + F.linear(F.silu(F.linear(h, T64(lw["wg"]))) * F.linear(h, T64(lw["wu"])), T64(lw["wd"]))
        head = w["embed"] if w["head"] is None else w["head"]
        out.append(F.linear(F.rms_norm(x, (d,), T64(w["final_norm"]), cfg["rms_eps"]), T64(head)).numpy())
    return np.stack(out)


def test_against_torch_library_composition():
    cfg = CFG
    w = _weights(cfg)
    rng = np.random.default_rng(0)
    ctx_len = np.array([5, 0, 19])
    kv = _random_ctx(cfg, ctx_len)
    tokens = rng.integers(0, cfg["vocab"], size=(3, 4)).astype(np.int32)
    got, _ = of.verify_forward(cfg, w, kv, tokens, ctx_len)
    want = _torch_reference(cfg, w, kv, tokens, ctx_len)
    assert got.shape == (3, 4, cfg["vocab"])
    assert np.max(np.abs(got - want)) < 1e-10
    assert np.max(np.abs(want)) > 0.1


def test_tied_head_uses_embedding():
    cfg = dict(CFG, tied_head=1)
    w = _weights(cfg)
    assert w["head"] is None
    tokens = np.array([[3, 7]], dtype=np.int32)
    kv = _random_ctx(cfg, [4])
    got, _ = of.verify_forward(cfg, w, kv, tokens, [4])
    want = _torch_reference(cfg, w, kv, tokens, [4])
    assert np.max(np.abs(got - want)) < 1e-10


def test_multi_position_pass_equals_sequential_decodes_and_full_causal_pass():
    cfg = CFG
    w = _weights(cfg, seed=3)
    rng = np.random.default_rng(1)
    C, k = 9, 3
    ctx_tokens = rng.integers(0, cfg["vocab"], size=(2, C)).astype(np.int32)
    new_tokens = rng.integers(0, cfg["vocab"], size=(2, k + 1)).astype(np.int32)
    kv = of.prefill(cfg, w, ctx_tokens)
    ctx_len = np.array([C, C])
    batched, new_kv = of.verify_forward(cfg, w, kv, new_tokens, ctx_len)

    # (a) one causal pass over context + new tokens from an empty cache
    full = np.concatenate([ctx_tokens, new_tokens], axis=1)
    empty = [[(np.zeros((0, 2, 16)), np.zeros((0, 2, 16))) for _ in range(2)] for _ in range(cfg["n_layers"])]
    full_logits, _ = of.verify_forward(cfg, w, empty, full, np.zeros(2, dtype=int))
    assert np.max(np.abs(full_logits[:, C:, :] - batched)) < 1e-10

    # (b) k+1 single-token decodes, appending each position's key/value to the cache
    cache = [[(kv[l][b][0].copy(), kv[l][b][1].copy()) for b in range(2)] for l in range(cfg["n_layers"])]
    for i in range(k + 1):
        step_logits, step_kv = of.verify_forward(cfg, w, cache, new_tokens[:, i:i + 1], ctx_len + i)
        assert np.max(np.abs(step_logits[:, 0, :] - batched[:, i, :])) < 1e-10
        for l in range(cfg["n_layers"]):
            assert np.max(np.abs(step_kv[l][0][:, 0] - new_kv[l][0][:, i])) < 1e-10
            cache[l] = [(np.concatenate([cache[l][b][0], step_kv[l][0][b]]),
                         np.concatenate([cache[l][b][1], step_kv[l][1][b]])) for b in range(2)]


def test_zero_output_projections_give_embedding_logits():
    cfg = CFG
    w = _weights(cfg, seed=4)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["wd"] = np.zeros_like(lw["wd"])
    tokens = np.array([[1, 2, 3]], dtype=np.int32)
    got, _ = of.verify_forward(cfg, w, _random_ctx(cfg, [6]), tokens, [6])
    x = w["embed"][tokens[0]].astype(np.float64)
    y = x / np.sqrt((x * x).mean(-1, keepdims=True) + cfg["rms_eps"]) * w["final_norm"]
    assert np.max(np.abs(got[0] - y @ w["head"].astype(np.float64).T)) < 1e-12


def test_zero_queries_average_the_visible_values():
    """One layer, wq = 0: every score is 0, so head output = mean of the values at positions 0..ctx+i.
    With wo = identity-like selection and no FFN contribution the residual carries that mean."""
    cfg = dict(CFG, n_layers=1, n_q_heads=4, n_kv_heads=4, head_dim=16, d_model=64)
    w = _weights(cfg, seed=5)
    lw = w["layers"][0]
    lw["wq"] = np.zeros_like(lw["wq"])
    lw["wo"] = np.eye(64, dtype=np.float32)
    lw["wd"] = np.zeros_like(lw["wd"])
    w["final_norm"] = np.ones(64, dtype=np.float32)
    ctx = 7
    kv = _random_ctx(cfg, [ctx])
    tokens = np.array([[4, 9, 11]], dtype=np.int32)
    logits, new_kv = of.verify_forward(cfg, w, kv, tokens, [ctx])
    V_all = np.concatenate([kv[0][0][1].astype(np.float64), new_kv[0][1][0]])        # [ctx+3, 4, 16]
    for i in range(3):
        mean_v = V_all[:ctx + i + 1].mean(axis=0).reshape(64)
        x = w["embed"][tokens[0, i]].astype(np.float64) + mean_v
        y = x / np.sqrt((x * x).mean() + cfg["rms_eps"])
        assert np.max(np.abs(logits[0, i] - y @ w["head"].astype(np.float64).T)) < 1e-12


def test_rope_closed_forms():
    rng = np.random.default_rng(6)
    dh, theta = 16, 1.0e4
    a = rng.standard_normal((1, 1, dh))
    b = rng.standard_normal((1, 1, dh))
    # position 0 is the identity; rotation keeps the norm
    assert np.allclose(of.rope(a, [0], theta), a)
    assert np.allclose(np.linalg.norm(of.rope(a, [123], theta)), np.linalg.norm(a))
    # the score depends on the position difference only
    s1 = (of.rope(a, [10], theta) * of.rope(b, [3], theta)).sum()
    s2 = (of.rope(a, [1010], theta) * of.rope(b, [1003], theta)).sum()
    assert abs(s1 - s2) < 1e-9
    # pair (j, j + dh/2) turns by pos * theta^(-2j/dh): check one pair against cos/sin by hand
    j, pos = 3, 5
    ang = pos * theta ** (-2.0 * j / dh)
    r = of.rope(a, [pos], theta)[0, 0]
    assert abs(r[j] - (a[0, 0, j] * np.cos(ang) - a[0, 0, j + 8] * np.sin(ang))) < 1e-12
    assert abs(r[j + 8] - (a[0, 0, j + 8] * np.cos(ang) + a[0, 0, j] * np.sin(ang))) < 1e-12


def test_grouped_query_equals_multi_head_with_repeated_kv_heads():
    cfg = CFG                                               # 4 query heads, 2 kv heads
    w = _weights(cfg, seed=7)
    ctx_len = [6, 11]
    kv = _random_ctx(cfg, ctx_len)
    tokens = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], dtype=np.int32)
    got, _ = of.verify_forward(cfg, w, kv, tokens, ctx_len)

    mha = dict(cfg, n_kv_heads=4)
    w2 = copy.deepcopy(w)
    for lw in w2["layers"]:
        for name in ("wk", "wv"):
            m = lw[name].reshape(2, 16, 64)
            lw[name] = np.repeat(m, 2, axis=0).reshape(64, 64)
    kv2 = [[(np.repeat(K, 2, axis=1), np.repeat(V, 2, axis=1)) for (K, V) in per] for per in kv]
    want, _ = of.verify_forward(mha, w2, kv2, tokens, ctx_len)
    assert np.max(np.abs(got - want)) < 1e-10


def test_sequences_are_independent():
    cfg = CFG
    w = _weights(cfg, seed=8)
    ctx_len = [3, 8, 5]
    kv = _random_ctx(cfg, ctx_len)
    tokens = np.arange(12, dtype=np.int32).reshape(3, 4)
    all_logits, _ = of.verify_forward(cfg, w, kv, tokens, ctx_len)
    one, _ = of.verify_forward(cfg, w, [[per[1]] for per in kv], tokens[1:2], ctx_len[1:2])
    assert np.max(np.abs(all_logits[1] - one[0])) < 1e-12


def test_cache_storage_rounding_matches_library_conversion_and_is_applied_to_new_entries():
    """The cache stores bf16 (or fp32): the oracle's rounding equals torch's conversion bit for bit, the
    returned new entries are storage-type values, and a step that re-reads them from the cache (next
    step's context) sees exactly what the writing step attended to."""
    rng = np.random.default_rng(9)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, size=5000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]])
    want = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(of.round_to_storage(a, "bf16"), want)
    assert np.array_equal(of.round_to_storage(a, "f32"), a.astype(np.float32).astype(np.float64))
    assert np.array_equal(of.round_to_storage(a, "f64"), a)

    cfg = dict(CFG, dtype="bf16")
    w = _weights(cfg, seed=11)
    kv = _random_ctx(cfg, [6])
    tokens = np.array([[1, 2, 3, 4]], dtype=np.int32)
    logits, new_kv = of.verify_forward(cfg, w, kv, tokens, [6])
    for l in range(cfg["n_layers"]):
        for t in new_kv[l]:
            assert np.array_equal(of.round_to_storage(t, "bf16"), t)
    # decode the last position separately on the cache extended by the first three: same logits
    cache = [[(np.concatenate([kv[l][0][0], new_kv[l][0][0][:3]]), np.concatenate([kv[l][0][1], new_kv[l][1][0][:3]]))]
             for l in range(cfg["n_layers"])]
    last, _ = of.verify_forward(cfg, w, cache, tokens[:, 3:], [9])
    assert np.max(np.abs(last[0, 0] - logits[0, 3])) < 1e-12
    # and the rounding matters: the unrounded variant differs
    plain, _ = of.verify_forward(dict(cfg, dtype="f64"), w, kv, tokens, [6])
    assert np.max(np.abs(plain - logits)) > 1e-6


def test_hidden_state_input_against_torch_composition_and_special_cases():
    """A draft that also takes hidden states: the first layer's input against torch library calls (rms_norm, cat,
    linear), the returned hidden state against the logits it must reproduce, and three reductions: w_fuse = [A | 0]
    ignores the hidden states; w_fuse = [0 | I] with unit gains starts the layers from RMSNorm(hidden); a hidden
    input scaled by a constant changes nothing (it is normalised)."""
    cfg = dict(CFG, n_layers=1, tied_head=1, fuse_hidden=1)
    d = cfg["d_model"]
    w = _weights(cfg, seed=4)
    assert w["fuse"]["w_fuse"].shape == (d, 2 * d)
    rng = np.random.default_rng(1)
    ctx_len = np.array([3, 0])
    kv = _random_ctx(cfg, ctx_len)
    tokens = rng.integers(0, cfg["vocab"], size=(2, 3)).astype(np.int32)
    hid = rng.standard_normal((2, 3, d)) * 2.5
    logits, new_kv, h_out = of.verify_forward(cfg, w, kv, tokens, ctx_len, hidden_in=hid, return_hidden=True)
    # (1) the layers run on x0 = linear(cat(rms_norm(embed), rms_norm(hidden))): feed x0 to a plain model through a
    # one-hot "embedding" table holding x0 itself
    T64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    e = F.rms_norm(F.embedding(torch.from_numpy(tokens.reshape(-1).astype(np.int64)), T64(w["embed"])), (d,), T64(w["fuse"]["norm_e"]), cfg["rms_eps"])
    h = F.rms_norm(T64(hid.reshape(-1, d)), (d,), T64(w["fuse"]["norm_h"]), cfg["rms_eps"])
    x0 = F.linear(torch.cat([e, h], dim=1), T64(w["fuse"]["w_fuse"])).numpy()
    plain_cfg = dict(cfg, fuse_hidden=0, vocab=6, tied_head=0)
    plain_w = dict(w, embed=x0, head=w["embed"])
    ids = np.arange(6, dtype=np.int32).reshape(2, 3)
    want = _torch_reference(plain_cfg, plain_w, kv, ids, ctx_len)
    assert np.max(np.abs(logits - want)) < 1e-10 and np.max(np.abs(want)) > 0.05
    # (2) the hidden state returned is what the head sees
    again = of.rmsnorm(h_out.reshape(-1, d), w["final_norm"], cfg["rms_eps"]) @ np.asarray(w["embed"], dtype=np.float64).T
    assert np.max(np.abs(again.reshape(logits.shape) - logits)) < 1e-10
    # (3) reductions
    wa = dict(w, fuse=dict(w["fuse"], w_fuse=np.concatenate([w["fuse"]["w_fuse"][:, :d], np.zeros((d, d))], axis=1)))
    a1, _ = of.verify_forward(cfg, wa, kv, tokens, ctx_len, hidden_in=hid)
    a2, _ = of.verify_forward(cfg, wa, kv, tokens, ctx_len, hidden_in=rng.standard_normal((2, 3, d)))
    assert np.max(np.abs(a1 - a2)) < 1e-12 and np.max(np.abs(a1 - logits)) > 1e-3
    wb = dict(w, fuse=dict(w_fuse=np.concatenate([np.zeros((d, d)), np.eye(d)], axis=1), norm_e=np.ones(d), norm_h=np.ones(d)))
    b1, _ = of.verify_forward(cfg, wb, kv, tokens, ctx_len, hidden_in=hid)
    table = of.rmsnorm(hid.reshape(-1, d), np.ones(d), cfg["rms_eps"])
    b2 = _torch_reference(plain_cfg, dict(w, embed=table, head=w["embed"]), kv, ids, ctx_len)
    assert np.max(np.abs(b1 - b2)) < 1e-10
    c1, _ = of.verify_forward(cfg, w, kv, tokens, ctx_len, hidden_in=hid * 7.0)
    assert np.max(np.abs(c1 - logits)) < 1e-4            # up to the epsilon inside the norm


def test_multi_layer_features_taps_and_their_projection():
    """Features at several depths (the EAGLE-3 input).  Target side: the tap after l layers is the last hidden state
    of the model cut to l layers (a prefix of a decoder does not see what follows), the tap after all layers is the
    returned hidden state, and the taps stand side by side in the order asked for.  Draft side: w_fc = [0 | I | 0]
    picks the middle tap, so the pass equals the single-state one fed that tap; a general w_fc equals the
    single-state pass fed torch's linear(features, w_fc)."""
    cfg = dict(CFG, n_layers=3)
    d = cfg["d_model"]
    w = _weights(cfg, seed=6)
    rng = np.random.default_rng(3)
    ctx_len = np.array([4, 1])
    kv = _random_ctx(cfg, ctx_len)
    tokens = rng.integers(0, cfg["vocab"], size=(2, 3)).astype(np.int32)
    logits, _, hid, feats = of.verify_forward(cfg, w, kv, tokens, ctx_len, return_hidden=True, tap_layers=(1, 3, 2))
    assert feats.shape == (2, 3, 3 * d)
    assert np.array_equal(feats[..., d:2 * d], hid)
    for col, l in ((0, 1), (2, 2)):
        cut_w = dict(w, layers=w["layers"][:l])
        _, _, h_cut = of.verify_forward(dict(cfg, n_layers=l), cut_w, kv[:l], tokens, ctx_len, return_hidden=True)
        assert np.array_equal(feats[..., col * d:(col + 1) * d], h_cut)
    assert np.max(np.abs(feats[..., :d] - feats[..., 2 * d:])) > 1e-3          # the depths differ
    logits2, _ = of.verify_forward(cfg, w, kv, tokens, ctx_len)
    assert np.array_equal(logits, logits2)                                       # asking for taps changes nothing else
    # draft side
    cfg_d = dict(CFG, n_layers=1, tied_head=1, fuse_hidden=1, fuse_taps=3)
    wd_ = _weights(cfg_d, seed=7)
    assert wd_["fuse"]["w_fc"].shape == (d, 3 * d)
    kv_d = _random_ctx(cfg_d, ctx_len, seed=5)
    scaled = feats * 3.0
    pick = dict(wd_, fuse=dict(wd_["fuse"], w_fc=np.concatenate([np.zeros((d, d)), np.eye(d), np.zeros((d, d))], axis=1)))
    a, _ = of.verify_forward(cfg_d, pick, kv_d, tokens, ctx_len, features_in=scaled)
    b, _ = of.verify_forward(cfg_d, pick, kv_d, tokens, ctx_len, hidden_in=scaled[..., d:2 * d])
    assert np.max(np.abs(a - b)) < 1e-12
    T64 = lambda x: torch.from_numpy(np.asarray(x, dtype=np.float64))
    g = F.linear(T64(scaled.reshape(-1, 3 * d)), T64(wd_["fuse"]["w_fc"])).numpy().reshape(2, 3, d)
    c, _, hc = of.verify_forward(cfg_d, wd_, kv_d, tokens, ctx_len, features_in=scaled, return_hidden=True)
    e, _, he = of.verify_forward(cfg_d, wd_, kv_d, tokens, ctx_len, hidden_in=g, return_hidden=True)
    assert np.max(np.abs(c - e)) < 1e-10 and np.max(np.abs(hc - he)) < 1e-10 and np.max(np.abs(c - a)) > 1e-3
    # every tap reaches the result: zeroing one third of the features changes the logits
    for col in range(3):
        z = scaled.copy()
        z[..., col * d:(col + 1) * d] = 0.0
        zl, _ = of.verify_forward(cfg_d, wd_, kv_d, tokens, ctx_len, features_in=z)
        assert np.max(np.abs(zl - c)) > 1e-4
