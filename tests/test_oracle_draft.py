"""Pins for the draft-side oracles: the proposal draw, the autoregressive draft loop and the cache
roll-back after verification.

The paper (Section 2.1) needs two things from the draft side: the drafted token is a sample of the
distribution q that the verifier is given (otherwise the rejection procedure is no longer lossless),
and the draft proposes k tokens one after the other.  Pinned here without retyping the oracle:
  * q against scipy's softmax; the drawn tokens against q by chi-square;
  * draft -> verify chain: with drafts drawn by the draft oracle and verified by the rejection oracle,
    the first emitted token follows the TARGET distribution (fails if the draw is biased or if its random
    stream is correlated with the verifier's streams);
  * the loop against a cache-free recomputation: every iteration's distribution equals the one a single
    causal pass over the whole token string gives;
  * roll-back against a set-based model and against "commit with the smaller acceptance" directly.
"""
import numpy as np
from scipy import stats
from scipy.special import softmax as scipy_softmax

from oracle import draft as od
from oracle import forward as of
from oracle import sampler
from oracle.commit import KVBook

CFG = dict(n_layers=1, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=48, vocab=50,
           rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f64", tied_head=1)


def _weights(cfg, seed=0, std=0.3):
    rng = np.random.default_rng(seed)
    d, Hq, Hkv, dh, F, V = cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["ffn_dim"], cfg["vocab"]
    layers = [dict(attn_norm=1 + 0.1 * rng.standard_normal(d), wq=rng.standard_normal((Hq * dh, d)) * std,
                   wk=rng.standard_normal((Hkv * dh, d)) * std, wv=rng.standard_normal((Hkv * dh, d)) * std,
                   wo=rng.standard_normal((d, Hq * dh)) * std, ffn_norm=1 + 0.1 * rng.standard_normal(d),
                   wg=rng.standard_normal((F, d)) * std, wu=rng.standard_normal((F, d)) * std,
                   wd=rng.standard_normal((d, F)) * std) for _ in range(cfg["n_layers"])]
    out = dict(embed=rng.standard_normal((V, d)), layers=layers, final_norm=1 + 0.1 * rng.standard_normal(d), head=None)
    if cfg.get("fuse_hidden", 0):
        out["fuse"] = dict(w_fuse=rng.standard_normal((d, 2 * d)) * std, norm_e=1 + 0.1 * rng.standard_normal(d),
                           norm_h=1 + 0.1 * rng.standard_normal(d))
        if cfg.get("fuse_taps", 0):
            out["fuse"]["w_fc"] = rng.standard_normal((d, cfg["fuse_taps"] * d)) * std
    return out


def test_proposal_distribution_is_softmax_and_tokens_follow_it():
    V, N, T = 16, 400_000, 0.8
    rng = np.random.default_rng(2)
    row = (rng.standard_normal(V) * 1.5).astype(np.float32)
    logits = np.broadcast_to(row, (N, V)).copy()
    x, q = sampler.draft_sample(logits, T, 11, 4, 2)
    want = scipy_softmax(row.astype(np.float64) / float(np.float32(T)))      # the temperature is an fp32 argument
    assert np.max(np.abs(q[0] - want)) < 1e-7 and np.all(q == q[0])
    obs = np.bincount(x, minlength=V).astype(np.float64)
    chi2 = float(((obs - want * N) ** 2 / (want * N)).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    # deterministic; a different row, step or seed is a different draw
    x2, _ = sampler.draft_sample(logits, T, 11, 4, 2)
    assert np.array_equal(x, x2)
    for args in ((11, 4, 3), (11, 5, 2), (12, 4, 2)):
        xo, _ = sampler.draft_sample(logits, T, *args)
        assert (xo != x).mean() > 0.5
    # the reported keys: winner above runner-up, and the winner is the reported token's key
    xs, qs, keys = sampler.draft_sample(logits[:5], T, 11, 4, 2, debug=True)
    for b in range(5):
        k_all = [want[v] / -np.log(sampler.uniform_draft(11, 4, b, 2, v)) for v in range(V)]
        assert int(np.argmax(k_all)) == xs[b] and abs(keys[b, 0] - max(k_all)) < 1e-12 * max(k_all)
        assert keys[b, 1] < keys[b, 0]


def test_draft_then_verify_chain_is_lossless():
    """Drafts drawn by the draft oracle, verified by the rejection oracle: first emitted token ~ target p_1,
    and the acceptance length has the closed-form mean for prefix-independent rows."""
    V, k, N = 12, 3, 500_000
    rng = np.random.default_rng(8)
    target = (rng.standard_normal((k + 1, V)) * 1.5).astype(np.float32)
    draft_logits = (target[:k] + rng.standard_normal((k, V))).astype(np.float32)
    drafts = np.zeros((N, k), dtype=np.int32)
    q = np.zeros((N, k, V), dtype=np.float32)
    for i in range(k):
        drafts[:, i], q[:, i, :] = sampler.draft_sample(np.broadcast_to(draft_logits[i], (N, V)).copy(), 1.0, 21, 9, i)
    n, out = sampler.reject_sample(np.broadcast_to(target, (N, k + 1, V)).copy(), q, drafts, 1.0, 21, 9)
    p = scipy_softmax(target.astype(np.float64), axis=-1)
    obs = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    chi2 = float(((obs - p[0] * N) ** 2 / (p[0] * N)).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    kept = n >= 1
    obs2 = np.bincount(out[kept, 1], minlength=V).astype(np.float64)
    chi2 = float(((obs2 - p[1] * kept.sum()) ** 2 / (p[1] * kept.sum())).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    beta = np.minimum(p[:k], q[0].astype(np.float64)).sum(axis=-1)
    alpha = 1 + beta[0] + beta[0] * beta[1] + beta[0] * beta[1] * beta[2]
    assert abs((n + 1).mean() - alpha) < 0.01


def test_draft_loop_equals_cache_free_recomputation():
    cfg = CFG
    w = _weights(cfg, seed=5)
    rng = np.random.default_rng(6)
    B, C, k, T = 3, 7, 4, 0.9
    ctx_tokens = rng.integers(0, cfg["vocab"], size=(B, C)).astype(np.int32)
    pending = rng.integers(0, cfg["vocab"], size=(B, 2)).astype(np.int32)
    kv = of.prefill(cfg, w, ctx_tokens)
    drafts, q, kv_out, new_len, keys = od.draft_loop(cfg, w, kv, pending, np.full(B, C), k, T, 77, 3)
    assert drafts.shape == (B, k) and q.shape == (B, k, cfg["vocab"]) and np.all(keys[..., 0] > keys[..., 1])
    assert list(new_len) == [C + 2 + k - 1] * B
    empty = [[(np.zeros((0, 2, 16)), np.zeros((0, 2, 16))) for _ in range(B)] for _ in range(cfg["n_layers"])]
    string = np.concatenate([ctx_tokens, pending], axis=1)
    for i in range(k):
        logits, _ = of.verify_forward(cfg, w, empty, string, np.zeros(B, dtype=int))
        x, qi = sampler.draft_sample(logits[:, -1, :].astype(np.float32), T, 77, 3, i)
        assert np.array_equal(x, drafts[:, i])
        assert np.max(np.abs(qi - q[:, i, :])) < 1e-6
        assert np.max(np.abs(q[:, i, :].sum(-1) - 1)) < 1e-5
        string = np.concatenate([string, x[:, None]], axis=1)
    # the cache the loop leaves is the cache of the string without the last draft
    full_kv = of.prefill(cfg, w, string[:, :-1])
    for b in range(B):
        assert kv_out[0][b][0].shape[0] == C + 2 + k - 1
        assert np.max(np.abs(kv_out[0][b][0] - full_kv[0][b][0])) < 1e-10
        assert np.max(np.abs(kv_out[0][b][1] - full_kv[0][b][1])) < 1e-10
    # drafts differ across sequences and positions (a constant output would pass the checks above trivially)
    assert len(set(drafts.reshape(-1).tolist())) > 3


def test_truncate_against_set_model_and_against_smaller_commit():
    P = 16
    for ctx in (0, 1, 15, 16, 17, 31, 32, 47):
        for k in (3, 7):
            for n in range(k + 1):
                for m in range(n + 1):
                    a = KVBook(n_pages=12, page_size=P)
                    a.assign(0, ctx, list(range(5, 5 + -(-ctx // P))))
                    a.reserve([0], k)
                    a.commit([0], [n], k)
                    got = a.truncate([0], [ctx + m + 1])
                    b = KVBook(n_pages=12, page_size=P)
                    b.assign(0, ctx, list(range(5, 5 + -(-ctx // P))))
                    b.reserve([0], k)
                    b.commit([0], [m], k)
                    assert got == [ctx + m + 1]
                    assert a.pages[0] == b.pages[0] and a.free == b.free and a.ctx_len == b.ctx_len
                    # set model: pages that hold positions 0 .. new-1
                    assert len(a.pages[0]) == len({p // P for p in range(ctx + m + 1)})
                    assert sorted(a.free + a.pages[0]) == list(range(12))
    # never forwards; batch order decides the stack order
    book = KVBook(n_pages=8, page_size=P)
    book.assign("a", 40, [1, 2, 3])
    book.assign("b", 33, [4, 5, 6])
    assert book.truncate(["a", "b"], [100, 16]) == [40, 16]
    assert book.pages["a"] == [1, 2, 3] and book.pages["b"] == [4]
    assert book.free[-2:] == [6, 5]
    assert book.truncate(["b", "a"], [0, 17]) == [0, 17]
    assert book.pages["b"] == [] and book.pages["a"] == [1, 2] and book.free[-2:] == [4, 3]


def test_rollout_over_several_steps_keeps_consistent_caches():
    """Three speculation steps in a row: lengths add up, the kept tokens re-fed as one causal pass reproduce both
    caches (a wrongly kept or dropped position, or a stale draft cache after roll-back, fails this), a draft that
    is the target itself gets everything accepted, and the run is deterministic."""
    cfg_t = dict(CFG, n_layers=2, tied_head=1)
    cfg_d = CFG
    w_t, w_d = _weights(cfg_t, seed=11), _weights(cfg_d, seed=12)
    rng = np.random.default_rng(13)
    B, C, k, T, S = 3, 6, 3, 1.0, 3
    string = rng.integers(0, cfg_t["vocab"], size=(B, C + 1)).astype(np.int32)      # C cached tokens, then t0
    kv_t = of.prefill(cfg_t, w_t, string[:, :C])
    kv_d = of.prefill(cfg_d, w_d, string[:, :C - 1])
    hist, kv_t2, kv_d2, ctx = od.rollout(cfg_t, w_t, cfg_d, w_d, kv_t, kv_d, string[:, C - 1], string[:, C], np.full(B, C), k, T, 5, S)
    assert len(hist) == S
    total = np.zeros(B, dtype=int)
    kept = [list(string[b]) for b in range(B)]                                       # ..., t0
    for h in hist:
        n, out = h["accept_len"], h["out_tokens"]
        assert np.all((0 <= n) & (n <= k))
        for b in range(B):
            assert list(out[b, :n[b]]) == list(h["drafts"][b, :n[b]]) and np.all(out[b, n[b] + 1:] == -1) and out[b, n[b]] >= 0
            assert h["tokens"][b, 0] == kept[b][-1]                                  # this step's first input = last emitted token
            kept[b] += list(out[b, :n[b] + 1])
        total += n + 1
    assert list(ctx) == list(C + total)
    assert len({tuple(h["accept_len"]) for h in hist}) > 1 or k == 0                 # acceptance really varies here
    for b in range(B):
        s = np.array(kept[b], dtype=np.int32)[None, :]
        want_t = of.prefill(cfg_t, w_t, s[:, :ctx[b]])
        want_d = of.prefill(cfg_d, w_d, s[:, :ctx[b] - 1])
        assert kv_t2[0][b][0].shape[0] == ctx[b] and kv_d2[0][b][0].shape[0] == ctx[b] - 1
        for l in range(cfg_t["n_layers"]):
            assert np.max(np.abs(kv_t2[l][b][0] - want_t[l][0][0])) < 1e-9 and np.max(np.abs(kv_t2[l][b][1] - want_t[l][0][1])) < 1e-9
        assert np.max(np.abs(kv_d2[0][b][0] - want_d[0][0][0])) < 1e-9 and np.max(np.abs(kv_d2[0][b][1] - want_d[0][0][1])) < 1e-9
    hist2, _, _, ctx2 = od.rollout(cfg_t, w_t, cfg_d, w_d, kv_t, kv_d, string[:, C - 1], string[:, C], np.full(B, C), k, T, 5, S)
    assert all(np.array_equal(a["out_tokens"], b["out_tokens"]) for a, b in zip(hist, hist2)) and list(ctx) == list(ctx2)
    # the target as its own draft: p == q, every draft is kept
    kv_same = of.prefill(cfg_d, w_d, string[:, :C])
    hist3, _, _, ctx3 = od.rollout(cfg_d, w_d, cfg_d, w_d, kv_same, kv_d, string[:, C - 1], string[:, C], np.full(B, C), k, T, 5, 2)
    assert all(np.all(h["accept_len"] == k) for h in hist3) and list(ctx3) == [C + 2 * (k + 1)] * B


def test_fused_draft_loop_chains_its_own_hidden_states():
    """The draft with hidden-state input: iteration 1 pairs the pending tokens with the hidden states it is given,
    iteration i > 1 pairs x_{i-1} with the draft's own hidden state of the position before.  Checked against a
    cache-free recomputation written position by position, and next_pending_hidden against its three cases."""
    cfg = dict(CFG, fuse_hidden=1)
    w = _weights(cfg, seed=8)
    d = cfg["d_model"]
    rng = np.random.default_rng(9)
    B, C, k, T = 2, 5, 3, 0.8
    ctx_tokens = rng.integers(0, cfg["vocab"], size=(B, C)).astype(np.int32)
    ctx_hidden = rng.standard_normal((B, C, d))
    pending = rng.integers(0, cfg["vocab"], size=(B, 2)).astype(np.int32)
    pend_hidden = rng.standard_normal((B, 2, d))
    empty = [[(np.zeros((0, 2, 16)), np.zeros((0, 2, 16))) for _ in range(B)] for _ in range(cfg["n_layers"])]
    _, kv0 = of.verify_forward(cfg, w, empty, ctx_tokens, np.zeros(B, dtype=int), hidden_in=ctx_hidden)
    kv = [[(kv0[l][0][b], kv0[l][1][b]) for b in range(B)] for l in range(cfg["n_layers"])]
    drafts, q, kv_out, new_len, _ = od.draft_loop(cfg, w, kv, pending, np.full(B, C), k, T, 31, 2, pend_hidden)
    # recomputation: one causal pass over the whole string with the hidden inputs assembled by hand
    string = np.concatenate([ctx_tokens, pending], axis=1)
    hidden = np.concatenate([ctx_hidden, pend_hidden], axis=1)
    for i in range(k):
        logits, _, h_out = of.verify_forward(cfg, w, empty, string, np.zeros(B, dtype=int), hidden_in=hidden, return_hidden=True)
        x, qi = sampler.draft_sample(logits[:, -1, :].astype(np.float32), T, 31, 2, i)
        assert np.array_equal(x, drafts[:, i]) and np.max(np.abs(qi - q[:, i, :])) < 1e-6
        string = np.concatenate([string, x[:, None]], axis=1)
        hidden = np.concatenate([hidden, h_out[:, -1:, :]], axis=1)          # the draft's own state before x
    assert list(new_len) == [C + 2 + k - 1] * B
    # a different pending hidden state changes the proposals' distribution
    _, q2, _, _, _ = od.draft_loop(cfg, w, kv, pending, np.full(B, C), k, T, 31, 2, pend_hidden[:, ::-1, :] * 1.0 + 0.5)
    assert np.max(np.abs(q2 - q)) > 1e-4
    # next step's pending hidden states
    H = rng.standard_normal((3, 4, d))
    old = rng.standard_normal((3, 2, d))
    new = od.next_pending_hidden(old, H, np.array([0, 2, 3]))
    assert np.array_equal(new[0, 0], old[0, 1]) and np.array_equal(new[0, 1], H[0, 0])
    assert np.array_equal(new[1, 0], H[1, 1]) and np.array_equal(new[1, 1], H[1, 2])
    assert np.array_equal(new[2, 0], H[2, 2]) and np.array_equal(new[2, 1], H[2, 3])


def test_feature_draft_loop_projects_the_first_pass_only_and_the_rollout_carries_features():
    """The multi-layer-feature draft (EAGLE-3 input): iteration 1 sends the pending tokens' features through w_fc,
    the chained iterations feed the draft's own d-wide state unprojected.  Checked against the single-state loop fed
    the projected features by hand (numpy matmul), and the two-model rollout against a step-by-step recomputation
    that collects the target's taps with separate cut-down models."""
    cfg = dict(CFG, fuse_hidden=1, fuse_taps=3)
    w = _weights(cfg, seed=8)
    d = cfg["d_model"]
    rng = np.random.default_rng(12)
    B, C, k, T = 2, 4, 3, 0.8
    kv = [[(rng.standard_normal((C, 2, 16)), rng.standard_normal((C, 2, 16))) for _ in range(B)] for _ in range(cfg["n_layers"])]
    pending = rng.integers(0, cfg["vocab"], size=(B, 2)).astype(np.int32)
    feats = rng.standard_normal((B, 2, 3 * d))
    drafts, q, _, new_len, _ = od.draft_loop(cfg, w, kv, pending, np.full(B, C), k, T, 31, 2, feats)
    by_hand = feats @ w["fuse"]["w_fc"].T
    drafts1, q1, _, new_len1, _ = od.draft_loop(dict(cfg, fuse_taps=0), w, kv, pending, np.full(B, C), k, T, 31, 2, by_hand)
    assert np.array_equal(drafts, drafts1) and np.max(np.abs(q - q1)) < 1e-7 and list(new_len) == list(new_len1)
    # two-model rollout: target with 3 layers, taps after layers 1, 3, 2
    cfg_t = dict(CFG, n_layers=3)
    w_t = _weights(cfg_t, seed=3)
    taps = (1, 3, 2)
    string = rng.integers(0, cfg["vocab"], size=(B, C + 1)).astype(np.int32)
    _, kv_t0, = of.verify_forward(cfg_t, w_t, [[(np.zeros((0, 2, 16)), np.zeros((0, 2, 16))) for _ in range(B)] for _ in range(3)],
                                  string[:, :C], np.zeros(B, dtype=int))
    kv_t = [[(kv_t0[l][0][b], kv_t0[l][1][b]) for b in range(B)] for l in range(3)]
    kv_d = [[(K[:C - 1], V[:C - 1]) for (K, V) in per] for per in kv]
    pend = rng.standard_normal((B, 2, 3 * d))
    hist, _, _, ctx = od.rollout(cfg_t, w_t, cfg, w, kv_t, kv_d, string[:, C - 1], string[:, C], np.full(B, C), k, T, 5, 2,
                                 pending_hidden=pend, tap_layers=taps)
    # recomputation of step 0's verify features and step 1's drafts
    tokens0 = hist[0]["tokens"]
    cols = []
    for l in taps:
        _, _, h = of.verify_forward(dict(cfg_t, n_layers=l), dict(w_t, layers=w_t["layers"][:l]), kv_t[:l], tokens0, np.full(B, C), return_hidden=True)
        cols.append(h)
    pend1 = od.next_pending_hidden(pend, np.concatenate(cols, axis=2), hist[0]["accept_len"])
    n0 = hist[0]["accept_len"]
    d0, _, kv_d_grown, _, _ = od.draft_loop(cfg, w, kv_d, np.stack([string[:, C - 1], string[:, C]], axis=1), np.full(B, C - 1), k, T, 5, 0, pend)
    assert np.array_equal(d0, hist[0]["drafts"])
    kv_d1 = [[(K[:C + int(n0[b])], V[:C + int(n0[b])]) for b, (K, V) in enumerate(per)] for per in kv_d_grown]
    # (per-sequence lengths differ: one sequence at a time)
    for b in range(B):
        one = [[per[b]] for per in kv_d1]
        pending1 = np.array([[tokens0[b, n0[b]], hist[0]["out_tokens"][b, n0[b]]]])
        d1, _, _, _, _ = od.draft_loop(cfg, w, one, pending1, np.array([C + int(n0[b])]), k, T, 5, 1, pend1[b:b + 1])
        # rows of one-sequence calls use random-stream row 0: only sequence 0 is comparable draw for draw
        if b == 0:
            assert np.array_equal(d1[0], hist[1]["drafts"][0])


def test_reduced_draft_vocabulary_is_still_lossless():
    """A draft head over a subset of the target's vocabulary (the EAGLE-3 design's reduced draft vocabulary): with the
    identity map the mapped draw is the plain one; otherwise q lives on the subset (zeros elsewhere, sums to 1), the
    drafted tokens are target ids inside the subset and follow q (chi-square), and drafts verified by the rejection
    oracle still give a first emitted token distributed as the target's p over the WHOLE vocabulary - tokens the draft
    can never propose come out of the residual - with the closed-form mean accept length."""
    V, Vd, k, N = 14, 6, 3, 400_000
    rng = np.random.default_rng(18)
    tmap = np.sort(rng.permutation(V)[:Vd])
    target = (rng.standard_normal((k + 1, V)) * 1.2).astype(np.float32)
    draft_logits = (target[:k][:, tmap] + rng.standard_normal((k, Vd)) * 0.7).astype(np.float32)
    # identity map
    lg = (rng.standard_normal((5, V)) * 2).astype(np.float32)
    x0, q0 = sampler.draft_sample(lg, 0.8, 3, 1, 2)
    x1, q1 = sampler.draft_sample_mapped(lg, np.arange(V), V, 0.8, 3, 1, 2)
    assert np.array_equal(x0, x1) and np.array_equal(q0, q1)
    drafts = np.zeros((N, k), dtype=np.int32)
    q = np.zeros((N, k, V), dtype=np.float32)
    for i in range(k):
        drafts[:, i], q[:, i, :] = sampler.draft_sample_mapped(np.broadcast_to(draft_logits[i], (N, Vd)).copy(), tmap, V, 1.0, 21, 9, i)
    outside = np.setdiff1d(np.arange(V), tmap)
    assert np.all(q[:, :, outside] == 0) and np.max(np.abs(q.sum(-1) - 1)) < 1e-6 and np.all(np.isin(drafts, tmap))
    qd = scipy_softmax(draft_logits.astype(np.float64), axis=-1)
    obs = np.bincount(drafts[:, 0], minlength=V)[tmap].astype(np.float64)
    chi2 = float(((obs - qd[0] * N) ** 2 / (qd[0] * N)).sum())
    assert stats.chi2.sf(chi2, df=Vd - 1) > 1e-4
    n, out = sampler.reject_sample(np.broadcast_to(target, (N, k + 1, V)).copy(), q, drafts, 1.0, 21, 9)
    p = scipy_softmax(target.astype(np.float64), axis=-1)
    obs = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    chi2 = float(((obs - p[0] * N) ** 2 / (p[0] * N)).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    assert obs[outside].sum() > 0.5 * N * p[0][outside].sum()                      # tokens outside the subset do get emitted
    beta = np.minimum(p[:k], q[0].astype(np.float64)).sum(axis=-1)
    alpha = 1 + beta[0] + beta[0] * beta[1] + beta[0] * beta[1] * beta[2]
    assert abs((n + 1).mean() - alpha) < 0.01
    # the loop with a reduced head: drafts are target ids, q is as wide as the target's vocabulary
    cfg = dict(CFG, tied_head=0, head_vocab=Vd)
    w = _weights(cfg, seed=5)
    w["head"] = np.random.default_rng(1).standard_normal((Vd, cfg["d_model"])) * 0.3
    tm = np.sort(np.random.default_rng(2).permutation(cfg["vocab"])[:Vd])
    B, C = 2, 4
    kv = [[(rng.standard_normal((C, 2, 16)), rng.standard_normal((C, 2, 16))) for _ in range(B)] for _ in range(cfg["n_layers"])]
    pending = rng.integers(0, cfg["vocab"], size=(B, 2)).astype(np.int32)
    d_, q_, _, _, _ = od.draft_loop(cfg, w, kv, pending, np.full(B, C), 3, 0.9, 5, 0, token_map=tm, v_full=cfg["vocab"])
    assert q_.shape == (B, 3, cfg["vocab"]) and np.all(np.isin(d_, tm)) and np.max(np.abs(q_.sum(-1) - 1)) < 1e-6
