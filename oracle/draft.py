"""CPU oracle for the draft side of a speculation step: a small decoder run autoregressively
for k positions, each time drawing the next drafted token from its own distribution.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Composition of the two other oracles:
``forward.verify_forward`` (the decoder) and ``sampler.draft_sample`` (q = softmax(logits / T), x ~ q).

What it follows.  The paper (Section 2.1; Section 3.1, draft-model settings) uses a learned draft
model that proposes k tokens per step (MTP-style: a single decoder layer with the output head tied to
the embedding), after which the target verifies them.  Conventions of this build:
  * the draft keeps a cache of its own; at the start of a step it lacks the positions of the
    ``pending`` tokens (in steady state two: the last input the previous verify kept and the token the
    verifier emitted), which the first iteration feeds together; its last logits row gives q_1;
  * iteration i > 1 feeds the single token x_{i-1}; x_i ~ q_i on random stream 2, row i-1;
  * after k iterations the draft's cache has grown by len(pending) + k - 1 positions: x_k is not fed.
"""
import numpy as np

from . import forward as _forward
from . import sampler as _sampler


def draft_loop(cfg, weights, kv_ctx, pending, ctx_len, k, temperature, seed, step, pending_hidden=None, token_map=None,
               v_full=None):
    """pending [B, P] int tokens not yet in the draft's cache, ctx_len [B] its cached length.

    A draft that takes hidden states (cfg fuse_hidden) gets pending_hidden [B, P, d]: for each pending token the
    verifier's hidden state of the position before it.  Iterations after the first pair the drafted token with the
    draft's own hidden state of the position before it (the last row of the previous iteration), as EAGLE- and
    MTP-style drafters chain their predictions.  A draft with cfg fuse_taps = n takes pending_hidden [B, P, n*d], the
    verifier's multi-layer features, through its w_fc in the first iteration; the chained ones are d wide as before.

    token_map [V_d] + v_full: a draft whose head covers a subset of the target's vocabulary (cfg head_vocab = V_d; its
    embedding still covers all of it, its inputs being target tokens): drafts are target ids and q is laid out over
    the target's v_full entries (``sampler.draft_sample_mapped``).

    Returns (drafts [B, k] int32, q [B, k, V] fp32, kv_ctx grown by the fed positions, new_len [B],
    keys [B, k, 2] = winning and runner-up key of every draw).
    """
    pending = np.asarray(pending)
    B = pending.shape[0]
    ctx_len = np.asarray(ctx_len, dtype=np.int64).copy()
    kv = [[(np.asarray(K, dtype=np.float64), np.asarray(V, dtype=np.float64)) for (K, V) in per_seq] for per_seq in kv_ctx]
    drafts = np.zeros((B, k), dtype=np.int32)
    q = np.zeros((B, k, int(v_full) if token_map is not None else cfg["vocab"]), dtype=np.float32)
    keys = np.zeros((B, k, 2), dtype=np.float64)
    feed = pending
    fused = bool(cfg.get("fuse_hidden", 0))
    feed_hidden = np.asarray(pending_hidden, dtype=np.float64) if fused else None
    taps = int(cfg.get("fuse_taps", 0)) if fused else 0
    for i in range(k):
        if fused and taps and i == 0:
            logits, new_kv, hid = _forward.verify_forward(cfg, weights, kv, feed, ctx_len, features_in=feed_hidden, return_hidden=True)
            feed_hidden = hid[:, -1:, :]
        elif fused:
            logits, new_kv, hid = _forward.verify_forward(cfg, weights, kv, feed, ctx_len, hidden_in=feed_hidden, return_hidden=True)
            feed_hidden = hid[:, -1:, :]
        else:
            logits, new_kv = _forward.verify_forward(cfg, weights, kv, feed, ctx_len)
        for layer in range(cfg["n_layers"]):
            for b in range(B):
                K, V = kv[layer][b]
                kv[layer][b] = (np.concatenate([K, new_kv[layer][0][b]]), np.concatenate([V, new_kv[layer][1][b]]))
        ctx_len += feed.shape[1]
        if token_map is not None:
            x, qi, keys[:, i, :] = _sampler.draft_sample_mapped(logits[:, -1, :].astype(np.float32), token_map, v_full, temperature, seed, step, i, debug=True)
        else:
            x, qi, keys[:, i, :] = _sampler.draft_sample(logits[:, -1, :].astype(np.float32), temperature, seed, step, i, debug=True)
        drafts[:, i] = x
        q[:, i, :] = qi
        feed = x.reshape(B, 1)
    return drafts, q, kv, ctx_len, keys


def next_pending_hidden(pending_hidden, target_hidden, accept_len):
    """Hidden states for the next step's two pending tokens (the last input the verifier kept, and the token it
    emitted): the verifier's hidden states of the positions before them.  With n accepted, the kept input is row n
    of the verify pass: the state before it is row n-1 - or, for n = 0, the state that was paired with the old
    emitted token (pending_hidden[b][1]) - and the state before the new emitted token is row n."""
    B = len(accept_len)
    out = np.zeros_like(np.asarray(pending_hidden, dtype=np.float64))
    for b in range(B):
        n = int(accept_len[b])
        out[b, 0] = target_hidden[b, n - 1] if n >= 1 else pending_hidden[b][1]
        out[b, 1] = target_hidden[b, n]
    return out


def rollout(cfg_t, w_t, cfg_d, w_d, kv_t, kv_d, prev, t0, ctx_len, k, temperature, seed, n_steps, pending_hidden=None,
            tap_layers=None, token_map=None):
    """Several speculation steps in a row (the decode phase of a rollout, Section 2.1-2.2): every step drafts k
    tokens with the draft model, verifies them with the target, keeps the accepted prefix and emits one more
    token, which is the first input of the next step.

    kv_t / kv_d: cached context of target (ctx_len[b] positions) and draft (ctx_len[b] - 1 positions: it lacks
    `prev`, the last input the target has cached); t0 [B]: the last emitted token (cached by neither).
    Random numbers: step s uses counter word `step = s`.  A draft with fuse_taps is fed the target's features at
    tap_layers in place of its last hidden state; pending_hidden is then [B, 2, n*d].

    Returns (history, kv_t, kv_d, ctx_len) with history[s] = dict(drafts [B,k], accept_len [B], out_tokens [B,k+1]);
    the caches hold what each model keeps after the last step (target: ctx_len positions, draft: ctx_len - 1).
    """
    from . import sampler as _s
    B = len(t0)
    ctx_len = np.asarray(ctx_len, dtype=np.int64).copy()
    prev = np.asarray(prev, dtype=np.int32).copy()
    t0 = np.asarray(t0, dtype=np.int32).copy()
    kv_t = [[(np.asarray(K, dtype=np.float64), np.asarray(V, dtype=np.float64)) for (K, V) in per] for per in kv_t]
    kv_d = [[(np.asarray(K, dtype=np.float64), np.asarray(V, dtype=np.float64)) for (K, V) in per] for per in kv_d]
    history = []
    for s in range(n_steps):
        pending = np.stack([prev, t0], axis=1)
        fused = bool(cfg_d.get("fuse_hidden", 0))
        drafts, q, kv_d_grown, _, _ = draft_loop(cfg_d, w_d, kv_d, pending, ctx_len - 1, k, temperature, seed, s,
                                                 pending_hidden if fused else None, token_map=token_map, v_full=cfg_t["vocab"])
        tokens = np.concatenate([t0[:, None], drafts], axis=1).astype(np.int32)
        if fused and tap_layers is not None:
            logits, new_kv, hid_t = _forward.verify_forward(cfg_t, w_t, kv_t, tokens, ctx_len, tap_layers=tap_layers)
        elif fused:
            logits, new_kv, hid_t = _forward.verify_forward(cfg_t, w_t, kv_t, tokens, ctx_len, return_hidden=True)
        else:
            logits, new_kv = _forward.verify_forward(cfg_t, w_t, kv_t, tokens, ctx_len)
        n, out = _s.reject_sample(logits.astype(np.float32), q, drafts, temperature, seed, s)
        if fused:
            pending_hidden = next_pending_hidden(pending_hidden, hid_t, n)
        history.append(dict(drafts=drafts, accept_len=n.copy(), out_tokens=out.copy(), tokens=tokens))
        for b in range(B):
            keep = int(n[b]) + 1                                   # inputs 0..n stay in the target's cache
            for layer in range(cfg_t["n_layers"]):
                K, V = kv_t[layer][b]
                kv_t[layer][b] = (np.concatenate([K, new_kv[layer][0][b][:keep]]), np.concatenate([V, new_kv[layer][1][b][:keep]]))
            new_len = int(ctx_len[b]) + keep
            for layer in range(cfg_d["n_layers"]):                 # the draft keeps one position less than the target
                K, V = kv_d_grown[layer][b]
                kv_d[layer][b] = (K[:new_len - 1], V[:new_len - 1])
            prev[b] = tokens[b, n[b]]
            t0[b] = out[b, n[b]]
            ctx_len[b] = new_len
    return history, kv_t, kv_d, ctx_len
