"""CPU oracle for the target model's batched verify forward pass.

TEST INFRASTRUCTURE ONLY (see the package docstring).  numpy, fp64 throughout, one operation
per line of the textbook decoder; ``@`` (matmul) is the only library primitive used as a step.

What it follows.  The paper (Section 2.1-2.2) says only that the target model verifies the k
drafted tokens of each sequence in one decode-phase forward pass; the decoder itself is the
standard pre-norm transformer the paper's models (Qwen3 / Llama class) use: RMSNorm, grouped-query
attention with rotary position embedding, SwiGLU feed-forward, untied or tied output head.

Conventions of this build (the paper does not state them):
  * input row i of sequence b is token t[b,i] at position ctx_len[b] + i; t[b,0] is the last
    emitted token (not yet cached), t[b,1..k] are the drafts; logits row i parameterises the
    distribution of the token that follows t[b,i];
  * RMSNorm: y = x / sqrt(mean(x^2) + eps) * g;
  * rotary embedding pairs element j with j + head_dim/2 and rotates the pair by the angle
    pos * theta^(-2j/head_dim); no long-context frequency scaling;
  * query head j uses key/value head j // (n_q_heads // n_kv_heads);
  * scores are scaled by 1/sqrt(head_dim); row i sees cache positions 0 .. ctx_len[b]+i;
  * silu(z) = z / (1 + exp(-z)); all projections are bias-free, weights are [out, in];
  * mixture-of-experts feed-forward (cfg["n_experts"] > 0; the paper's 235B-A22B target, Section 3.1, is of this
    kind): router logits r = h Wr^T, probabilities softmax(r) over all experts, the top_k most probable experts
    (ties to the lower index) with their probabilities renormalised to sum to one, output = the weighted sum of
    those experts' SwiGLU feed-forwards; every expert has its own gate, up and down matrices;
  * the cache stores keys and values in the model's storage type (cfg["dtype"]: "bf16", "f32", or
    "f64" for none) and attention reads what the cache stores: the keys and values of the k+1 input
    positions are rounded to that type (round to nearest even) before any row attends to them, so
    that a position's key and value are the same numbers in the step that writes them and in every
    later step - which is what makes the verified distribution the one plain decoding would use;
  * 8-bit matrices (``matrix`` below): E4M3 codes with one fp32 scale per output row, W[n][k] = decode(code) * scale[n];
    everything else is computed as with any other matrix;
  * an 8-bit cache (cfg["kv_dtype"] == "fp8_e4m3", see ``oracle/fp8.py``) stores encode(x / scale) with one scale
    per (layer, kv head) for keys and one for values, and attention reads decode(code) * scale.
"""
import numpy as np

from . import fp8


def rmsnorm(x, gain, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def rope(x, positions, theta):
    """x [T, H, dh], positions [T] -> rotated copy."""
    x = np.asarray(x, dtype=np.float64)
    dh = x.shape[-1]
    half = dh // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / dh)
    angle = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]      # [T, half]
    c = np.cos(angle)[:, None, :]
    s = np.sin(angle)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def round_to_storage(a, dtype_name):
    """fp64 array rounded to the cache's storage type, returned as fp64."""
    a = np.asarray(a, dtype=np.float64)
    if dtype_name == "f64":
        return a
    f = a.astype(np.float32)                         # round to nearest even (IEEE conversion)
    if dtype_name == "f32":
        return f.astype(np.float64)
    if dtype_name == "bf16":                         # keep the upper 16 bits, nearest even on the dropped ones
        u = f.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).astype(np.float64)
    raise ValueError("unknown storage type %r" % (dtype_name,))


def silu(z):
    return z / (1.0 + np.exp(-z))


def softmax(s):
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def moe_route(h, router, top_k):
    """h [M, d], router [E, d] -> (experts [M, top_k] int, most probable first; weights [M, top_k] summing to one;
    probabilities [M, E])."""
    r = np.asarray(h, dtype=np.float64) @ np.asarray(router, dtype=np.float64).T
    M, E = r.shape
    prob = np.zeros((M, E))
    experts = np.zeros((M, top_k), dtype=np.int64)
    weight = np.zeros((M, top_k))
    for m in range(M):
        prob[m] = softmax(r[m])
        left = prob[m].copy()
        for j in range(top_k):
            e = int(np.argmax(left))                # first maximum: ties go to the lower index
            experts[m, j] = e
            weight[m, j] = prob[m, e]
            left[e] = -1.0
        weight[m] /= np.sum(weight[m])
    return experts, weight, prob


def moe_ffn(h, w, top_k, route_log=None):
    """Mixture-of-experts SwiGLU feed-forward of rows h [M, d]; w: router [E,d], wg/wu [E,F,d], wd [E,d,F]."""
    h = np.asarray(h, dtype=np.float64)
    experts, weight, prob = moe_route(h, w["router"], top_k)
    if route_log is not None:
        route_log.append((experts, weight, prob))
    out = np.zeros_like(h)
    for m in range(h.shape[0]):
        for j in range(top_k):
            e = experts[m, j]
            gate = matrix(w, "wg", e) @ h[m]
            up = matrix(w, "wu", e) @ h[m]
            out[m] += weight[m, j] * (matrix(w, "wd", e) @ (silu(gate) * up))
    return out


def matrix(w, key, expert=None):
    """A projection matrix of the dict w in fp64 (expert: one of the stacked expert matrices).  8-bit matrices (the
    dict also holds key + "_scale", one factor per output row, and w[key] holds E4M3 codes as uint8):
    W[n][k] = decode(code[n][k]) * scale[n]."""
    m = w[key] if expert is None else w[key][expert]
    if key + "_scale" in w:
        sc = w[key + "_scale"] if expert is None else w[key + "_scale"][expert]
        return fp8.decode(np.asarray(m, dtype=np.uint8)) * np.asarray(sc, dtype=np.float64)[:, None]
    return np.asarray(m, dtype=np.float64)


def verify_forward(cfg, weights, kv_ctx, tokens, ctx_len, route_log=None, hidden_in=None, return_hidden=False,
                   kv_scales=None, features_in=None, tap_layers=None):
    """One verify forward.

    cfg      dict: n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab,
                   rope_theta, rms_eps, dtype (storage type of the cache).
    weights  dict: 'embed' [V,d], 'layers' (list of dicts with attn_norm [d], wq [Hq*dh,d],
                   wk, wv [Hkv*dh,d], wo [d,Hq*dh], ffn_norm [d], wg, wu [F,d], wd [d,F]),
                   'final_norm' [d], 'head' [V,d] or None (tied to 'embed').
    kv_ctx   kv_ctx[layer][b] = (K [ctx_len[b], Hkv, dh], V [ctx_len[b], Hkv, dh]) cached context.
    tokens   [B, k+1] int, ctx_len [B] int.
    Mixture-of-experts models (cfg n_experts, top_k > 0): every layer dict has 'router' [E,d] and stacked
    wg, wu [E,F,d], wd [E,d,F]; route_log (a list) receives per layer (experts, weights, probabilities).

    Draft models that take the verifier's hidden states (cfg fuse_hidden; the paper's EAGLE-3 and MTP drafting
    paths, Section 2.3, consume target hidden states; the combination used here is the MTP one): weights['fuse'] =
    dict(w_fuse [d, 2d], norm_e [d], norm_h [d]) and hidden_in [B, k+1, d]; the input of the first layer is
    w_fuse . [RMSNorm(embedding) * norm_e ; RMSNorm(hidden_in) * norm_h], hidden_in[b][i] being the hidden state
    of the position before input i.

    Multi-layer features (the EAGLE-3 drafting path, Section 2.3: the draft sees the target's state at several depths,
    not only the last): tap_layers = (l_1, .., l_n), 1 <= l_i <= n_layers, makes the target also return the residual
    stream after l_i layers, side by side, [B, k+1, n*d].  A draft with cfg fuse_taps = n holds one more matrix,
    weights['fuse']['w_fc'] [d, n*d]; given features_in [B, k+1, n*d] it takes hidden_in = w_fc . features_in (no
    norm before it; the fusion above normalises the product).  Chained draft passes feed hidden_in directly.

    8-bit cache (cfg kv_dtype "fp8_e4m3"): kv_scales = (k_scale [L, Hkv], v_scale [L, Hkv]); kv_ctx then holds the
    values the cache returns (decode(code) * scale), and so does new_kv.

    Returns (logits [B,k+1,V] fp64, new_kv) with new_kv[layer] = (K [B,k+1,Hkv,dh], V [...]),
    the keys (after rotation) and values of the k+1 input positions as the cache stores them; with return_hidden
    also the residual stream after the last layer, before the final norm, [B,k+1,d]; with tap_layers, last of
    all, the features [B,k+1,n*d].
    """
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    group = Hq // Hkv
    eps, theta = cfg["rms_eps"], cfg["rope_theta"]
    scale = 1.0 / np.sqrt(float(dh))

    embed = np.asarray(weights["embed"], dtype=np.float64)
    x = embed[tokens.reshape(-1)]                                   # [B*T, d]
    if cfg.get("fuse_hidden", 0):
        f = weights["fuse"]
        if features_in is not None:
            assert hidden_in is None and cfg.get("fuse_taps", 0) > 0
            feats = np.asarray(features_in, dtype=np.float64).reshape(B * T, cfg["fuse_taps"] * cfg["d_model"])
            h_in = feats @ np.asarray(f["w_fc"], dtype=np.float64).T
        else:
            h_in = np.asarray(hidden_in, dtype=np.float64).reshape(B * T, -1)
        both = np.concatenate([rmsnorm(x, f["norm_e"], eps), rmsnorm(h_in, f["norm_h"], eps)], axis=1)
        x = both @ np.asarray(f["w_fuse"], dtype=np.float64).T
    pos = (np.asarray(ctx_len)[:, None] + np.arange(T)[None, :]).reshape(-1)

    new_kv = []
    taps = {}
    for layer in range(cfg["n_layers"]):
        w = weights["layers"][layer]
        h = rmsnorm(x, w["attn_norm"], eps)
        q = (h @ matrix(w, "wq").T).reshape(B * T, Hq, dh)
        kx = (h @ matrix(w, "wk").T).reshape(B * T, Hkv, dh)
        vx = (h @ matrix(w, "wv").T).reshape(B * T, Hkv, dh)
        q = rope(q, pos, theta)
        if cfg.get("kv_dtype") == "fp8_e4m3":
            kx = fp8.store(rope(kx, pos, theta), np.asarray(kv_scales[0], dtype=np.float64)[layer][None, :, None])
            vx = fp8.store(vx, np.asarray(kv_scales[1], dtype=np.float64)[layer][None, :, None])
        else:
            kx = round_to_storage(rope(kx, pos, theta), cfg["dtype"])
            vx = round_to_storage(vx, cfg["dtype"])
        new_kv.append((kx.reshape(B, T, Hkv, dh).copy(), vx.reshape(B, T, Hkv, dh).copy()))

        attn = np.zeros((B * T, Hq, dh), dtype=np.float64)
        for b in range(B):
            Kc, Vc = kv_ctx[layer][b]
            K_all = np.concatenate([np.asarray(Kc, dtype=np.float64).reshape(-1, Hkv, dh), kx[b * T:(b + 1) * T]])
            V_all = np.concatenate([np.asarray(Vc, dtype=np.float64).reshape(-1, Hkv, dh), vx[b * T:(b + 1) * T]])
            for i in range(T):
                visible = int(ctx_len[b]) + i + 1                   # positions 0 .. ctx+i
                for j in range(Hq):
                    g = j // group
                    s = (K_all[:visible, g, :] @ q[b * T + i, j, :]) * scale
                    attn[b * T + i, j, :] = softmax(s) @ V_all[:visible, g, :]
        x = x + attn.reshape(B * T, Hq * dh) @ matrix(w, "wo").T

        h = rmsnorm(x, w["ffn_norm"], eps)
        if cfg.get("n_experts", 0) > 0:
            x = x + moe_ffn(h, w, cfg["top_k"], route_log)
        else:
            gate = h @ matrix(w, "wg").T
            up = h @ matrix(w, "wu").T
            x = x + (silu(gate) * up) @ matrix(w, "wd").T
        taps[layer + 1] = x                                         # x is rebound, never updated in place

    head = weights.get("head")
    head = embed if head is None else matrix(weights, "head")
    logits = rmsnorm(x, weights["final_norm"], eps) @ head.T
    out = (logits.reshape(B, T, -1), new_kv)
    if return_hidden:
        out += (x.reshape(B, T, -1).copy(),)
    if tap_layers is not None:
        out += (np.concatenate([taps[int(l)] for l in tap_layers], axis=1).reshape(B, T, -1),)
    return out


def prefill(cfg, weights, tokens, kv_scales=None):
    """Cache contents for context tokens [B, C]: a verify forward from an empty cache.

    Returns kv_ctx in the form ``verify_forward`` takes.
    """
    tokens = np.asarray(tokens)
    B = tokens.shape[0]
    Hkv, dh = cfg["n_kv_heads"], cfg["head_dim"]
    empty = [[(np.zeros((0, Hkv, dh)), np.zeros((0, Hkv, dh))) for _ in range(B)]
             for _ in range(cfg["n_layers"])]
    _, new_kv = verify_forward(cfg, weights, empty, tokens, np.zeros(B, dtype=np.int64), kv_scales=kv_scales)
    return [[(new_kv[layer][0][b], new_kv[layer][1][b]) for b in range(B)] for layer in range(cfg["n_layers"])]
