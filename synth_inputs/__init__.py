"""Seeded synthetic inputs for the verify step: configurations, weights, contexts, page tables.

This module serves both the HIP path and the CPU oracle and holds none of the method's
arithmetic: it only draws random tensors of the shapes and distributions the workloads have,
rounds them to the storage type, and moves data between the logical (per sequence) and the
physical (paged pool) view by plain indexing.  It imports neither the oracle nor the product
package.

Recipe (all draws are functions of an integer seed through ``torch.Generator``):
  * matrices and embedding ~ N(0, 0.02) (0.02 is the standard deviation), rounded to the
    model's storage type; RMSNorm gains are 1;
  * token ids uniform over the vocabulary; context lengths integer-uniform on a closed interval;
  * cached context K and V entries ~ N(0, 1) rounded to the storage type (used where a real
    prefill is too large for the CPU oracle);
  * physical pages are handed out from a shuffled list (worst-case fragmentation) or in order.
"""
import math

import numpy as np
import torch

PAGE_SIZE = 16
DEFAULT_SEED = 20260427

# name -> model description.  dtype is the storage type of weights and of the KV cache.
MODELS = {
    # Tiny fp32 decoder: 2 layers, MHA, vocab 1024.
    "tiny_fp32": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=704,
                      vocab=1024, rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f32", tied_head=0),
    # Small bf16 model for parity tests of the MFMA path: several tiles plus ragged tails in N and V.
    "small_bf16": dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1280,
                       vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=0),
    # Llama-3-8B-shaped.
    "llama8b_bf16": dict(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336,
                         vocab=128256, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=0),
    # Mixture-of-experts models: a small one for parity tests, and a 4-layer slice at the widths of a
    # 235B-A22B-class target: 64 query / 4 kv heads, 128 experts, top-8, expert width 1536.
    "small_moe_bf16": dict(n_layers=2, d_model=512, n_q_heads=16, n_kv_heads=1, head_dim=128, ffn_dim=256, vocab=4000,
                           rope_theta=1.0e6, rms_eps=1.0e-6, dtype="bf16", tied_head=0, n_experts=12, top_k=3,
                           expert_ffn_dim=256),
    "moe235b_slice_bf16": dict(n_layers=4, d_model=4096, n_q_heads=64, n_kv_heads=4, head_dim=128, ffn_dim=1536,
                               vocab=151936, rope_theta=1.0e6, rms_eps=1.0e-6, dtype="bf16", tied_head=0, n_experts=128,
                               top_k=8, expert_ffn_dim=1536),
    # Single-layer draft models (MTP-style: one decoder layer, output head tied to the embedding).
    "draft_tiny_fp32": dict(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=704,
                            vocab=1024, rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f32", tied_head=1),
    "draft_small_bf16": dict(n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1280,
                             vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1),
    # The same, taking the verifier's hidden states as a second input (EAGLE-3 / MTP style input fusion).
    "draft_fused_small_bf16": dict(n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1280,
                                   vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1, fuse_hidden=1),
    "draft1l_fused_8b_bf16": dict(n_layers=1, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336,
                                  vocab=128256, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1, fuse_hidden=1),
    # The EAGLE-3 input: the verifier's residual stream at three depths, side by side, through w_fc [d, 3d] first.
    "draft_eagle3_small_bf16": dict(n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1792,
                                    vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1, fuse_hidden=1,
                                    fuse_taps=3),
    "draft1l_eagle3_8b_bf16": dict(n_layers=1, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336,
                                   vocab=128256, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1, fuse_hidden=1,
                                   fuse_taps=3),
    # The same with the reduced draft vocabulary of that design: an untied head over a subset of the target's tokens.
    "draft_eagle3r_small_bf16": dict(n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1792,
                                     vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=0, fuse_hidden=1,
                                     fuse_taps=3, head_vocab=992),
    "draft1l_eagle3r_8b_bf16": dict(n_layers=1, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336,
                                    vocab=128256, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=0, fuse_hidden=1,
                                    fuse_taps=3, head_vocab=32000),
    # A four-layer target for it at the small widths (taps after layers 1, 2 and 4).
    "small4_bf16": dict(n_layers=4, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=1280,
                        vocab=4000, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=0),
    "draft1l_8b_bf16": dict(n_layers=1, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn_dim=14336,
                            vocab=128256, rope_theta=5.0e5, rms_eps=1.0e-5, dtype="bf16", tied_head=1),
}

# name -> batch description of the verify step.
WORKLOADS = {
    "tiny_fp32_b4_ctx128_k3": dict(model="tiny_fp32", B=4, k=3, ctx_lo=128, ctx_hi=128, noise_std=0.5,
                                   temperature=1.0),
    "small_bf16_b5_k3": dict(model="small_bf16", B=5, k=3, ctx_lo=37, ctx_hi=700, noise_std=1.0,
                             temperature=1.0),
    "llama8b_b32_ctx1k-8k_k3": dict(model="llama8b_bf16", B=32, k=3, ctx_lo=1024, ctx_hi=8192, noise_std=1.0,
                                    temperature=1.0),
}
# Continuous rollout: 32 batch slots, 64 sequences (32 waiting, prompts cached), response lengths long-tailed
# (log-normal, median 24 tokens, clipped to 4..160): the slots drain unevenly, the tail runs with few live slots.
WORKLOADS["rollout_b32_q32_ctx1k-8k_k3"] = dict(model="llama8b_bf16", B=64, slots=32, k=3, ctx_lo=1024, ctx_hi=8192,
                                                noise_std=1.0, temperature=1.0, resp_median=24, resp_sigma=0.8,
                                                resp_lo=4, resp_hi=160)
# Draft + target pair: a single-layer draft run autoregressively for k = 5, then the
# 8B-shaped verify, B = 64, contexts of 4096 tokens.
WORKLOADS["draft_pair_b64_ctx4096_k5"] = dict(model="llama8b_bf16", draft_model="draft1l_8b_bf16", B=64, k=5, ctx_lo=4096,
                                              ctx_hi=4096, noise_std=0.0, temperature=1.0)
WORKLOADS["draft_pair_fused_b64_ctx4096_k5"] = dict(model="llama8b_bf16", draft_model="draft1l_fused_8b_bf16", B=64, k=5,
                                                    ctx_lo=4096, ctx_hi=4096, noise_std=0.0, temperature=1.0)
WORKLOADS["draft_pair_eagle3_b64_ctx4096_k5"] = dict(model="llama8b_bf16", draft_model="draft1l_eagle3_8b_bf16", B=64, k=5,
                                                     ctx_lo=4096, ctx_hi=4096, noise_std=0.0, temperature=1.0,
                                                     tap_layers=(2, 16, 29))
WORKLOADS["draft_pair_eagle3r_b64_ctx4096_k5"] = dict(WORKLOADS["draft_pair_eagle3_b64_ctx4096_k5"], draft_model="draft1l_eagle3r_8b_bf16")
WORKLOADS["draft_pair_eagle3_small_b5_k4"] = dict(model="small4_bf16", draft_model="draft_eagle3_small_bf16", B=5, k=4, ctx_lo=20,
                                                  ctx_hi=600, noise_std=0.0, temperature=0.9, tap_layers=(1, 2, 4))
WORKLOADS["draft_pair_eagle3r_small_b5_k4"] = dict(WORKLOADS["draft_pair_eagle3_small_b5_k4"], draft_model="draft_eagle3r_small_bf16")
WORKLOADS["draft_pair_fused_small_b5_k4"] = dict(model="small_bf16", draft_model="draft_fused_small_bf16", B=5, k=4, ctx_lo=20,
                                                 ctx_hi=600, noise_std=0.0, temperature=0.9)
WORKLOADS["draft_pair_small_b5_k4"] = dict(model="small_bf16", draft_model="draft_small_bf16", B=5, k=4, ctx_lo=20,
                                           ctx_hi=600, noise_std=0.0, temperature=0.9)
WORKLOADS["draft_pair_tiny_b4_k3"] = dict(model="tiny_fp32", draft_model="draft_tiny_fp32", B=4, k=3, ctx_lo=100,
                                          ctx_hi=140, noise_std=0.0, temperature=1.0)
# Mixture-of-experts verify slice: B = 128, contexts uniform in [4096, 32768], k = 3.
WORKLOADS["moe235b_slice_b128_ctx4k-32k_k3"] = dict(model="moe235b_slice_bf16", B=128, k=3, ctx_lo=4096, ctx_hi=32768,
                                                    noise_std=1.0, temperature=1.0)
WORKLOADS["small_moe_b6_k3"] = dict(model="small_moe_bf16", B=6, k=3, ctx_lo=5, ctx_hi=600, noise_std=1.0, temperature=1.0)
# Large rollout batch: B=256, contexts uniform in [2048, 16384], k swept.  The
# cache of 32 distinct layers would not fit one GPU (309 GB on average), so layer l uses layer
# pool l mod 8 (same bytes streamed per step, an eighth of the footprint); the draft noise of
# sequence b is scaled by 2*Beta(4,2) so acceptance rates are mixed over the batch.
for _k in (1, 3, 5, 7):
    WORKLOADS["llama8b_b256_ctx2k-16k_k%d" % _k] = dict(
        model="llama8b_bf16", B=256, k=_k, ctx_lo=2048, ctx_hi=16384, noise_std=1.0, temperature=1.0,
        layer_alias_mod=8, noise_beta=(4.0, 2.0))


# 8-bit (E4M3) KV cache variants: the same models and workloads with the cache stored as codes under one scale per
# (layer, kv head).  With one byte per element the B=256 cache of 32 distinct layers (155 GB) fits one GPU un-aliased.
for _name in ("small_bf16", "llama8b_bf16"):
    MODELS[_name + "_kv8"] = dict(MODELS[_name], kv_dtype="fp8_e4m3")
    MODELS[_name + "_w8kv8"] = dict(MODELS[_name], kv_dtype="fp8_e4m3", w_dtype="fp8_e4m3")     # 8-bit matrices as well
    MODELS[_name + "_w8"] = dict(MODELS[_name], w_dtype="fp8_e4m3")
# a draft with 8-bit matrices: its output head is then a matrix of its own (the quantised embedding), not tied
MODELS["draft1l_8b_bf16_w8"] = dict(MODELS["draft1l_8b_bf16"], tied_head=0, w_dtype="fp8_e4m3", kv_dtype="fp8_e4m3")
MODELS["moe235b_slice_bf16_w8kv8"] = dict(MODELS["moe235b_slice_bf16"], kv_dtype="fp8_e4m3", w_dtype="fp8_e4m3")
WORKLOADS["small_bf16_kv8_b5_k3"] = dict(WORKLOADS["small_bf16_b5_k3"], model="small_bf16_kv8")
WORKLOADS["llama8b_kv8_b32_ctx1k-8k_k3"] = dict(WORKLOADS["llama8b_b32_ctx1k-8k_k3"], model="llama8b_bf16_kv8")
WORKLOADS["small_bf16_w8kv8_b5_k3"] = dict(WORKLOADS["small_bf16_b5_k3"], model="small_bf16_w8kv8")
WORKLOADS["llama8b_w8kv8_b32_ctx1k-8k_k3"] = dict(WORKLOADS["llama8b_b32_ctx1k-8k_k3"], model="llama8b_bf16_w8kv8")
WORKLOADS["llama8b_w8_b32_ctx1k-8k_k3"] = dict(WORKLOADS["llama8b_b32_ctx1k-8k_k3"], model="llama8b_bf16_w8")
# the same continuous rollout driven by the single-layer draft model instead of the n-gram drafter
WORKLOADS["rollout_pair_b32_q32_ctx1k-8k_k3"] = dict(WORKLOADS["rollout_b32_q32_ctx1k-8k_k3"], draft_model="draft1l_8b_bf16", noise_std=0.0)
WORKLOADS["rollout_w8kv8_b32_q32_ctx1k-8k_k3"] = dict(WORKLOADS["rollout_b32_q32_ctx1k-8k_k3"], model="llama8b_bf16_w8kv8")
WORKLOADS["draft_pair_w8kv8_b64_ctx4096_k5"] = dict(WORKLOADS["draft_pair_b64_ctx4096_k5"], model="llama8b_bf16_w8kv8",
                                                    draft_model="draft1l_8b_bf16_w8")
WORKLOADS["moe235b_slice_w8kv8_b128_ctx4k-32k_k3"] = dict(WORKLOADS["moe235b_slice_b128_ctx4k-32k_k3"], model="moe235b_slice_bf16_w8kv8")
WORKLOADS["llama8b_w8kv8_b256_ctx2k-16k_k3"] = dict(WORKLOADS["llama8b_b256_ctx2k-16k_k3"], model="llama8b_bf16_w8kv8", layer_alias_mod=0)
WORKLOADS["llama8b_kv8_b256_ctx2k-16k_k3"] = dict(WORKLOADS["llama8b_b256_ctx2k-16k_k3"], model="llama8b_bf16_kv8",
                                                  layer_alias_mod=0)


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64}[name]


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def weight_shapes(cfg):
    """Canonical, ordered list of (name, shape).  Matrices are [out_features, in_features]."""
    d, Hq, Hkv, dh, F, V = (cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                            cfg["ffn_dim"], cfg["vocab"])
    out = [("embed", (V, d))]
    E = cfg.get("n_experts", 0)
    for l in range(cfg["n_layers"]):
        out += [(f"l{l}.attn_norm", (d,)), (f"l{l}.wq", (Hq * dh, d)), (f"l{l}.wk", (Hkv * dh, d)),
                (f"l{l}.wv", (Hkv * dh, d)), (f"l{l}.wo", (d, Hq * dh)), (f"l{l}.ffn_norm", (d,))]
        if E > 0:        # mixture of experts: stacked expert matrices, then the router
            Fe = cfg["expert_ffn_dim"]
            out += [(f"l{l}.wg", (E, Fe, d)), (f"l{l}.wu", (E, Fe, d)), (f"l{l}.wd", (E, d, Fe)), (f"l{l}.router", (E, d))]
        else:
            out += [(f"l{l}.wg", (F, d)), (f"l{l}.wu", (F, d)), (f"l{l}.wd", (d, F))]
    out.append(("final_norm", (d,)))
    if not cfg.get("tied_head", 0):
        out.append(("head", (cfg.get("head_vocab", 0) or V, d)))
    if cfg.get("fuse_hidden", 0):      # a draft model that also takes the verifier's hidden states
        out += [("w_fuse", (d, 2 * d)), ("fuse_e_norm", (d,)), ("fuse_h_norm", (d,))]
        if cfg.get("fuse_taps", 0):    # ... at several depths: their projection down to d channels
            out += [("w_fc", (d, cfg["fuse_taps"] * d))]
    return out


def make_weights(cfg, seed=DEFAULT_SEED, device="cpu", std=0.02):
    """Ordered dict name -> tensor in the model's storage type on ``device``."""
    g = _gen(seed, device)
    dt = torch_dtype(cfg["dtype"])
    weights = {}
    for name, shape in weight_shapes(cfg):
        if name.endswith("norm"):
            weights[name] = torch.ones(shape, dtype=dt, device=device)
        elif name.endswith("router"):          # router logits of a unit-RMS input ~ N(0, 1)
            weights[name] = (torch.randn(shape, generator=g, device=device, dtype=torch.float32) / math.sqrt(shape[-1])).to(dt)
        else:
            weights[name] = (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(dt)
    if cfg.get("w_dtype") == "fp8_e4m3":
        # 8-bit matrices: the bf16 draws above become E4M3 codes under one scale per output row (absmax / 448, the
        # library's cast); the scales follow all other entries, in matrix order
        scales = {}
        for name in [n for n in weights if n.split(".")[-1] in W8_MATRICES]:
            w = weights[name].to(torch.float32)
            sc = (w.abs().amax(dim=-1) / 448.0).clamp_min(1e-12)       # (stacked expert matrices: one scale per expert and row)
            weights[name] = (w / sc[..., None]).to(torch.float8_e4m3fn)
            scales[name + ".scale"] = sc
            del w
        weights.update(scales)
    return weights


W8_MATRICES = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "head")


def weights_for_oracle(cfg, weights, library_decode=False, own_decode_layers=(0,)):
    """The same values as nested fp32 numpy arrays in the layout the oracle's forward takes.  8-bit matrices go as
    bytes plus scales and the oracle decodes them itself; with library_decode (the full-size shapes, where the oracle's
    elementwise decode of 8e9 codes would take minutes) they go as the library's cast of the codes times the scale, which
    the oracle's decode is pinned against code by code - except the layers in own_decode_layers, which still go as codes
    and scales, so that the oracle's own decoder is on the full-size path too."""
    def f(name):
        # (stacked expert matrices stay with the library's cast: a layer of them is billions of codes)
        own = any(name.startswith("l%d." % l) for l in own_decode_layers) and not (cfg.get("n_experts", 0) > 0 and name.split(".")[-1] in ("wg", "wu", "wd"))
        if name + ".scale" in weights and library_decode and not own:
            return (weights[name].detach().to("cpu", torch.float32) * weights[name + ".scale"].detach().to("cpu", torch.float32)[..., None]).numpy()
        if name + ".scale" in weights:                # 8-bit matrix: the oracle gets the codes (bytes) and the scales
            return weights[name].detach().to("cpu").view(torch.uint8).numpy()
        return weights[name].detach().to("cpu", torch.float32).numpy()

    def scales_of(prefix, keys):
        if library_decode and not any(prefix == "l%d." % l for l in own_decode_layers):
            return {}
        return {k + "_scale": weights[prefix + k + ".scale"].detach().to("cpu", torch.float32).numpy()
                for k in keys if prefix + k + ".scale" in weights and not (library_decode and cfg.get("n_experts", 0) > 0 and k in ("wg", "wu", "wd"))}
    layers = []
    names = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd") + (("router",) if cfg.get("n_experts", 0) > 0 else ())
    for l in range(cfg["n_layers"]):
        layers.append({k: f(f"l{l}.{k}") for k in names})
        layers[-1].update(scales_of(f"l{l}.", names))
    out = {"embed": f("embed"), "layers": layers, "final_norm": f("final_norm"),
           "head": None if cfg.get("tied_head", 0) else f("head")}
    out.update(scales_of("", ("head",)))
    if cfg.get("fuse_hidden", 0):
        out["fuse"] = {"w_fuse": f("w_fuse"), "norm_e": f("fuse_e_norm"), "norm_h": f("fuse_h_norm")}
        if cfg.get("fuse_taps", 0):
            out["fuse"]["w_fc"] = f("w_fc")
    return out


def make_batch(workload, seed=DEFAULT_SEED, shuffle_pages=True, extra_pages=8):
    """Token ids, context lengths and page lists of one verify step (host side, numpy).

    Returns dict: tokens0 [B] (the last emitted token of each sequence), ctx_len [B],
    ctx_tokens (list of [ctx_len[b]] arrays), page_lists (list of int lists covering exactly the
    context), n_pages (pool size: what the contexts need, what the step may add, plus slack).
    """
    cfg = MODELS[workload["model"]]
    rng = np.random.Generator(np.random.Philox(int(seed) + 1))
    B, k = workload["B"], workload["k"]
    ctx_len = rng.integers(workload["ctx_lo"], workload["ctx_hi"] + 1, size=B).astype(np.int64)
    tokens0 = rng.integers(0, cfg["vocab"], size=B).astype(np.int32)
    ctx_tokens = [rng.integers(0, cfg["vocab"], size=int(c)).astype(np.int32) for c in ctx_len]
    ctx_pages = [-(-int(c) // PAGE_SIZE) for c in ctx_len]
    step_pages = [-(-(int(c) + k + 1) // PAGE_SIZE) for c in ctx_len]
    n_pages = sum(step_pages) + extra_pages
    order = rng.permutation(n_pages) if shuffle_pages else np.arange(n_pages)
    page_lists, at = [], 0
    for n in ctx_pages:
        page_lists.append([int(p) for p in order[at:at + n]])
        at += n
    noise_scale = np.ones(B)
    if workload.get("noise_beta"):
        noise_scale = 2.0 * rng.beta(workload["noise_beta"][0], workload["noise_beta"][1], size=B)
    return dict(tokens0=tokens0, ctx_len=ctx_len, ctx_tokens=ctx_tokens, page_lists=page_lists,
                n_pages=int(n_pages), noise_scale=noise_scale)


def make_logical_kv(cfg, ctx_len, seed=DEFAULT_SEED, device="cpu"):
    """Synthetic cached context: kv[layer][b] = (K, V), each [ctx_len[b], Hkv, dh] ~ N(0,1) in storage type."""
    g = _gen(int(seed) + 2, device)
    kv8 = cfg.get("kv_dtype") == "fp8_e4m3"          # the tensors then hold codes: N(0, KV8_NOMINAL) cast by the library
    dt = torch.float8_e4m3fn if kv8 else torch_dtype(cfg["dtype"])
    std = KV8_NOMINAL if kv8 else 1.0
    Hkv, dh = cfg["n_kv_heads"], cfg["head_dim"]
    kv = []
    for _ in range(cfg["n_layers"]):
        per_seq = []
        for c in ctx_len:
            K = (torch.randn((int(c), Hkv, dh), generator=g, device=device, dtype=torch.float32) * std).to(dt)
            V = (torch.randn((int(c), Hkv, dh), generator=g, device=device, dtype=torch.float32) * std).to(dt)
            per_seq.append((K, V))
        kv.append(per_seq)
    return kv


def kv_for_oracle(kv):
    """kv[layer][b] = (K, V) tensors -> the same nesting with fp32 numpy arrays (an 8-bit cache, whose tensors hold
    codes: the bytes as uint8 arrays; the oracle turns them into values itself)."""
    def conv(t):
        t = t.detach().to("cpu")
        return t.view(torch.uint8).numpy() if t.dtype == torch.float8_e4m3fn else t.to(torch.float32).numpy()
    return [[(conv(K), conv(V)) for (K, V) in per_seq] for per_seq in kv]


KV8_NOMINAL = 48.0      # standard deviation of the synthetic cached context in code units (|x| stays below 448)


def kv_scales(cfg, seed=DEFAULT_SEED):
    """Synthetic calibration of an 8-bit cache: (k_scale, v_scale), each [L, Hkv] fp32, between 1/64 and 1/43 (not
    powers of two), so that N(0,1)-sized entries use the upper binades of the format without saturating."""
    rng = np.random.Generator(np.random.Philox(int(seed) + 31))
    shape = (cfg["n_layers"], cfg["n_kv_heads"])
    return ((1.0 + 0.5 * rng.random(shape)) / 64.0).astype(np.float32), ((1.0 + 0.5 * rng.random(shape)) / 64.0).astype(np.float32)


def round_to_storage(array, dtype_name):
    """Round an fp64/fp32 numpy array to the storage type and return it as fp32 numpy."""
    t = torch.from_numpy(np.ascontiguousarray(array, dtype=np.float32))
    return t.to(torch_dtype(dtype_name)).to(torch.float32).numpy()


def make_sampler_case(B, k, V, seed=DEFAULT_SEED, logit_std=3.0, noise_std=1.0, temperature=1.0):
    """Free-standing sampler inputs: logits ~ N(0, logit_std), q = softmax((logits + noise)/T), drafts ~ q.

    Row i of q is built from logits row i (the row that judges draft i+1).  numpy, fp32.
    """
    rng = np.random.Generator(np.random.Philox(int(seed) + 3))
    logits = (rng.standard_normal((B, k + 1, V)) * logit_std).astype(np.float32)
    noisy = (logits[:, :k, :].astype(np.float64) + rng.standard_normal((B, k, V)) * noise_std) / temperature
    noisy -= noisy.max(axis=-1, keepdims=True)
    q = np.exp(noisy)
    q /= q.sum(axis=-1, keepdims=True)
    q = q.astype(np.float32)
    cdf = np.cumsum(q.astype(np.float64), axis=-1)
    u = rng.random((B, k, 1)) * cdf[..., -1:]
    draft = np.minimum((cdf < u).sum(axis=-1), V - 1).astype(np.int32)
    return logits, q, draft


def draw_from(prob, rng):
    """One categorical draw per row of ``prob`` [..., V] by inverse CDF (input generation only)."""
    cdf = np.cumsum(np.asarray(prob, dtype=np.float64), axis=-1)
    u = rng.random(cdf.shape[:-1] + (1,)) * cdf[..., -1:]
    return np.minimum((cdf < u).sum(axis=-1), prob.shape[-1] - 1).astype(np.int32)


def noisy_draft_distribution(logits_row, noise, temperature):
    """q = softmax((logits + noise) / T) in fp64, returned as fp32 (the draft model stand-in)."""
    z = (np.asarray(logits_row, dtype=np.float64) + noise) / temperature
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def make_token_map(cfg, seed=DEFAULT_SEED):
    """Which tokens of the vocabulary a reduced draft head (cfg head_vocab) covers: a seeded subset, increasing, int32."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    return np.sort(rng.permutation(cfg["vocab"])[:cfg["head_vocab"]]).astype(np.int32)


def device_draft_step(logits_row, std, temperature, generator):
    """The draft stand-in on the device, for the full-size workloads: q = softmax((logits + N(0, std)) / T) and one token
    drawn from it per row.  logits_row [B, V] fp32 device tensor, std [B, 1]; torch library calls only."""
    noise = torch.randn(logits_row.shape, generator=generator, device=logits_row.device, dtype=torch.float32) * std
    q = torch.softmax((logits_row + noise) / temperature, dim=-1)
    return q, torch.multinomial(q, 1, generator=generator)[:, 0].to(torch.int32)


def ceil_div(a, b):
    return -(-a // b)


__all__ = ["PAGE_SIZE", "DEFAULT_SEED", "MODELS", "WORKLOADS", "torch_dtype", "weight_shapes", "make_weights",
           "weights_for_oracle", "make_batch", "make_logical_kv", "kv_for_oracle", "round_to_storage",
           "make_sampler_case", "draw_from", "noisy_draft_distribution", "ceil_div", "math"]


def response_lengths(workload, seed=DEFAULT_SEED):
    """Long-tailed synthetic response lengths [B] (int32) of a continuous-rollout workload: log-normal with the
    workload's median and sigma, clipped to [resp_lo, resp_hi]."""
    rng = np.random.default_rng(int(seed) + 23)
    n = workload["B"]
    x = np.exp(rng.normal(np.log(workload["resp_median"]), workload["resp_sigma"], size=n))
    return np.clip(np.rint(x), workload["resp_lo"], workload["resp_hi"]).astype(np.int32)
