"""Build a full verify-step workload on the GPU from the seeded generators (used by bench.py and
by the full-size parity tests).  Plumbing only: tensors are drawn, moved and indexed with torch;
the draft stand-in (q = softmax((logits + noise) / T), x ~ q) is input generation, and the target
logits it needs come from running the library's own forward pass during set-up.
"""
import numpy as np
import torch

import synth_inputs as si

from . import binding as sv
from .session import VerifySession


def fill_pool(sess, cfg, g, seed):
    """Synthetic cached context: every slot of the pool ~ N(0,1) in the storage type; an 8-bit cache gets the codes of
    N(0, KV8_NOMINAL) entries (the library's cast) under the synthetic scales, which are installed and returned."""
    chunk = 1 << 28
    flat = sess.pool
    if not sess.kv8:
        for at in range(0, flat.numel(), chunk):
            flat[at:at + chunk].normal_(generator=g)
        return None
    for at in range(0, flat.numel(), chunk):
        n = min(chunk, flat.numel() - at)
        draw = torch.empty(n, dtype=torch.bfloat16, device=flat.device).normal_(0.0, si.KV8_NOMINAL, generator=g)
        flat[at:at + n] = draw.to(torch.float8_e4m3fn).view(torch.uint8)
    scales = si.kv_scales(cfg, seed=seed)
    sess.set_scales(*scales)
    return scales


class DeviceWorkload:
    def __init__(self, workload_name, seed=si.DEFAULT_SEED, shuffle_pages=True, device="cuda", extra_pages=None,
                 drop_canonical=True):
        self.name = workload_name
        self.wl = dict(si.WORKLOADS[workload_name])
        self.cfg = si.MODELS[self.wl["model"]]
        self.seed = seed
        self.device = torch.device(device)
        B, k = self.wl["B"], self.wl["k"]
        self.B, self.k = B, k
        self.batch = si.make_batch(self.wl, seed=seed, shuffle_pages=shuffle_pages)
        self.ctx_len = self.batch["ctx_len"]
        weights = si.make_weights(self.cfg, seed=seed, device=device)
        n_pages = self.batch["n_pages"] + (extra_pages if extra_pages is not None else 4 * B + 64)
        self.sess = VerifySession(self.cfg, weights, max_seqs=B, max_ctx_len=int(self.ctx_len.max()) + 256,
                                  n_pages=n_pages, layer_alias_mod=self.wl.get("layer_alias_mod", 0), device=device)
        if drop_canonical and self.cfg["dtype"] == "bf16":
            # the library re-tiled the matrices into its own buffer; keep only what it still reads
            keep = {"embed"} | {n for n in weights if n.endswith("norm")}
            self.weights = {n: t for n, t in weights.items() if n in keep}
            self.sess.weights = list(self.weights.values())
            del weights
            torch.cuda.empty_cache()
        else:
            self.weights = weights
        # synthetic cached context: every slot of the pool ~ N(0,1) in the storage type
        g = torch.Generator(device=device)
        g.manual_seed(int(seed) + 2)
        self.kv_scales = fill_pool(self.sess, self.cfg, g, seed)
        self.seq_ids = torch.arange(B, dtype=torch.int32, device=device)
        for b in range(B):
            self.sess.assign(b, int(self.ctx_len[b]), self.batch["page_lists"][b])
        self.tokens = torch.zeros((B, k + 1), dtype=torch.int32, device=device)
        self.tokens[:, 0] = torch.from_numpy(self.batch["tokens0"]).to(device)
        self.q = torch.zeros((B, k, self.cfg["vocab"]), dtype=torch.float32, device=device)
        self.snapshot = torch.empty(sv.spec_kv_state_bytes(self.sess.kv), dtype=torch.uint8, device=device)
        sv.spec_kv_snapshot(self.sess.kv, self.snapshot)

    def make_drafts(self):
        """Fill tokens[:, 1:] and q: k passes of the target, each fixing the next draft token."""
        g = torch.Generator(device=self.device)
        g.manual_seed(int(self.seed) + 5)
        T = self.wl["temperature"]
        std = (self.wl["noise_std"] * torch.from_numpy(self.batch["noise_scale"]).to(self.device, torch.float32))[:, None]
        for i in range(1, self.k + 1):
            logits = self.sess.forward(self.seq_ids, self.tokens)
            self.q[:, i - 1, :], self.tokens[:, i] = si.device_draft_step(logits[:, i - 1, :], std, T, g)
        torch.cuda.synchronize()

    def logical_kv(self, layer, b):
        """(K, V) [ctx_len[b], Hkv, dh] of sequence b as the cache holds them (device tensors)."""
        K, V = self.sess.read_logical_kv(layer, self.batch["page_lists"][b], int(self.ctx_len[b]))
        if self.sess.kv8:                                 # bytes -> the library's 8-bit float type (codes)
            K, V = K.view(torch.float8_e4m3fn), V.view(torch.float8_e4m3fn)
        return K, V

    def restore(self, stream=None):
        sv.spec_kv_restore(self.sess.kv, self.snapshot, stream)

    def close(self):
        self.sess.close()


def algorithmic_bytes(cfg, ctx_len, B, k):
    """Bytes one verify step must move, per kernel class (weights once per step, cached K/V once
    per sequence, logits written once and read by the sampler)."""
    L, D, F, V = cfg["n_layers"], cfg["d_model"], cfg["ffn_dim"], cfg["vocab"]
    nq, nkv = cfg["n_q_heads"] * cfg["head_dim"], cfg["n_kv_heads"] * cfg["head_dim"]
    eb = 2 if cfg["dtype"] == "bf16" else 4
    kvb = 1 if cfg.get("kv_dtype") == "fp8_e4m3" else eb
    web = 1 if cfg.get("w_dtype") == "fp8_e4m3" else eb
    layer_w = (nq + 2 * nkv) * D + D * nq + 2 * F * D + D * F
    if cfg.get("n_experts", 0) > 0:          # every expert's matrices are touched once the batch is a few dozen rows
        E, Fe = cfg["n_experts"], cfg["expert_ffn_dim"]
        layer_w = (nq + 2 * nkv) * D + D * nq + E * 3 * Fe * D + E * D
    head_w = V * D
    active_w = layer_w                         # matrix entries one input row multiplies with, per layer
    if cfg.get("n_experts", 0) > 0:
        active_w = (nq + 2 * nkv) * D + D * nq + cfg["top_k"] * 3 * cfg["expert_ffn_dim"] * D + cfg["n_experts"] * D
    tokens = int(np.sum(ctx_len)) + B * (k + 1)
    return dict(
        gemm_flops=2.0 * (L * active_w + head_w) * B * (k + 1),
        gemm=(L * layer_w + head_w) * web,
        gemm_layers=L * layer_w * web,
        gemm_head=head_w * web,
        attn=tokens * 2 * nkv * kvb * L,
        sampler=B * (k + 1 + 2) * V * 4,
        logits_write=B * (k + 1) * V * 4,
    )


class DraftPairWorkload(DeviceWorkload):
    """A target workload plus a single-layer draft model with a cache of its own that is one position
    behind the target's (the draft's first pass of a step feeds the previous input and the last emitted
    token together).  Drafts and q come from the draft loop itself, not from make_drafts."""

    def __init__(self, workload_name, seed=si.DEFAULT_SEED, device="cuda"):
        super().__init__(workload_name, seed=seed, device=device)
        from .draft import DraftLoop
        self.draft_cfg = si.MODELS[self.wl["draft_model"]]
        B, k = self.B, self.k
        dweights = si.make_weights(self.draft_cfg, seed=seed + 17, device=device)
        dctx = self.ctx_len - 1
        step_pages = [-(-(int(c) + k + 2) // si.PAGE_SIZE) for c in dctx]
        n_pages = sum(step_pages) + 8 * B + 64          # room for a few consecutive steps of a rollout
        self.dsess = VerifySession(self.draft_cfg, dweights, max_seqs=B, max_ctx_len=int(dctx.max()) + 256, n_pages=n_pages,
                                   device=device)
        keep = {"embed"} | {n for n in dweights if n.endswith("norm")}
        if self.draft_cfg["dtype"] == "bf16":
            self.dsess.weights = [t for n, t in dweights.items() if n in keep]
        del dweights
        torch.cuda.empty_cache()
        g = torch.Generator(device=device)
        g.manual_seed(int(seed) + 19)
        self.draft_kv_scales = fill_pool(self.dsess, self.draft_cfg, g, seed + 17)
        rng = np.random.Generator(np.random.Philox(int(seed) + 23))
        order = rng.permutation(n_pages)
        at = 0
        for b in range(B):
            need = -(-int(dctx[b]) // si.PAGE_SIZE)
            self.dsess.assign(b, int(dctx[b]), [int(p) for p in order[at:at + need]])
            at += need
        prev = torch.from_numpy(rng.integers(0, self.cfg["vocab"], size=B).astype(np.int32)).to(device)
        self.pending = torch.stack([prev, self.tokens[:, 0]], dim=1).contiguous()
        # a draft with a reduced head: which target tokens its entries are
        self.token_map = None
        if self.draft_cfg.get("head_vocab", 0):
            self.token_map = torch.from_numpy(si.make_token_map(self.draft_cfg, seed=seed + 29)).to(device)
        self.loop = DraftLoop(self.dsess, B, k, token_map=self.token_map, target_vocab=self.cfg["vocab"])
        # a draft with hidden-state input: the target's hidden states before the two pending tokens (synthetic)
        self.pending_hidden = None
        self.tap_layers = tuple(self.wl["tap_layers"]) if self.draft_cfg.get("fuse_taps", 0) else None
        if self.draft_cfg.get("fuse_hidden", 0):
            width = self.cfg["d_model"] * max(1, int(self.draft_cfg.get("fuse_taps", 0)))     # features: several states side by side
            self.pending_hidden = torch.randn((B, 2, width), generator=g, device=device, dtype=torch.float32)
            self.target_hidden = torch.zeros((B, k + 1, width), dtype=torch.float32, device=device)
        self.dsnapshot = torch.empty(sv.spec_kv_state_bytes(self.dsess.kv), dtype=torch.uint8, device=device)
        sv.spec_kv_snapshot(self.dsess.kv, self.dsnapshot)

    def restore(self, stream=None):
        super().restore(stream)
        sv.spec_kv_restore(self.dsess.kv, self.dsnapshot, stream)

    def close(self):
        self.dsess.close()
        super().close()
