"""Device-memory plumbing around the C ABI: allocate the buffers a verify step needs with torch,
move cache contents between the logical (per sequence) and the paged view by indexing, and call
the three entry points in order.  No arithmetic of the method happens here.
"""
import numpy as np
import torch

from . import binding as sv


class VerifySession:
    """One model + one paged KV cache on the current GPU."""

    def __init__(self, cfg, weights, max_seqs, max_ctx_len, n_pages, layer_alias_mod=0, device="cuda"):
        self.cfg = dict(cfg)
        self.device = torch.device(device)
        self.weights = list(weights.values()) if isinstance(weights, dict) else list(weights)
        self.model = sv.spec_model_create(self.cfg, self.weights)
        self.max_seqs, self.n_pages, self.alias = int(max_seqs), int(n_pages), int(layer_alias_mod)
        self.dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[cfg["dtype"]]
        self.kv8 = cfg.get("kv_dtype") == "fp8_e4m3"
        if self.kv8:                       # 8-bit cache: the pool holds E4M3 codes, moved around as bytes
            self.dtype = torch.uint8
        nbytes = sv.spec_kv_pool_bytes(self.model, self.n_pages, self.alias)
        self.pool = torch.empty(nbytes // self.dtype.itemsize, dtype=self.dtype, device=self.device)
        self.kv = sv.spec_kv_alloc(self.model, self.max_seqs, int(max_ctx_len), self.n_pages, self.pool, self.alias)
        self.k_scale = self.v_scale = None
        P, dh = sv.SPEC_PAGE_SIZE, cfg["head_dim"]
        # in-block element order, asked from the library
        self.perm = [torch.tensor([sv.spec_kv_block_offset(self.kv, is_v, t, c) for t in range(P) for c in range(dh)],
                                  dtype=torch.long, device=self.device) for is_v in (0, 1)]
        self._bufs = {}

    def set_scales(self, k_scale, v_scale):
        """8-bit cache: fp32 scales [n_layers, n_kv_heads] for keys and values (kept alive here)."""
        self.k_scale = torch.as_tensor(k_scale, dtype=torch.float32).to(self.device).contiguous()
        self.v_scale = torch.as_tensor(v_scale, dtype=torch.float32).to(self.device).contiguous()
        sv.spec_kv_set_scales(self.kv, self.k_scale, self.v_scale)

    def close(self):
        if self.kv is not None:
            sv.spec_kv_free(self.kv)
            self.kv = None
        if self.model is not None:
            sv.spec_model_destroy(self.model)
            self.model = None

    # ------------------------------------------------------------------ cache contents (plain indexing)
    def pool_view(self):
        """[layer_pool, page, K|V, kv_head, PAGE*head_dim] view of the pool."""
        pools = self.cfg["n_layers"] if self.alias == 0 else min(self.alias, self.cfg["n_layers"])
        return self.pool.view(pools, self.n_pages, 2, self.cfg["n_kv_heads"], sv.SPEC_PAGE_SIZE * self.cfg["head_dim"])

    def write_logical_kv(self, layer, page_ids, K, V):
        """K, V [n_tokens, Hkv, dh] -> the sequence's pages of `layer` (tokens beyond n_tokens zero-filled).
        8-bit cache: K, V are the codes (uint8, or float8_e4m3fn tensors whose bytes are taken)."""
        P, dh, Hkv = sv.SPEC_PAGE_SIZE, self.cfg["head_dim"], self.cfg["n_kv_heads"]
        n_tok = K.shape[0]
        npg = -(-n_tok // P)
        if npg == 0:
            return
        pages = torch.as_tensor(list(page_ids)[:npg], dtype=torch.long, device=self.device)
        lp = layer if self.alias == 0 else layer % self.alias
        view = self.pool_view()
        for is_v, src in ((0, K), (1, V)):
            pad = torch.zeros((npg * P, Hkv, dh), dtype=self.dtype, device=self.device)
            pad[:n_tok] = src.view(torch.uint8).to(self.device) if self.kv8 else src.to(self.device, self.dtype)
            blocks = pad.view(npg, P, Hkv, dh).permute(0, 2, 1, 3).reshape(npg, Hkv, P * dh)
            phys = torch.empty_like(blocks)
            phys[:, :, self.perm[is_v]] = blocks
            view[lp, pages, is_v] = phys

    def read_logical_kv(self, layer, page_ids, n_tokens):
        """Inverse of write_logical_kv: (K, V) [n_tokens, Hkv, dh] of a sequence."""
        P, dh, Hkv = sv.SPEC_PAGE_SIZE, self.cfg["head_dim"], self.cfg["n_kv_heads"]
        npg = -(-n_tokens // P)
        pages = torch.as_tensor(list(page_ids)[:npg], dtype=torch.long, device=self.device)
        lp = layer if self.alias == 0 else layer % self.alias
        view = self.pool_view()
        out = []
        for is_v in (0, 1):
            phys = view[lp, pages, is_v]                                   # [npg, Hkv, P*dh]
            blocks = phys[:, :, self.perm[is_v]].view(npg, Hkv, P, dh).permute(0, 2, 1, 3).reshape(npg * P, Hkv, dh)
            out.append(blocks[:n_tokens].clone())
        return out[0], out[1]

    def assign(self, seq, ctx_len, page_ids):
        sv.spec_kv_seq_assign(self.kv, int(seq), int(ctx_len), page_ids)

    def state(self):
        return sv.spec_kv_get_state(self.kv, self.max_seqs, self.n_pages)

    # ------------------------------------------------------------------ the step
    def step_buffers(self, B, k):
        key = (B, k)
        if key not in self._bufs:
            V, dev = self.cfg.get("head_vocab", 0) or self.cfg["vocab"], self.device      # entries of a logits row
            ws_bytes = sv.spec_verify_workspace_bytes(self.model, self.kv, B, k)
            if ws_bytes == 0:
                raise ValueError("spec_verify_workspace_bytes rejected B=%d k=%d" % (B, k))
            self._bufs[key] = dict(
                logits=torch.empty((B, k + 1, V), dtype=torch.float32, device=dev),
                workspace=torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev),
                sample_ws=torch.empty(sv.spec_sample_workspace_bytes(B, k), dtype=torch.uint8, device=dev),
                accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                out_tokens=torch.empty((B, k + 1), dtype=torch.int32, device=dev),
                dbg=torch.empty((B, max(k, 1), 3), dtype=torch.float32, device=dev),
                new_ctx_len=torch.empty(B, dtype=torch.int32, device=dev),
                commit_slots=torch.empty((B, k + 1), dtype=torch.int32, device=dev),
            )
        return self._bufs[key]

    def forward(self, seq_ids, tokens, stream=None, hidden_in=None, hidden_out=None, features_in=None, tap_layers=None,
                taps_out=None):
        """seq_ids [B] int32, tokens [B, k+1] int32 device tensors -> logits [B, k+1, V] (device, fp32).
        hidden_in / hidden_out [B, k+1, d] fp32: hidden-state input of a fuse_hidden model / hidden states out;
        features_in [B, k+1, n*d]: the same input as multi-layer features (a fuse_taps model);
        tap_layers + taps_out [B, k+1, n*d]: the residual stream after those layers, side by side."""
        B, T = tokens.shape
        buf = self.step_buffers(B, T - 1)
        ws = buf["workspace"]
        off = (-ws.data_ptr()) % 256
        if features_in is not None:
            sv.spec_verify_forward_features(self.model, self.kv, B, T - 1, seq_ids, tokens, features_in, buf["logits"], hidden_out,
                                            ws[off:off + ws.numel() - 256], stream)
        elif tap_layers is not None:
            sv.spec_verify_forward_taps(self.model, self.kv, B, T - 1, seq_ids, tokens, buf["logits"], tap_layers, taps_out,
                                        ws[off:off + ws.numel() - 256], stream)
        elif hidden_in is None and hidden_out is None:
            sv.spec_verify_forward(self.model, self.kv, B, T - 1, seq_ids, tokens, buf["logits"], ws[off:off + ws.numel() - 256],
                                   stream)
        else:
            sv.spec_verify_forward_hidden(self.model, self.kv, B, T - 1, seq_ids, tokens, hidden_in, buf["logits"], hidden_out,
                                          ws[off:off + ws.numel() - 256], stream)
        return buf["logits"]

    def sample(self, logits, q, draft, temperature, seed, step, stream=None, debug=True):
        B, T, V = logits.shape
        buf = self.step_buffers(B, T - 1)
        sv.spec_reject_sample(B, T - 1, V, logits, q, draft, temperature, seed, step, buf["accept_len"],
                              buf["out_tokens"], buf["dbg"] if debug else None, buf["sample_ws"], stream)
        return buf["accept_len"], buf["out_tokens"]

    def commit(self, seq_ids, accept_len, k, stream=None):
        B = seq_ids.shape[0]
        buf = self.step_buffers(B, k)
        sv.spec_commit_kv(self.kv, B, k, seq_ids, accept_len, buf["new_ctx_len"], buf["commit_slots"], stream)
        return buf["new_ctx_len"], buf["commit_slots"]

    def step(self, seq_ids, tokens, q, draft, temperature, seed, step, stream=None, debug=False):
        """The whole hot path: forward -> rejection sampling -> commit, one stream, no host sync."""
        logits = self.forward(seq_ids, tokens, stream)
        accept_len, out_tokens = self.sample(logits, q, draft, temperature, seed, step, stream, debug)
        self.commit(seq_ids, accept_len, tokens.shape[1] - 1, stream)
        return logits, accept_len, out_tokens
