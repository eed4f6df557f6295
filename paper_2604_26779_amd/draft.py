"""Device-memory plumbing for the draft side of a speculation step: k autoregressive passes of a
draft model (a VerifySession of its own: its own weights and paged cache), each followed by
``spec_draft_sample`` and a commit of the fed positions, and the roll-back of the draft's cache
after verification.  Only pointers, strides and call order are handled here.
"""
import torch

from . import binding as sv


class DraftLoop:
    def __init__(self, draft_session, B, k, token_map=None, target_vocab=None):
        """token_map [head_vocab] int32 device tensor + target_vocab: for a draft whose head covers a subset of the target's
        vocabulary (cfg head_vocab): its drafts are written as target ids and q over the target's vocabulary."""
        self.sess, self.B, self.k = draft_session, int(B), int(k)
        self.token_map = token_map
        self.head_vocab = int(draft_session.cfg.get("head_vocab", 0))
        assert (self.head_vocab > 0) == (token_map is not None), "a draft with a reduced head needs its token map (and only such a draft)"
        self.q_width = int(target_vocab) if token_map is not None else draft_session.cfg["vocab"]
        dev = draft_session.device
        self.feed = torch.zeros(B, dtype=torch.int32, device=dev)          # the single token of passes 2..k
        self.ones = torch.ones(B, dtype=torch.int32, device=dev)
        self.zeros = torch.zeros(B, dtype=torch.int32, device=dev)
        self.drafts = torch.zeros((B, k), dtype=torch.int32, device=dev)
        self.new_len = torch.zeros(B, dtype=torch.int32, device=dev)
        self.sample_ws = torch.empty(sv.spec_draft_sample_workspace_bytes(B), dtype=torch.uint8, device=dev)
        # a draft that takes hidden states chains its own: the last row of a pass feeds the next pass
        self.fused = bool(draft_session.cfg.get("fuse_hidden", 0))
        # ... and may take the verifier's states at several depths (features, n * d wide) on the first pass of a step
        self.taps = int(draft_session.cfg.get("fuse_taps", 0)) if self.fused else 0
        d = draft_session.cfg["d_model"]
        self.hid_first = None                                               # [B, P, d], allocated on first use
        self.hid = [torch.zeros((B, 1, d), dtype=torch.float32, device=dev) for _ in range(2)] if self.fused else None

    def run(self, seq_ids, pending, q_out, temperature, seed, step, stream=None, pending_hidden=None):
        """pending [B, P] int32 (tokens the draft's cache lacks; P = 2 in steady state), q_out [B, k, V] fp32;
        pending_hidden [B, P, d] fp32 for a draft with hidden-state input (the verifier's hidden state of the position
        before each pending token; [B, P, n * d] features for a draft with fuse_taps = n).

        Fills self.drafts [B, k] and q_out; the draft's cache grows by P + k - 1 positions."""
        sess, B, k = self.sess, self.B, self.k
        V = self.head_vocab or sess.cfg["vocab"]                      # entries of the draft's logits rows
        W = self.q_width                                              # entries of a q row
        P = pending.shape[1]
        assert q_out.shape == (B, k, W) and q_out.is_contiguous() and pending.is_contiguous()
        if self.fused:
            assert pending_hidden is not None and pending_hidden.is_contiguous()
            if self.hid_first is None or self.hid_first.shape[1] != P:
                self.hid_first = torch.zeros((B, P, sess.cfg["d_model"]), dtype=torch.float32, device=sess.device)
        for i in range(k):
            if i == 0:
                if self.fused:
                    if self.taps:
                        logits = sess.forward(seq_ids, pending, stream, features_in=pending_hidden, hidden_out=self.hid_first)
                    else:
                        logits = sess.forward(seq_ids, pending, stream, hidden_in=pending_hidden, hidden_out=self.hid_first)
                    self.hid[0].copy_(self.hid_first[:, P - 1:P, :])
                else:
                    logits = sess.forward(seq_ids, pending, stream)                      # [B, P, V]
                last = logits.data_ptr() + (P - 1) * V * 4
                stride = P * V
            else:
                if self.fused:
                    logits = sess.forward(seq_ids, self.feed.view(B, 1), stream, hidden_in=self.hid[(i - 1) & 1],
                                          hidden_out=self.hid[i & 1])
                else:
                    logits = sess.forward(seq_ids, self.feed.view(B, 1), stream)        # [B, 1, V]
                last, stride = logits.data_ptr(), V
            if self.token_map is not None:
                sv.spec_draft_sample_mapped(B, V, last, stride, temperature, seed, step, i,
                                            self.drafts.data_ptr() + 4 * i, k, self.feed, 1,
                                            q_out.data_ptr() + 4 * i * W, k * W, self.token_map, W, stream, self.sample_ws)
            else:
                sv.spec_draft_sample(B, V, last, stride, temperature, seed, step, i,
                                     self.drafts.data_ptr() + 4 * i, k, self.feed, 1,
                                     q_out.data_ptr() + 4 * i * V, k * V, stream, self.sample_ws)
            fed = P if i == 0 else 1
            sv.spec_commit_kv(sess.kv, B, fed - 1, seq_ids, self.ones if fed == 2 else self._full(fed - 1), None, None, stream)
        return self.drafts

    def _full(self, n):
        if n == 0:
            return self.zeros
        if n == 1:
            return self.ones
        return torch.full((self.B,), n, dtype=torch.int32, device=self.sess.device)

    def roll_back(self, seq_ids, target_new_ctx_len, stream=None):
        """After the target's commit: keep target_new_ctx_len - 1 positions (never more than cached)."""
        sv.spec_kv_truncate(self.sess.kv, self.B, seq_ids, target_new_ctx_len, -1, self.new_len, stream)
        return self.new_len


class RolloutLoop:
    """Consecutive speculation steps on one stream with no host round trip: draft loop -> verify forward ->
    rejection sampling -> commit -> roll-back of the draft's cache -> next step's inputs.  Only call order and
    buffers are handled here."""

    def __init__(self, target_session, draft_session, B, k, tap_layers=None, token_map=None):
        """tap_layers: for a draft with fuse_taps, the target layers whose output it is fed; token_map: for a draft with a
        reduced head, its entries' ids in the target's vocabulary."""
        self.t, self.B, self.k = target_session, int(B), int(k)
        self.loop = DraftLoop(draft_session, B, k, token_map=token_map, target_vocab=target_session.cfg["vocab"])
        dev = target_session.device
        V = target_session.cfg["vocab"]
        self.tokens = torch.zeros((B, k + 1), dtype=torch.int32, device=dev)
        self.pending = torch.zeros((B, 2), dtype=torch.int32, device=dev)
        self.q = torch.zeros((B, k, V), dtype=torch.float32, device=dev)
        self.fused = self.loop.fused
        self.tap_layers = tuple(int(l) for l in tap_layers) if self.loop.taps else None
        assert not self.loop.taps or len(self.tap_layers) == self.loop.taps
        if self.fused:
            d = target_session.cfg["d_model"] * max(1, self.loop.taps)
            self.hidden_width = d
            self.pending_hidden = torch.zeros((B, 2, d), dtype=torch.float32, device=dev)
            self.target_hidden = torch.zeros((B, k + 1, d), dtype=torch.float32, device=dev)

    def start(self, prev, t0, pending_hidden=None):
        """prev, t0 [B] int32 device tensors: the last input the target has cached and the last emitted token;
        pending_hidden [B, 2, d] for a draft with hidden-state input: the target's hidden states before each of them."""
        self.pending[:, 0] = prev
        self.pending[:, 1] = t0
        self.tokens[:, 0] = t0
        if self.fused:
            self.pending_hidden.copy_(pending_hidden)

    def run(self, seq_ids, n_steps, temperature, seed, step0=0, accept_out=None, tokens_out=None, stream=None):
        """accept_out [n_steps, B] int32, tokens_out [n_steps, B, k+1] int32 (device, optional) receive every
        step's accept lengths and emitted tokens."""
        t, B, k = self.t, self.B, self.k
        V = t.cfg["vocab"]
        buf = t.step_buffers(B, k)
        ws = buf["workspace"]
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + ws.numel() - 256]
        for s in range(n_steps):
            drafts = self.loop.run(seq_ids, self.pending, self.q, temperature, seed, step0 + s, stream,
                                   self.pending_hidden if self.fused else None)
            self.tokens[:, 1:] = drafts
            acc = accept_out[s] if accept_out is not None else buf["accept_len"]
            out = tokens_out[s] if tokens_out is not None else buf["out_tokens"]
            if self.tap_layers:
                sv.spec_verify_forward_taps(t.model, t.kv, B, k, seq_ids, self.tokens, buf["logits"], self.tap_layers,
                                            self.target_hidden, ws, stream)
            elif self.fused:
                sv.spec_verify_forward_hidden(t.model, t.kv, B, k, seq_ids, self.tokens, None, buf["logits"], self.target_hidden,
                                              ws, stream)
            else:
                sv.spec_verify_forward(t.model, t.kv, B, k, seq_ids, self.tokens, buf["logits"], ws, stream)
            sv.spec_reject_sample(B, k, V, buf["logits"], self.q, drafts, temperature, seed, step0 + s, acc, out, None,
                                  buf["sample_ws"], stream)
            sv.spec_commit_kv(t.kv, B, k, seq_ids, acc, buf["new_ctx_len"], None, stream)
            self.loop.roll_back(seq_ids, buf["new_ctx_len"], stream)
            sv.spec_next_step_inputs(B, k, self.tokens, out, acc, self.pending, stream)
            if self.fused:
                sv.spec_next_step_hidden(B, k, self.hidden_width, self.target_hidden, acc, self.pending_hidden, stream)


class NgramRollout:
    """Consecutive speculation steps with the model-free n-gram drafter, on one stream with no host round trip:
    drafts from the histories -> verify forward -> rejection sampling with point-mass drafts -> commit -> history
    update.  Only call order and buffers are handled here; histories are rows of a caller-owned [n_rows, cap]
    int32 device array, batch entry b using row seq_ids[b]."""

    def __init__(self, target_session, B, k, n_max=3, n_min=1):
        self.t, self.B, self.k, self.n_max, self.n_min = target_session, int(B), int(k), int(n_max), int(n_min)
        dev = target_session.device
        self.tokens = torch.zeros((B, k + 1), dtype=torch.int32, device=dev)
        self.drafts = torch.zeros((B, k), dtype=torch.int32, device=dev)
        self.n_drafted = torch.zeros(B, dtype=torch.int32, device=dev)

    def run(self, seq_ids, hist, hist_len, n_steps, temperature, seed, step0=0, accept_out=None, tokens_out=None, stream=None):
        t, B, k = self.t, self.B, self.k
        V = t.cfg["vocab"]
        buf = t.step_buffers(B, k)
        ws = buf["workspace"]
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + ws.numel() - 256]
        for s in range(n_steps):
            sv.spec_ngram_draft(B, k, self.n_max, self.n_min, hist, hist_len, seq_ids, self.tokens, self.n_drafted, stream)
            self.drafts.copy_(self.tokens[:, 1:])
            acc = accept_out[s] if accept_out is not None else buf["accept_len"]
            out = tokens_out[s] if tokens_out is not None else buf["out_tokens"]
            sv.spec_verify_forward(t.model, t.kv, B, k, seq_ids, self.tokens, buf["logits"], ws, stream)
            sv.spec_reject_sample(B, k, V, buf["logits"], None, self.drafts, temperature, seed, step0 + s, acc, out, None,
                                  buf["sample_ws"], stream)
            sv.spec_commit_kv(t.kv, B, k, seq_ids, acc, buf["new_ctx_len"], None, stream)
            sv.spec_ngram_append(B, k, hist, hist_len, seq_ids, out, acc, stream)


class ContinuousRollout:
    """A rollout over B batch slots that outlives its sequences: n-gram drafts -> verify forward -> rejection
    sampling -> commit -> history update -> next inputs -> slot bookkeeping (finished sequences retire, waiting ones
    take their slot, the rest idle) -> release of the retired caches; one stream, no host round trip.  Sequence ids
    index every per-sequence array (histories, lengths, targets, first tokens); waiting sequences are already
    prefilled.  Only call order and buffers are handled here."""

    def __init__(self, target_session, B, k, slot_seq, target_len, queue, first_token, n_max=3, n_min=1):
        self.t, self.B, self.k, self.n_max, self.n_min = target_session, int(B), int(k), int(n_max), int(n_min)
        dev = target_session.device
        n_seqs = int(target_len.shape[0])
        self.slot_seq = slot_seq.to(dev, torch.int32).clone()
        self.target_len = target_len.to(dev, torch.int32)
        self.first_token = first_token.to(dev, torch.int32)
        self.queue = queue.to(dev, torch.int32) if queue is not None and len(queue) else None
        self.active = torch.ones(B, dtype=torch.int32, device=dev)
        self.gen_len = torch.zeros(n_seqs, dtype=torch.int32, device=dev)
        self.queue_head = torch.zeros(1, dtype=torch.int32, device=dev)
        self.produced = torch.zeros(1, dtype=torch.int64, device=dev)
        self.tokens = torch.zeros((B, k + 1), dtype=torch.int32, device=dev)
        self.drafts = torch.zeros((B, k), dtype=torch.int32, device=dev)
        self.release_seq = torch.zeros(B, dtype=torch.int32, device=dev)
        self.keep_len = torch.zeros(B, dtype=torch.int32, device=dev)
        self.n_live = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scratch = torch.zeros(B * (k + 3), dtype=torch.int32, device=dev)
        self.B_cur = int(B)                    # slots a step covers: all of them until compact() shrinks the batch

    def compact(self, granule=8, stream=None):
        """Move the live slots to the front and shrink the batch to them (rounded up to `granule` slots; the idle
        slots behind keep riding along).  Reads the live count back: a host synchronisation.  Returns the count."""
        sv.spec_rollout_compact(self.B_cur, self.k, self.slot_seq, self.active, self.tokens, self.n_live, self.scratch, stream)
        n = int(self.n_live.item())
        self.B_cur = max(granule, min(self.B_cur, -(-n // granule) * granule)) if n > 0 else min(self.B_cur, granule)
        return n

    def run(self, hist, hist_len, n_steps, temperature, seed, step0=0, live_out=None, stream=None):
        """live_out [n_steps] int32 (device, optional) receives the number of live slots after every step."""
        t, B, k = self.t, self.B_cur, self.k
        V = t.cfg["vocab"]
        buf = t.step_buffers(B, k)
        ws = buf["workspace"]
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + ws.numel() - 256]
        acc, out = buf["accept_len"], buf["out_tokens"]
        drafts = self.drafts[:B]               # the first B rows of contiguous [slots, ...] arrays are contiguous
        for s in range(n_steps):
            sv.spec_ngram_draft(B, k, self.n_max, self.n_min, hist, hist_len, self.slot_seq, self.tokens, None, stream)
            drafts.copy_(self.tokens[:B, 1:])
            sv.spec_verify_forward(t.model, t.kv, B, k, self.slot_seq, self.tokens, buf["logits"], ws, stream)
            sv.spec_reject_sample(B, k, V, buf["logits"], None, drafts, temperature, seed, step0 + s, acc, out, None,
                                  buf["sample_ws"], stream)
            sv.spec_commit_kv(t.kv, B, k, self.slot_seq, acc, buf["new_ctx_len"], None, stream)
            sv.spec_ngram_append(B, k, hist, hist_len, self.slot_seq, out, acc, stream)
            sv.spec_rollout_retire(B, k, self.slot_seq, self.active, acc, self.gen_len, self.target_len, self.queue,
                                   self.queue_head, self.first_token, self.tokens, self.release_seq, self.keep_len,
                                   self.produced, stream)
            sv.spec_kv_truncate(t.kv, B, self.release_seq, self.keep_len, 0, None, stream)
            if live_out is not None:
                live_out[s] = self.active[:B].sum()


class ContinuousPairRollout:
    """The continuous rollout with a draft model instead of the n-gram drafter: draft loop -> verify forward -> rejection
    sampling -> commit -> roll-back of the draft's cache -> next inputs and pending pairs -> slot bookkeeping (finished
    sequences retire, waiting ones take their slot together with their own pending pair, the rest idle) -> release of the
    retired sequences' pages in both caches; one stream, no host round trip.  Sequence ids index every per-sequence
    array; waiting sequences are prefilled in both caches (the draft's one position behind the verifier's).  Only call
    order and buffers are handled here."""

    def __init__(self, target_session, draft_session, B, k, slot_seq, target_len, queue, prev_token, first_token, seq_hidden=None,
                 tap_layers=None, token_map=None):
        """seq_hidden [n_seqs, 2, d] fp32: for a draft with hidden-state input, every sequence's own pair of verifier
        hidden states (the positions before its last prompt token and before its first input); for a draft with
        fuse_taps = n they are features, [n_seqs, 2, n * d], and tap_layers names the n target layers."""
        self.t, self.d, self.B, self.k = target_session, draft_session, int(B), int(k)
        dev = target_session.device
        n_seqs = int(target_len.shape[0])
        self.loop = DraftLoop(draft_session, B, k, token_map=token_map, target_vocab=target_session.cfg["vocab"])
        self.fused = self.loop.fused
        assert not self.fused or seq_hidden is not None, "a draft with hidden-state input needs every sequence's own pair of hidden states"
        self.tap_layers = tuple(int(l) for l in tap_layers) if self.loop.taps else None
        assert not self.loop.taps or len(self.tap_layers) == self.loop.taps
        self.slot_seq = slot_seq.to(dev, torch.int32).clone()
        self.slot_seq_before = self.slot_seq.clone()
        self.target_len = target_len.to(dev, torch.int32)
        self.prev_token = prev_token.to(dev, torch.int32)
        self.first_token = first_token.to(dev, torch.int32)
        self.queue = queue.to(dev, torch.int32) if queue is not None and len(queue) else None
        self.active = torch.ones(B, dtype=torch.int32, device=dev)
        self.gen_len = torch.zeros(n_seqs, dtype=torch.int32, device=dev)
        self.queue_head = torch.zeros(1, dtype=torch.int32, device=dev)
        self.produced = torch.zeros(1, dtype=torch.int64, device=dev)
        self.tokens = torch.zeros((B, k + 1), dtype=torch.int32, device=dev)
        self.pending = torch.zeros((B, 2), dtype=torch.int32, device=dev)
        self.q = torch.zeros((B, k, target_session.cfg["vocab"]), dtype=torch.float32, device=dev)
        self.release_seq = torch.zeros(B, dtype=torch.int32, device=dev)
        self.keep_len = torch.zeros(B, dtype=torch.int32, device=dev)
        idx = self.slot_seq.long()
        self.tokens[:, 0] = self.first_token[idx]
        self.pending[:, 0] = self.prev_token[idx]
        self.pending[:, 1] = self.first_token[idx]
        if self.fused:
            d = target_session.cfg["d_model"] * max(1, self.loop.taps)
            self.hidden_width = d
            self.seq_hidden = seq_hidden.to(dev, torch.float32).contiguous()
            self.pending_hidden = self.seq_hidden[idx].contiguous()
            self.target_hidden = torch.zeros((B, k + 1, d), dtype=torch.float32, device=dev)

    def run(self, n_steps, temperature, seed, step0=0, live_out=None, accept_out=None, stream=None):
        """live_out [n_steps] int32, accept_out [n_steps, B] int32 (device, optional): live slots after and accept
        lengths of every step."""
        t, B, k = self.t, self.B, self.k
        V = t.cfg["vocab"]
        buf = t.step_buffers(B, k)
        ws = buf["workspace"]
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + ws.numel() - 256]
        out = buf["out_tokens"]
        for s in range(n_steps):
            acc = accept_out[s] if accept_out is not None else buf["accept_len"]
            drafts = self.loop.run(self.slot_seq, self.pending, self.q, temperature, seed, step0 + s, stream,
                                   self.pending_hidden if self.fused else None)
            self.tokens[:, 1:] = drafts
            if self.tap_layers:
                sv.spec_verify_forward_taps(t.model, t.kv, B, k, self.slot_seq, self.tokens, buf["logits"], self.tap_layers,
                                            self.target_hidden, ws, stream)
            elif self.fused:
                sv.spec_verify_forward_hidden(t.model, t.kv, B, k, self.slot_seq, self.tokens, None, buf["logits"], self.target_hidden,
                                              ws, stream)
            else:
                sv.spec_verify_forward(t.model, t.kv, B, k, self.slot_seq, self.tokens, buf["logits"], ws, stream)
            sv.spec_reject_sample(B, k, V, buf["logits"], self.q, drafts, temperature, seed, step0 + s, acc, out, None,
                                  buf["sample_ws"], stream)
            sv.spec_commit_kv(t.kv, B, k, self.slot_seq, acc, buf["new_ctx_len"], None, stream)
            self.loop.roll_back(self.slot_seq, buf["new_ctx_len"], stream)
            sv.spec_next_step_inputs(B, k, self.tokens, out, acc, self.pending, stream)
            if self.fused:
                sv.spec_next_step_hidden(B, k, self.hidden_width, self.target_hidden, acc, self.pending_hidden, stream)
            self.slot_seq_before.copy_(self.slot_seq)
            sv.spec_rollout_retire(B, k, self.slot_seq, self.active, acc, self.gen_len, self.target_len, self.queue,
                                   self.queue_head, self.first_token, self.tokens, self.release_seq, self.keep_len,
                                   self.produced, stream)
            sv.spec_rollout_pending(B, self.slot_seq_before, self.slot_seq, self.active, self.prev_token, self.first_token,
                                    self.pending, stream)
            if self.fused:
                sv.spec_rollout_pending_hidden(B, self.slot_seq_before, self.slot_seq, self.active, self.seq_hidden,
                                               self.pending_hidden, stream)
            sv.spec_kv_truncate(t.kv, B, self.release_seq, self.keep_len, 0, None, stream)
            sv.spec_kv_truncate(self.d.kv, B, self.release_seq, self.keep_len, 0, None, stream)
            if live_out is not None:
                live_out[s] = self.active.sum()
