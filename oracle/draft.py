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


def draft_loop(cfg, weights, kv_ctx, pending, ctx_len, k, temperature, seed, step):
    """pending [B, P] int tokens not yet in the draft's cache, ctx_len [B] its cached length.

    Returns (drafts [B, k] int32, q [B, k, V] fp32, kv_ctx grown by the fed positions, new_len [B],
    keys [B, k, 2] = winning and runner-up key of every draw).
    """
    pending = np.asarray(pending)
    B = pending.shape[0]
    ctx_len = np.asarray(ctx_len, dtype=np.int64).copy()
    kv = [[(np.asarray(K, dtype=np.float64), np.asarray(V, dtype=np.float64)) for (K, V) in per_seq] for per_seq in kv_ctx]
    drafts = np.zeros((B, k), dtype=np.int32)
    q = np.zeros((B, k, cfg["vocab"]), dtype=np.float32)
    keys = np.zeros((B, k, 2), dtype=np.float64)
    feed = pending
    for i in range(k):
        logits, new_kv = _forward.verify_forward(cfg, weights, kv, feed, ctx_len)
        for layer in range(cfg["n_layers"]):
            for b in range(B):
                K, V = kv[layer][b]
                kv[layer][b] = (np.concatenate([K, new_kv[layer][0][b]]), np.concatenate([V, new_kv[layer][1][b]]))
        ctx_len += feed.shape[1]
        x, qi, keys[:, i, :] = _sampler.draft_sample(logits[:, -1, :].astype(np.float32), temperature, seed, step, i, debug=True)
        drafts[:, i] = x
        q[:, i, :] = qi
        feed = x.reshape(B, 1)
    return drafts, q, kv, ctx_len, keys
