"""Pins for the mixture-of-experts feed-forward of the forward oracle.

The paper's large target (Section 3.1: a 235B-parameter model with 22B active) is a top-k routed
mixture of experts; the oracle's reading (softmax over all experts, top-k, renormalise, weighted sum of
SwiGLU experts) is pinned here to things that are not a retyping of it:
  * an independent composition from torch library routines (softmax, topk, gather, einsum, silu);
  * identical experts == that expert's dense feed-forward (weights must sum to one);
  * top_k == n_experts == the full softmax mixture; one expert == dense;
  * the routing is invariant to a constant added to all router logits, and an expert whose router row is
    made dominant receives every row with weight -> 1;
  * whole decoder: a mixture model with identical experts gives the logits of the dense model.
"""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import forward as of


def _experts(rng, E, Fe, d, std=0.3):
    return dict(router=rng.standard_normal((E, d)) / np.sqrt(d) * 3.0, wg=rng.standard_normal((E, Fe, d)) * std,
                wu=rng.standard_normal((E, Fe, d)) * std, wd=rng.standard_normal((E, d, Fe)) * std)


def _torch_moe(h, w, top_k):
    h = torch.from_numpy(h)
    r = F.linear(h, torch.from_numpy(w["router"]))
    prob = F.softmax(r, dim=-1)
    val, idx = torch.topk(prob, top_k, dim=-1)
    val = val / val.sum(-1, keepdim=True)
    wg, wu, wd = (torch.from_numpy(w[n]) for n in ("wg", "wu", "wd"))
    gate = torch.einsum("efd,md->mef", wg, h)
    up = torch.einsum("efd,md->mef", wu, h)
    y_all = torch.einsum("edf,mef->med", wd, F.silu(gate) * up)                  # every expert on every row
    picked = torch.gather(y_all, 1, idx[:, :, None].expand(-1, -1, h.shape[1]))
    return (val[:, :, None] * picked).sum(1).numpy(), idx.numpy(), val.numpy()


def test_against_torch_library_composition():
    rng = np.random.default_rng(0)
    E, Fe, d, M, top_k = 10, 24, 32, 17, 3
    w = _experts(rng, E, Fe, d)
    h = rng.standard_normal((M, d))
    log = []
    got = of.moe_ffn(h, w, top_k, log)
    want, idx, val = _torch_moe(h, w, top_k)
    assert np.max(np.abs(got - want)) < 1e-10 and np.max(np.abs(want)) > 0.1
    experts, weight, prob = log[0]
    assert np.array_equal(experts, idx)                       # most probable first, like topk
    assert np.max(np.abs(weight - val)) < 1e-14
    assert np.max(np.abs(weight.sum(-1) - 1)) < 1e-14 and np.max(np.abs(prob.sum(-1) - 1)) < 1e-14
    assert len({tuple(sorted(r)) for r in experts.tolist()}) > 3          # routing really varies over rows


def test_identical_experts_full_mixture_and_single_expert():
    rng = np.random.default_rng(1)
    E, Fe, d, M = 6, 16, 24, 9
    w = _experts(rng, E, Fe, d)
    h = rng.standard_normal((M, d))
    dense = lambda e: (of.silu(h @ w["wg"][e].T) * (h @ w["wu"][e].T)) @ w["wd"][e].T
    same = dict(w, wg=np.repeat(w["wg"][:1], E, 0), wu=np.repeat(w["wu"][:1], E, 0), wd=np.repeat(w["wd"][:1], E, 0))
    assert np.max(np.abs(of.moe_ffn(h, same, 2) - dense(0))) < 1e-12
    # all experts chosen: the plain softmax mixture
    r = h @ w["router"].T
    p = np.exp(r - r.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    full = sum(p[:, e:e + 1] * dense(e) for e in range(E))
    assert np.max(np.abs(of.moe_ffn(h, w, E) - full)) < 1e-12
    one = {n: w[n][:1] for n in w}
    assert np.max(np.abs(of.moe_ffn(h, one, 1) - dense(0))) < 1e-12


def test_routing_invariances_and_ties():
    rng = np.random.default_rng(2)
    E, Fe, d, M = 8, 8, 16, 11
    w = _experts(rng, E, Fe, d)
    h = rng.standard_normal((M, d))
    e0, w0, _ = of.moe_route(h, w["router"], 3)
    # a constant added to every router logit (a common direction added to every router row) changes nothing
    shift = rng.standard_normal(d)
    e1, w1, _ = of.moe_route(h, w["router"] + shift[None, :], 3)
    assert np.array_equal(e0, e1) and np.max(np.abs(w0 - w1)) < 1e-12
    # an expert made dominant for the rows' mean direction is picked first for rows aligned with it
    hh = np.abs(h)
    boosted = w["router"].copy()
    boosted[5] += 50.0 / d
    e2, w2, _ = of.moe_route(hh, boosted, 3)
    assert np.all(e2[:, 0] == 5) and np.all(w2[:, 0] > 0.9)
    # exact ties go to the lower index, in order
    tie = np.zeros((4, d))
    e3, w3, _ = of.moe_route(h, tie, 2)
    assert np.all(e3 == np.array([0, 1])) and np.allclose(w3, 0.5)


def test_decoder_with_identical_experts_equals_dense_decoder():
    cfg_d = dict(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn_dim=40, vocab=30,
                 rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f64", tied_head=0)
    cfg_m = dict(cfg_d, n_experts=5, top_k=2, expert_ffn_dim=40)
    rng = np.random.default_rng(3)
    d, F_, V = 32, 40, 30
    layers_d, layers_m = [], []
    for _ in range(2):
        base = dict(attn_norm=1 + 0.1 * rng.standard_normal(d), wq=rng.standard_normal((32, d)) * 0.2,
                    wk=rng.standard_normal((16, d)) * 0.2, wv=rng.standard_normal((16, d)) * 0.2,
                    wo=rng.standard_normal((d, 32)) * 0.2, ffn_norm=1 + 0.1 * rng.standard_normal(d))
        wg, wu, wd = rng.standard_normal((F_, d)) * 0.2, rng.standard_normal((F_, d)) * 0.2, rng.standard_normal((d, F_)) * 0.2
        layers_d.append(dict(base, wg=wg, wu=wu, wd=wd))
        layers_m.append(dict(base, wg=np.repeat(wg[None], 5, 0), wu=np.repeat(wu[None], 5, 0), wd=np.repeat(wd[None], 5, 0),
                             router=rng.standard_normal((5, d))))
    common = dict(embed=rng.standard_normal((V, d)), final_norm=np.ones(d), head=rng.standard_normal((V, d)))
    ctx = np.array([3, 0])
    kv = [[(rng.standard_normal((c, 2, 8)), rng.standard_normal((c, 2, 8))) for c in ctx] for _ in range(2)]
    tokens = rng.integers(0, V, size=(2, 3))
    dense, _ = of.verify_forward(cfg_d, dict(common, layers=layers_d), kv, tokens, ctx)
    log = []
    mixed, _ = of.verify_forward(cfg_m, dict(common, layers=layers_m), kv, tokens, ctx, route_log=log)
    assert np.max(np.abs(dense - mixed)) < 1e-10
    assert len(log) == 2 and log[0][0].shape == (6, 2)
