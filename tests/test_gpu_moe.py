"""GPU parity of the mixture-of-experts verify forward against the CPU oracle.

The router's top-k choice is an integer decided by floating point: where the oracle's own margin between
the last chosen and the first rejected expert (difference of router logits) is below 2e-3 in some layer,
the kernels' bf16-pair arithmetic may legitimately choose the other expert, and every later row of that
sequence (which attends to the affected position) changes with it.  Such rows are counted, reported and
exempted; all other rows must meet the bf16 logits tolerance (2e-2 abs + 1e-2 rel).  The exempted rows depend on the
oracle and the inputs alone; the seeds below are ones for which they stay at or below a tenth of the rows.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import forward as of
from tests.helpers import random_norm_gains

pytestmark = pytest.mark.gpu

MARGIN = 2e-3


def _run(cfg, ctx_list, k, seed):
    from paper_2604_26779_amd.session import VerifySession
    B = len(ctx_list)
    weights = random_norm_gains(si.make_weights(cfg, seed=seed), seed)
    w_or = si.weights_for_oracle(cfg, weights)
    ctx_len = np.array(ctx_list, dtype=np.int64)
    kv = si.make_logical_kv(cfg, ctx_len, seed=seed)
    kv8 = cfg.get("kv_dtype") == "fp8_e4m3"               # 8-bit cache: codes under the synthetic scales
    scales = si.kv_scales(cfg, seed=seed) if kv8 else None
    kv_or = si.kv_for_oracle(kv)
    if kv8:
        from oracle import fp8
        kv_or = fp8.cache_values(kv_or, scales)
    rng = np.random.default_rng(seed)
    n_pages = sum(-(-(int(c) + k + 1) // si.PAGE_SIZE) for c in ctx_len) + 16
    order = rng.permutation(n_pages)
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=B, max_ctx_len=int(ctx_len.max()) + 64,
                         n_pages=n_pages)
    sess.pool.fill_(0x7F if kv8 else float("nan"))
    if kv8:
        sess.set_scales(*scales)
    at = 0
    for b in range(B):
        need = -(-int(ctx_len[b]) // si.PAGE_SIZE)
        pages = [int(p) for p in order[at:at + need]]
        at += need
        sess.assign(b, int(ctx_len[b]), pages)
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, pages, kv[l][b][0], kv[l][b][1])
    tokens = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
    log = []
    want, _ = of.verify_forward(cfg, w_or, kv_or, tokens, ctx_len, route_log=log, kv_scales=scales)
    got = sess.forward(torch.arange(B, dtype=torch.int32, device="cuda"), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    sess.close()
    assert np.isfinite(got).all()

    # rows whose routing the oracle itself decides by less than MARGIN, and the rows after them in the sequence
    top_k = cfg["top_k"]
    fragile = np.zeros((B, k + 1), dtype=bool)
    loads = []
    for experts, weight, prob in log:
        if top_k < cfg["n_experts"]:                       # with every expert chosen there is nothing to decide
            srt = np.sort(np.log(prob), axis=-1)[:, ::-1]
            margin = (srt[:, top_k - 1] - srt[:, top_k]).reshape(B, k + 1)
            fragile |= margin < MARGIN
        loads.append(np.bincount(experts.reshape(-1), minlength=cfg["n_experts"]))
    exempt = np.logical_or.accumulate(fragile, axis=1)
    err = np.abs(got - want)
    bad = err > 2e-2 + 1e-2 * np.abs(want)
    rows_bad = bad.any(-1)
    assert not np.any(rows_bad & ~exempt), ("mismatch outside the exempted rows", np.argwhere(rows_bad & ~exempt)[:5],
                                           float(err[~exempt].max()))
    max_err = float(err[~exempt].max()) if (~exempt).any() else 0.0
    return max_err, int(exempt.sum()), B * (k + 1), loads


def test_small_moe_workload():
    wl = si.WORKLOADS["small_moe_b6_k3"]
    cfg = si.MODELS[wl["model"]]
    ctx = [int(c) for c in si.make_batch(wl)["ctx_len"]]
    max_err, n_exempt, n_rows, loads = _run(cfg, ctx, wl["k"], seed=14)
    print("small moe: max abs err %.3e on %d rows, %d exempted; rows per expert (layer 0): %s" % (max_err, n_rows - n_exempt, n_exempt, loads[0]))
    assert n_exempt <= max(2, n_rows // 10), (n_exempt, n_rows)


@pytest.mark.parametrize("B,k,changes,seed", [
    (96, 3, {}, 675),                                             # ~96 rows per expert: two 64-row tiles each, M = 384
    (3, 0, {}, 21),                                               # fewer rows than experts: most experts idle
    (20, 5, dict(n_experts=4, top_k=4), 145),                     # every expert on every row
    (33, 1, dict(n_experts=200, top_k=8, n_q_heads=8, n_kv_heads=2), 234),   # more experts than one wavefront's lanes
    (8, 2, dict(n_experts=5, top_k=1, expert_ffn_dim=768), 58),   # top-1 routing, wider experts
])
def test_moe_shapes(B, k, changes, seed):
    cfg = dict(si.MODELS["small_moe_bf16"], vocab=1000)
    cfg.update(changes)
    rng = np.random.default_rng(B + k)
    ctx = [int(c) for c in rng.integers(0, 150, size=B)]
    max_err, n_exempt, n_rows, loads = _run(cfg, ctx, k, seed=seed)
    print("moe B=%d k=%d %s: max abs err %.3e on %d rows, %d exempted; max rows/expert %d, idle experts %d" %
          (B, k, changes, max_err, n_rows - n_exempt, n_exempt, loads[0].max(), (loads[0] == 0).sum()))
    assert n_exempt <= max(2, n_rows // 10), (n_exempt, n_rows)


def test_small_moe_with_the_8bit_cache():
    """The mixture-of-experts forward over the E4M3 cache (64 query rows per kv head: the 4-row-block attention)."""
    wl = si.WORKLOADS["small_moe_b6_k3"]
    cfg = dict(si.MODELS[wl["model"]], kv_dtype="fp8_e4m3")
    ctx = [int(c) for c in si.make_batch(wl)["ctx_len"]]
    max_err, n_exempt, n_rows, loads = _run(cfg, ctx, wl["k"], seed=12)
    print("small moe, 8-bit cache: max abs err %.3e on %d rows, %d exempted" % (max_err, n_rows - n_exempt, n_exempt))
    assert n_exempt <= max(2, n_rows // 10), (n_exempt, n_rows)


@pytest.mark.parametrize("B,k,changes", [(6, 3, {}), (96, 3, {}), (20, 5, dict(n_experts=4, top_k=4)), (8, 2, dict(n_experts=5, top_k=1, expert_ffn_dim=768))])
def test_moe_with_8bit_matrices_and_cache(B, k, changes):
    """Expert, attention and head matrices as E4M3 codes with one scale per (expert and) output row, over the E4M3 cache:
    the grouped expert GEMMs widen the codes like the dense ones and take each expert's own scales."""
    cfg = dict(si.MODELS["small_moe_bf16"], vocab=1000, kv_dtype="fp8_e4m3", w_dtype="fp8_e4m3")
    cfg.update(changes)
    rng = np.random.default_rng(B + k)
    ctx = [int(c) for c in rng.integers(0, 150, size=B)]
    max_err, n_exempt, n_rows, loads = _run(cfg, ctx, k, seed=B * 7 + k)
    print("moe, 8-bit matrices and cache, B=%d k=%d %s: max abs err %.3e on %d rows, %d exempted" % (B, k, changes, max_err, n_rows - n_exempt, n_exempt))
    assert n_exempt <= max(2, n_rows // 10), (n_exempt, n_rows)


def test_router_weights_that_overflow_do_not_poison_the_step():
    """A router whose matrix holds infinities gives logits that are +inf, -inf or NaN (inf - inf).  The routing must
    still pick top_k distinct experts inside the range with finite weights: the logits of the step are finite, and a second session with healthy weights in the same process still matches the oracle."""
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["small_moe_bf16"]
    B, k = 5, 2
    weights = si.make_weights(cfg, seed=3)
    bad = {n: t.clone() for n, t in weights.items()}
    bad["l0.router"][2, :] = float("inf")                  # expert 2: +-inf or NaN on every row
    bad["l1.router"][5, ::2] = float("-inf")
    bad["l1.router"][7, 0] = float("nan")
    ctx = np.array([40, 3, 90, 17, 64])
    n_pages = sum(-(-(int(c) + k + 1) // si.PAGE_SIZE) for c in ctx) + 8
    sess = VerifySession(cfg, {n: t.cuda() for n, t in bad.items()}, max_seqs=B, max_ctx_len=160, n_pages=n_pages)
    sess.pool.zero_()
    at = 0
    for b in range(B):
        need = -(-int(ctx[b]) // si.PAGE_SIZE)
        sess.assign(b, int(ctx[b]), list(range(at, at + need)))
        at += need
    tokens = torch.randint(0, cfg["vocab"], (B, k + 1), dtype=torch.int32, device="cuda")
    seq = torch.arange(B, dtype=torch.int32, device="cuda")
    a = sess.forward(seq, tokens).clone()
    torch.cuda.synchronize()
    assert torch.isfinite(a).all()
    sess.close()
    max_err, n_exempt, n_rows, _ = _run(cfg, [30, 70, 5], 2, seed=14)
    assert max_err < 2e-2 and n_exempt <= n_rows // 3
