"""GPU parity of the verify step with the 8-bit (E4M3) KV cache against the CPU oracle, through the C ABI.

What is compared, and how:
  * logits against the fp64 oracle that reads decode(code) * scale and encodes the k+1 new positions before
    attending to them: the bf16 tolerance (2e-2 abs + 1e-2 rel).  The cached codes are inputs (identical on
    both sides); the new positions' codes are decided by floating point (fp32 kernels, fp64 oracle), so
  * the new positions' codes in the cache are compared one by one: equal, except that a code may be the
    neighbouring one (one step of the 3-bit mantissa) where the value sat at a rounding boundary (near zero, where
    the grid is finer than the kernels' own error, within 1e-3 in value); such elements are counted, printed and
    bounded (1 %); the cached context's bytes must be untouched;
  * every attention layout (1..4 row blocks per workgroup, row groups, chunk lengths, masked last pages, empty
    caches, chunk boundaries) with the pool's unused bytes set to the format's NaN code.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import forward as of
from oracle import fp8
from tests.helpers import random_norm_gains, logits_close
from tests.test_gpu_step import _run_custom_bf16

pytestmark = pytest.mark.gpu

TOL = (2e-2, 1e-2)


def _sign_magnitude_rank(code):
    """Position of a code on the number line's grid (so that neighbours differ by one; +-0 coincide)."""
    code = code.astype(np.int64)
    return np.where(code & 0x80, -(code & 0x7F), code & 0x7F)


def test_kv8_small_workload_logits_and_cache_codes():
    from paper_2604_26779_amd.session import VerifySession
    wl = dict(si.WORKLOADS["small_bf16_kv8_b5_k3"])
    cfg = si.MODELS[wl["model"]]
    seed = si.DEFAULT_SEED
    weights = random_norm_gains(si.make_weights(cfg, seed=seed), seed)
    w_or = si.weights_for_oracle(cfg, weights)
    batch = si.make_batch(wl, seed=seed)
    ctx_len, B, k = batch["ctx_len"], wl["B"], wl["k"]
    scales = si.kv_scales(cfg, seed=seed)
    kv = si.make_logical_kv(cfg, ctx_len, seed=seed)                 # codes
    kv_or = fp8.cache_values(si.kv_for_oracle(kv), scales)
    rng = np.random.default_rng(11)
    tokens = np.concatenate([batch["tokens0"][:, None], rng.integers(0, cfg["vocab"], size=(B, k))], axis=1).astype(np.int32)
    want, new_kv = of.verify_forward(cfg, w_or, kv_or, tokens, ctx_len, kv_scales=scales)

    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=B + 2, max_ctx_len=int(ctx_len.max()) + 64,
                         n_pages=batch["n_pages"] + 4 * B + 64)
    sess.pool.fill_(0x7F)
    with pytest.raises(Exception):                                   # no scales yet
        sess.forward(torch.arange(B, dtype=torch.int32, device="cuda"), torch.from_numpy(tokens).cuda())
    sess.set_scales(*scales)
    seq_ids = np.arange(B, dtype=np.int32) + 1
    for b in range(B):
        sess.assign(int(seq_ids[b]), int(ctx_len[b]), batch["page_lists"][b])
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, batch["page_lists"][b], kv[l][b][0], kv[l][b][1])
    got = sess.forward(torch.from_numpy(seq_ids).cuda(), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    ok, max_err, worst = logits_close(got.cpu().numpy(), want, *TOL)
    plain, _ = of.verify_forward(dict(cfg, kv_dtype=None), w_or, kv_or, tokens, ctx_len)
    print("8-bit cache, small workload: logits max abs err %.3e against the 8-bit oracle (the oracle with the new positions"
          " kept in bf16 differs from it by %.3e)" % (max_err, np.abs(plain - want).max()))
    assert ok, (max_err, worst)

    st = sess.state()
    flips = total = 0
    for b, s in enumerate(seq_ids):
        pages = [int(p) for p in st["page_table"][int(s)][:st["n_pages"][int(s)]]]
        c = int(ctx_len[b])
        for l in range(cfg["n_layers"]):
            K, V = sess.read_logical_kv(l, pages, c + k + 1)
            for which, dev in ((0, K.cpu().numpy()), (1, V.cpu().numpy())):
                assert np.array_equal(dev[:c], kv[l][b][which].view(torch.uint8).numpy())           # context untouched
                want_code = fp8.encode(new_kv[l][which][b] / np.asarray(scales[which], dtype=np.float64)[l][None, :, None])
                diff = np.abs(_sign_magnitude_rank(dev[c:]) - _sign_magnitude_rank(want_code))
                # near zero the grid (2^-9 * scale) is finer than the kernels' own error: compare values there
                far = np.abs(fp8.decode(dev[c:]) - fp8.decode(want_code)) * np.float64(scales[which][l])[None, :, None] > 1e-3
                assert not np.any((diff > 1) & far), "a stored code is neither the oracle's neighbour nor within 1e-3 of it"
                flips += int((diff >= 1).sum())
                total += diff.size
    print("new positions' codes: %d of %d one step from the oracle's" % (flips, total))
    assert flips <= 0.01 * total
    sess.close()


def test_kv8_edge_contexts_and_chunk_boundaries():
    ok, max_err, worst = _run_custom_bf16([0, 1, 15, 16, 17, 509, 511, 512, 513, 1023, 1024], k=3, kv8=True)
    print("8-bit cache, edge contexts: logits max abs err %.3e" % max_err)
    assert ok, (max_err, worst)


@pytest.mark.parametrize("k,heads", [(3, (8, 2)), (7, (8, 2)), (15, (8, 2)), (2, (32, 2)), (11, (16, 2))])
def test_kv8_row_block_counts_and_row_groups(k, heads):
    """16, 32, 64, 48 and 96 query rows per kv head: 1, 2, 4, 3 row blocks per workgroup and two row groups."""
    rng = np.random.default_rng(k)
    ctx = [int(c) for c in rng.integers(1, 700, size=4)] + [511, 0]
    ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=k, vocab=1000, kv8=True, n_q_heads=heads[0], n_kv_heads=heads[1])
    print("8-bit cache, k=%d Hq/Hkv=%s: logits max abs err %.3e" % (k, heads, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("row_blocks,chunk_pages", [(1, 4), (2, 12), (4, 256), (0, 64)])
def test_kv8_attention_layouts(row_blocks, chunk_pages):
    from paper_2604_26779_amd import binding as sv
    sv.spec_tune_set("attn_row_blocks", row_blocks)
    sv.spec_tune_set("attn_chunk_pages", chunk_pages)
    try:
        ctx = [0, 5, 16, 63, 64, 65, 130, 255, 300, 517, 700, 1023, 1030]
        ok, max_err, worst = _run_custom_bf16(ctx, k=5, seed=31 + row_blocks, vocab=1000, kv8=True, n_q_heads=16, n_kv_heads=1)
    finally:
        sv.spec_tune_set("attn_row_blocks", 0)
        sv.spec_tune_set("attn_chunk_pages", 0)
    print("8-bit cache, row blocks %d, chunk %d pages: logits max abs err %.3e" % (row_blocks, chunk_pages, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("key_scale", [6.0, 200.0])
def test_kv8_peaked_attention_and_exponent_range(key_scale):
    """Key scales 6 and 200 times larger: scores spread over tens and thousands of units (200: the fixed reference point's
    exponent check fails and the chunks are recomputed with the moving reference)."""
    rng = np.random.default_rng(int(key_scale))
    ctx = [int(c) for c in rng.integers(30, 1500, size=5)] + [513, 16]
    ok, max_err, worst = _run_custom_bf16(ctx, k=3, seed=21, vocab=1000, key_scale=key_scale, kv8=True)
    print("8-bit cache, key scale x%.0f: logits max abs err %.3e" % (key_scale, max_err))
    assert ok, (max_err, worst)


def test_kv8_every_code_is_read_exactly():
    """The cached keys and values of one head run through all 254 finite codes (both signs, subnormals, 448): with
    queries against them the logits stay within tolerance only if the kernel widens every code to the value the format
    defines (a wrong subnormal or top-binade value moves the attention output by far more than the tolerance)."""
    from paper_2604_26779_amd.session import VerifySession
    cfg = dict(si.MODELS["small_bf16_kv8"], vocab=1000)
    seed = 77
    weights = random_norm_gains(si.make_weights(cfg, seed=seed), seed)
    w_or = si.weights_for_oracle(cfg, weights)
    ctx_len = np.array([254, 40], dtype=np.int64)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    rng = np.random.default_rng(seed)
    kv = []
    for l in range(cfg["n_layers"]):
        per = []
        for c in ctx_len:
            K = np.stack([np.stack([rng.permutation(codes)[:c] for _ in range(cfg["head_dim"])], axis=1)
                          for _ in range(cfg["n_kv_heads"])], axis=1)          # [c, Hkv, dh]
            V = np.stack([np.stack([rng.permutation(codes)[:c] for _ in range(cfg["head_dim"])], axis=1)
                          for _ in range(cfg["n_kv_heads"])], axis=1)
            per.append((torch.from_numpy(K.copy()), torch.from_numpy(V.copy())))
        kv.append(per)
    scales = (np.full((cfg["n_layers"], cfg["n_kv_heads"]), 1.0 / 256, dtype=np.float32),
              np.full((cfg["n_layers"], cfg["n_kv_heads"]), 1.0 / 128, dtype=np.float32))
    kv_or = [[(fp8.decode(K.numpy()) * float(scales[0][l][0]), fp8.decode(V.numpy()) * float(scales[1][l][0])) for (K, V) in per]
             for l, per in enumerate(kv)]
    tokens = rng.integers(0, cfg["vocab"], size=(2, 3)).astype(np.int32)
    want, _ = of.verify_forward(cfg, w_or, kv_or, tokens, ctx_len, kv_scales=scales)
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=2, max_ctx_len=512, n_pages=64)
    sess.pool.fill_(0x7F)
    sess.set_scales(*scales)
    at = 0
    for b in range(2):
        n = -(-int(ctx_len[b]) // si.PAGE_SIZE)
        pages = list(range(at, at + n))
        at += n
        sess.assign(b, int(ctx_len[b]), pages)
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, pages, kv[l][b][0], kv[l][b][1])
    got = sess.forward(torch.arange(2, dtype=torch.int32, device="cuda"), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    ok, max_err, worst = logits_close(got.cpu().numpy(), want, *TOL)
    print("8-bit cache, all codes: logits max abs err %.3e" % max_err)
    assert ok, (max_err, worst)
    sess.close()


# ------------------------------------------------------------------------------------------ 8-bit matrices
W8 = dict(w_dtype="fp8_e4m3")


@pytest.mark.parametrize("B,k,kv8", [(1, 0, False), (1, 7, True), (16, 3, True), (24, 3, False), (32, 3, True), (40, 3, True), (33, 7, False), (9, 2, True)])
def test_w8_row_block_counts(B, k, kv8):
    """E4M3 matrices with one scale per output row (the codes are inputs, the oracle multiplies by the dequantised
    matrix): M = 1 .. 264 rows, i.e. every row-block count of the 128-column tile (fused and unfused SwiGLU, K split
    and unsplit), more than one row tile, ragged column counts (vocabulary 1000), with either cache type."""
    rng = np.random.default_rng(B * 10 + k)
    ctx = [int(c) for c in rng.integers(3, 200, size=B)]
    ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000, kv8=kv8, **W8)
    print("8-bit matrices, B=%d k=%d (M=%d), 8-bit cache %s: logits max abs err %.3e" % (B, k, B * (k + 1), kv8, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("B,k,big_from", [(64, 3, 8), (33, 7, 8), (12, 15, 6), (96, 3, 8)])
def test_w8_large_row_tiles(B, k, big_from):
    """The 192- and 256-row x 256-column tiles with 8-bit matrices (plain and fused SwiGLU epilogues, split K)."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_big_min_blocks")
    sv.spec_tune_set("gemm_big_min_blocks", big_from)
    try:
        rng = np.random.default_rng(B * 10 + k)
        ctx = [int(c) for c in rng.integers(3, 120, size=B)]
        ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000, kv8=True, **W8)
    finally:
        sv.spec_tune_set("gemm_big_min_blocks", before)
    print("8-bit matrices, B=%d k=%d (M=%d), big tiles from %d row blocks: logits max abs err %.3e" % (B, k, B * (k + 1), big_from, max_err))
    assert ok, (max_err, worst)


def test_w8_description_checks():
    """8-bit matrices are refused where the kernels have no path for them, with an error and nothing launched."""
    from paper_2604_26779_amd import binding as sv
    for changes in (dict(tied_head=1), dict(dtype="f32", head_dim=64)):
        cfg = dict(si.MODELS["small_bf16_w8"], **changes)
        desc = sv.make_desc(cfg)
        n = sv.lib().spec_model_weight_count(__import__("ctypes").byref(desc))
        dummy = [torch.zeros(64, dtype=torch.uint8, device="cuda")] * n
        with pytest.raises(sv.SpecError):
            sv.spec_model_create(cfg, dummy)


def test_scales_are_refused_for_a_cache_that_is_not_8bit():
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = dict(si.MODELS["small_bf16"], vocab=1000)
    weights = si.make_weights(cfg, seed=1)
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=2, max_ctx_len=64, n_pages=16)
    one = torch.ones(cfg["n_layers"] * cfg["n_kv_heads"], dtype=torch.float32, device="cuda")
    with pytest.raises(sv.SpecError):
        sv.spec_kv_set_scales(sess.kv, one, one)
    sess.close()
