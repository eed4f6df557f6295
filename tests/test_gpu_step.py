"""GPU parity of the whole verify step (forward -> rejection sampling -> KV commit) through the
C ABI against the CPU oracle, on workloads the oracle finishes in seconds:

  * tiny_fp32_b4_ctx128_k3 : the fp32 configuration, true prefill computed by the oracle;
    logits within 1e-4, end-to-end sampling and commit compared with the oracle's own chain.
  * small_bf16_b5_k3       : the MFMA path at a size that spans several GEMM tiles, ragged N and
    vocabulary tails, ragged contexts (several attention chunks, partial pages), GQA;
    logits within 2e-2 abs + 1e-2 rel of the fp64 oracle on bf16-rounded weights and cache.
Drafts and draft distributions come from the oracle run autoregressively (never from the HIP path).
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import commit as oracle_commit
from oracle import forward as of
from oracle import sampler as oracle_sampler
from tests.helpers import random_norm_gains, assert_sampler_parity, logits_close, oracle_drafts

pytestmark = pytest.mark.gpu

SEED = si.DEFAULT_SEED
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 1e-2)}
KV_TOL = {"f32": 1e-5, "bf16": 2e-2}


def _setup(workload_name, k=None, prefill="oracle", shuffle=True, seed=SEED, B=None):
    from paper_2604_26779_amd.session import VerifySession
    wl = dict(si.WORKLOADS[workload_name])
    if k is not None:
        wl["k"] = k
    if B is not None:
        wl["B"] = B
    cfg = si.MODELS[wl["model"]]
    weights = random_norm_gains(si.make_weights(cfg, seed=seed), seed)
    w_or = si.weights_for_oracle(cfg, weights)
    batch = si.make_batch(wl, seed=seed, shuffle_pages=shuffle)
    ctx_len = batch["ctx_len"]
    if prefill == "oracle":
        toks = np.stack(batch["ctx_tokens"]) if len(set(ctx_len)) == 1 else None
        if toks is not None:
            kv_or = of.prefill(cfg, w_or, toks)
        else:
            per = [of.prefill(cfg, w_or, t[None, :]) for t in batch["ctx_tokens"]]
            kv_or = [[per[b][l][0] for b in range(len(per))] for l in range(cfg["n_layers"])]
        # the cache holds storage-type values: round what the oracle computed, then both sides use that
        kv_or = [[(si.round_to_storage(K, cfg["dtype"]), si.round_to_storage(V, cfg["dtype"])) for (K, V) in per_l]
                 for per_l in kv_or]
    else:
        kv_or = si.kv_for_oracle(si.make_logical_kv(cfg, ctx_len, seed=seed))
    max_ctx = int(ctx_len.max()) + 64
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=wl["B"] + 2, max_ctx_len=max_ctx,
                         n_pages=batch["n_pages"] + 4 * wl["B"] + 64)
    sess.pool.normal_()                                   # stale data everywhere a step must not read
    seq_ids = np.arange(wl["B"], dtype=np.int32) + 1      # sequence ids differ from batch positions
    for b in range(wl["B"]):
        sess.assign(int(seq_ids[b]), int(ctx_len[b]), batch["page_lists"][b])
        for l in range(cfg["n_layers"]):
            K, V = kv_or[l][b]
            sess.write_logical_kv(l, batch["page_lists"][b], torch.from_numpy(K), torch.from_numpy(V))
    return wl, cfg, w_or, kv_or, batch, sess, seq_ids


def _book(batch, sess, seq_ids, ctx_len):
    book = oracle_commit.KVBook(sess.n_pages, si.PAGE_SIZE)
    for b, s in enumerate(seq_ids):
        book.assign(int(s), int(ctx_len[b]), batch["page_lists"][b])
    return book


def _check_state(sess, book, seq_ids):
    st = sess.state()
    for s in seq_ids:
        s = int(s)
        assert st["ctx_len"][s] == book.ctx_len[s]
        assert st["n_pages"][s] == len(book.pages[s])
        assert list(st["page_table"][s][:len(book.pages[s])]) == book.pages[s]
    assert list(st["free_stack"]) == book.free


@pytest.mark.parametrize("workload", ["tiny_fp32_b4_ctx128_k3", "small_bf16_b5_k3"])
def test_full_step_parity(workload):
    wl, cfg, w_or, kv_or, batch, sess, seq_ids = _setup(workload)
    B, k, T_ = wl["B"], wl["k"], wl["temperature"]
    ctx_len = batch["ctx_len"]
    tokens, q = oracle_drafts(cfg, w_or, kv_or, batch["tokens0"], ctx_len, k, wl["noise_std"], T_, SEED)
    want_logits, new_kv = of.verify_forward(cfg, w_or, kv_or, tokens, ctx_len)

    d_seq = torch.from_numpy(seq_ids).cuda()
    d_tok = torch.from_numpy(tokens).cuda()
    logits = sess.forward(d_seq, d_tok)
    torch.cuda.synchronize()
    got = logits.cpu().numpy()
    ok, max_err, worst = logits_close(got, want_logits, *TOL[cfg["dtype"]])
    print(workload, "logits max abs err %.3e (|logit| max %.2f)" % (max_err, np.abs(want_logits).max()))
    assert ok, (max_err, worst)

    # the k+1 new cache entries of every layer sit in the reserved slots
    book = _book(batch, sess, seq_ids, ctx_len)
    book.reserve([int(s) for s in seq_ids], k)
    st = sess.state()
    for b, s in enumerate(seq_ids):
        pages = book.pages[int(s)]
        assert list(st["page_table"][int(s)][:len(pages)]) == pages
        for l in range(cfg["n_layers"]):
            K, V = sess.read_logical_kv(l, pages, int(ctx_len[b]) + k + 1)
            K, V = K.float().cpu().numpy(), V.float().cpu().numpy()
            c = int(ctx_len[b])
            assert np.array_equal(K[:c], kv_or[l][b][0]) and np.array_equal(V[:c], kv_or[l][b][1])   # context untouched
            assert np.max(np.abs(K[c:] - new_kv[l][0][b])) < KV_TOL[cfg["dtype"]] * max(1.0, np.abs(new_kv[l][0][b]).max())
            assert np.max(np.abs(V[c:] - new_kv[l][1][b])) < KV_TOL[cfg["dtype"]] * max(1.0, np.abs(new_kv[l][1][b]).max())

    # sampling: (1) kernel vs oracle sampler on identical logits (the oracle's), bit-exact modulo flagged trials
    seed, step = 424242, 3
    d_q, d_draft = torch.from_numpy(q).cuda(), torch.from_numpy(tokens[:, 1:].copy()).cuda()
    d_or_logits = torch.from_numpy(want_logits.astype(np.float32)).cuda()
    n_dev, out_dev = sess.sample(d_or_logits, d_q, d_draft, T_, seed, step)
    torch.cuda.synchronize()
    n_or, out_or, pqu, keys = oracle_sampler.reject_sample(want_logits.astype(np.float32), q, tokens[:, 1:], T_, seed, step,
                                                           debug=True)
    print(workload, "sampler on oracle logits", assert_sampler_parity(n_dev.cpu().numpy(), out_dev.cpu().numpy(), n_or, out_or, pqu, keys, exact=True))

    # (2) the chained step: HIP logits -> HIP sampler -> HIP commit, no host sync in between.
    # Nothing the HIP path produced is handed to the oracle: the chain is checked for what must hold
    # whatever it sampled, and (fp32 configuration, logits equal to 1e-4) against the oracle's own chain.
    from paper_2604_26779_amd import binding as sv
    snap = torch.empty(sv.spec_kv_state_bytes(sess.kv), dtype=torch.uint8, device="cuda")
    sv.spec_kv_snapshot(sess.kv, snap)
    n_dev, out_dev = sess.sample(logits, d_q, d_draft, T_, seed, step)
    new_len, slots = sess.commit(d_seq, n_dev, k)
    torch.cuda.synchronize()
    n_gpu, out_gpu = n_dev.cpu().numpy(), out_dev.cpu().numpy()
    if cfg["dtype"] == "f32":
        print(workload, "end-to-end", assert_sampler_parity(n_gpu, out_gpu, n_or, out_or, pqu, keys, max_exempt_frac=0.5))
    assert np.all((n_gpu >= 0) & (n_gpu <= k))
    assert list(new_len.cpu().numpy()) == list(ctx_len + n_gpu + 1)
    slots_h = slots.cpu().numpy()
    for b in range(B):
        assert np.array_equal(out_gpu[b, :n_gpu[b]], tokens[b, 1:1 + n_gpu[b]])
        assert 0 <= out_gpu[b, n_gpu[b]] < cfg["vocab"] and np.all(out_gpu[b, n_gpu[b] + 1:] == -1)
        assert np.all(slots_h[b, :n_gpu[b] + 1] >= 0) and np.all(slots_h[b, n_gpu[b] + 1:] == -1)
    print(workload, "accepted lengths", n_gpu.tolist(), "alpha = %.2f" % oracle_commit.mean_acceptance_length(n_gpu))

    # (3) commit parity: same state, accept lengths from the ORACLE's sampler on both sides
    sv.spec_kv_restore(sess.kv, snap)
    new_len, slots = sess.commit(d_seq, torch.from_numpy(n_or).cuda(), k)
    want_len, want_slots = book.commit([int(s) for s in seq_ids], n_or, k)
    assert list(new_len.cpu().numpy()) == want_len
    assert slots.cpu().numpy().tolist() == want_slots
    _check_state(sess, book, seq_ids)
    sess.close()


@pytest.mark.parametrize("workload,k", [("small_bf16_b5_k3", 1), ("small_bf16_b5_k3", 7), ("tiny_fp32_b4_ctx128_k3", 0),
                                        ("tiny_fp32_b4_ctx128_k3", 5)])
def test_logits_parity_other_draft_lengths(workload, k):
    wl, cfg, w_or, kv_or, batch, sess, seq_ids = _setup(workload, k=k, prefill="synthetic")
    rng = np.random.default_rng(k)
    tokens = np.concatenate([batch["tokens0"][:, None], rng.integers(0, cfg["vocab"], size=(wl["B"], k))], axis=1).astype(np.int32)
    want, _ = of.verify_forward(cfg, w_or, kv_or, tokens, batch["ctx_len"])
    logits = sess.forward(torch.from_numpy(seq_ids).cuda(), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    ok, max_err, worst = logits_close(logits.cpu().numpy(), want, *TOL[cfg["dtype"]])
    print(workload, "k=%d" % k, "logits max abs err %.3e" % max_err)
    assert ok, (max_err, worst)
    sess.close()


def test_multi_step_rollout_matches_oracle_bookkeeping_and_logits():
    """Three chained steps with forced accept lengths (commit driven from a device tensor): contexts,
    page lists and the free stack follow the oracle's book, and the third step's logits - which read
    K/V written by the first two - match the oracle's forward over the grown cache."""
    wl, cfg, w_or, kv_or, batch, sess, seq_ids = _setup("small_bf16_b5_k3", prefill="synthetic")
    B, k = wl["B"], wl["k"]
    rng = np.random.default_rng(77)
    ctx_len = batch["ctx_len"].copy()
    book = _book(batch, sess, seq_ids, ctx_len)
    d_seq = torch.from_numpy(seq_ids).cuda()
    kv_cur = [[(K.copy(), V.copy()) for (K, V) in per] for per in kv_or]
    for step in range(3):
        tokens = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
        want, new_kv = of.verify_forward(cfg, w_or, kv_cur, tokens, ctx_len)
        logits = sess.forward(d_seq, torch.from_numpy(tokens).cuda())
        torch.cuda.synchronize()
        ok, max_err, worst = logits_close(logits.cpu().numpy(), want, *TOL["bf16"])
        assert ok, (step, max_err, worst)
        n = rng.integers(0, k + 1, size=B).astype(np.int32)
        book.reserve([int(s) for s in seq_ids], k)
        new_len, slots = sess.commit(d_seq, torch.from_numpy(n).cuda(), k)
        want_len, want_slots = book.commit([int(s) for s in seq_ids], n, k)
        assert list(new_len.cpu().numpy()) == want_len and slots.cpu().numpy().tolist() == want_slots
        _check_state(sess, book, seq_ids)
        # the oracle's cache keeps the accepted prefix, rounded to the storage type like the real cache
        for l in range(cfg["n_layers"]):
            for b in range(B):
                keepK = si.round_to_storage(new_kv[l][0][b][:n[b] + 1], cfg["dtype"])
                keepV = si.round_to_storage(new_kv[l][1][b][:n[b] + 1], cfg["dtype"])
                kv_cur[l][b] = (np.concatenate([kv_cur[l][b][0], keepK]), np.concatenate([kv_cur[l][b][1], keepV]))
        ctx_len = ctx_len + n + 1
    sess.close()


def test_snapshot_restore_and_page_permutation_invariance():
    wl, cfg, w_or, kv_or, batch, sess, seq_ids = _setup("small_bf16_b5_k3", prefill="synthetic", shuffle=True)
    from paper_2604_26779_amd import binding as sv
    B, k = wl["B"], wl["k"]
    rng = np.random.default_rng(5)
    tokens = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
    d_seq, d_tok = torch.from_numpy(seq_ids).cuda(), torch.from_numpy(tokens).cuda()
    snap = torch.empty(sv.spec_kv_state_bytes(sess.kv), dtype=torch.uint8, device="cuda")
    sv.spec_kv_snapshot(sess.kv, snap)
    first = sess.forward(d_seq, d_tok).clone()
    sess.commit(d_seq, torch.full((B,), k, dtype=torch.int32, device="cuda"), k)
    sv.spec_kv_restore(sess.kv, snap)
    again = sess.forward(d_seq, d_tok).clone()
    torch.cuda.synchronize()
    assert torch.equal(first, again)                       # same state, same launch: bit-identical
    st = sess.state()
    assert list(st["ctx_len"][seq_ids]) == list(batch["ctx_len"])
    with pytest.raises(sv.SpecError):
        sv.spec_kv_restore(sess.kv, torch.empty_like(snap))
    sess.close()
    # contiguous instead of shuffled physical pages: logits must not depend on where pages live
    wl2, cfg2, _, _, batch2, sess2, seq_ids2 = _setup("small_bf16_b5_k3", prefill="synthetic", shuffle=False)
    other = sess2.forward(torch.from_numpy(seq_ids2).cuda(), d_tok)
    torch.cuda.synchronize()
    assert torch.equal(first, other)
    sess2.close()


def test_forward_argument_errors_and_pool_exhaustion():
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["tiny_fp32"]
    weights = {n: t.cuda() for n, t in si.make_weights(cfg).items()}
    sess = VerifySession(cfg, weights, max_seqs=4, max_ctx_len=64, n_pages=3)
    sess.assign(0, 16, [2])
    sess.assign(1, 15, [0])
    with pytest.raises(sv.SpecError) as e:                 # page already in use
        sess.assign(2, 5, [0])
    assert e.value.status == sv.SPEC_EINVAL
    with pytest.raises(sv.SpecError):                      # wrong number of pages
        sess.assign(2, 17, [1])
    d_seq = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    tok = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    buf = sess.step_buffers(2, 3)
    with pytest.raises(sv.SpecError) as e:                 # sequence 0 needs a page, sequence 1 needs a page, one is free
        sess.forward(d_seq, tok)
    assert e.value.status == sv.SPEC_ENOMEM
    with pytest.raises(sv.SpecError) as e:                 # workspace too small
        sv.spec_verify_forward(sess.model, sess.kv, 2, 3, d_seq, tok, buf["logits"], buf["workspace"][:256])
    assert e.value.status == sv.SPEC_EINVAL
    with pytest.raises(sv.SpecError):                      # k out of range
        sv.spec_verify_forward(sess.model, sess.kv, 2, 16, d_seq, tok, buf["logits"], buf["workspace"])
    # one sequence alone fits
    sess.forward(d_seq[:1], tok[:1])
    torch.cuda.synchronize()
    assert sess.state()["n_pages"][0] == 2
    sess.close()
    with pytest.raises(sv.SpecError) as e:                 # bf16 path needs head_dim 128
        VerifySession(dict(cfg, dtype="bf16"), {n: t.bfloat16() for n, t in weights.items()}, 2, 64, 8)
    assert e.value.status == sv.SPEC_EUNSUPPORTED


def _run_custom_bf16(ctx_list, k, seed=3, vocab=None, key_scale=1.0, key_scale_fn=None, kv8=False, **model_changes):
    """small_bf16 model, synthetic cache, explicit context lengths: returns (max err, worst over tolerance).
    kv8: the 8-bit cache (codes under the synthetic scales; key_scale then multiplies the key scales instead)."""
    from paper_2604_26779_amd.session import VerifySession
    cfg = dict(si.MODELS["small_bf16_kv8" if kv8 else "small_bf16"])
    cfg.update(model_changes)
    if vocab:
        cfg["vocab"] = vocab
    B = len(ctx_list)
    weights = random_norm_gains(si.make_weights(cfg, seed=seed), seed)
    w_or = si.weights_for_oracle(cfg, weights)
    ctx_len = np.array(ctx_list, dtype=np.int64)
    kv = si.make_logical_kv(cfg, ctx_len, seed=seed)
    scales = None
    if kv8:
        assert key_scale_fn is None
        scales = si.kv_scales(cfg, seed=seed)
        scales = (scales[0] * np.float32(key_scale), scales[1])
        key_scale = 1.0
    if key_scale != 1.0:        # larger cached keys -> larger scores -> a peaked softmax (a few keys carry the weight)
        kv = [[((K.float() * key_scale).to(K.dtype), V) for (K, V) in per_seq] for per_seq in kv]
    if key_scale_fn is not None:    # a scale per cached position: key_scale_fn(ctx) -> [ctx] factors
        kv = [[((K.float() * torch.as_tensor(key_scale_fn(K.shape[0]), dtype=torch.float32).view(-1, 1, 1)).to(K.dtype), V)
               for (K, V) in per_seq] for per_seq in kv]
    kv_or = si.kv_for_oracle(kv)
    if kv8:
        from oracle import fp8
        kv_or = fp8.cache_values(kv_or, scales)
    rng = np.random.default_rng(seed)
    n_ctx_pages = [-(-int(c) // si.PAGE_SIZE) for c in ctx_len]
    n_pages = sum(-(-(int(c) + k + 1) // si.PAGE_SIZE) for c in ctx_len) + 16
    order = rng.permutation(n_pages)
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=B, max_ctx_len=int(ctx_len.max()) + 64,
                         n_pages=n_pages)
    sess.pool.fill_(0x7F if kv8 else float("nan"))       # (NaN in either storage type) whatever a step reads beyond its data must not matter
    if kv8:
        sess.set_scales(*scales)
    at = 0
    for b in range(B):
        pages = [int(p) for p in order[at:at + n_ctx_pages[b]]]
        at += n_ctx_pages[b]
        sess.assign(b, int(ctx_len[b]), pages)
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, pages, kv[l][b][0], kv[l][b][1])
    tokens = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
    want, _ = of.verify_forward(cfg, w_or, kv_or, tokens, ctx_len, kv_scales=scales)
    got = sess.forward(torch.arange(B, dtype=torch.int32, device="cuda"), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    sess.close()
    assert np.isfinite(got).all()
    ok, max_err, worst = logits_close(got, want, *TOL["bf16"])
    return ok, max_err, worst


def test_bf16_edge_contexts_empty_page_and_chunk_boundaries():
    """Context lengths at the degenerate points: empty cache, one token, page boundaries (15/16/17),
    attention-chunk boundaries (511/512/513 tokens = 32 pages per chunk), new positions straddling a page
    and a chunk; the pool is NaN-filled so any read past a sequence's data shows."""
    ok, max_err, worst = _run_custom_bf16([0, 1, 15, 16, 17, 509, 511, 512, 513, 1023, 1024], k=3)
    print("edge contexts: logits max abs err %.3e" % max_err)
    assert ok, (max_err, worst)


@pytest.mark.parametrize("B,k", [(1, 0), (1, 7), (40, 3), (33, 7), (9, 2)])
def test_bf16_row_block_counts_and_multiple_row_tiles(B, k):
    """M = B*(k+1) from 1 to 264: every row-block count of the GEMM tile (1..4, fused and unfused
    SwiGLU), more than one 128-row tile (M = 160, 264: the weights are streamed once per tile), odd k."""
    rng = np.random.default_rng(B * 10 + k)
    ctx = [int(c) for c in rng.integers(3, 200, size=B)]
    ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000)
    print("B=%d k=%d (M=%d): logits max abs err %.3e" % (B, k, B * (k + 1), max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("k,heads", [(15, (8, 2)), (3, (16, 1)), (2, (32, 2)), (11, (16, 2))])
def test_bf16_more_than_32_query_rows_per_kv_head(k, heads):
    """(k+1) * G = 64, 64, 48 and 96 query rows per kv head: the attention splits them into row groups of 32."""
    rng = np.random.default_rng(k)
    ctx = [int(c) for c in rng.integers(1, 700, size=4)] + [511, 0]
    ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=k, vocab=1000, n_q_heads=heads[0], n_kv_heads=heads[1])
    print("k=%d Hq/Hkv=%s: logits max abs err %.3e" % (k, heads, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("key_scale", [6.0, 20.0])
def test_bf16_peaked_attention(key_scale):
    """The synthetic cache gives nearly flat attention; trained models do not.  With the cached keys scaled up the
    scores spread over tens of units and a handful of keys carry the softmax: the online softmax's rescaling, the
    hi+lo split of the probabilities and the merge of chunks with very different maxima are then what is tested."""
    rng = np.random.default_rng(int(key_scale))
    ctx = [int(c) for c in rng.integers(30, 1500, size=5)] + [513, 16]
    ok, max_err, worst = _run_custom_bf16(ctx, k=3, seed=21, vocab=1000, key_scale=key_scale)
    print("key scale %.0f: logits max abs err %.3e" % (key_scale, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("row_blocks,chunk_pages", [(1, 4), (2, 12), (3, 32), (4, 256), (0, 8)])
def test_bf16_attention_layouts(row_blocks, chunk_pages):
    """96 query rows per kv head (6 row blocks) under every way of laying them over workgroups (1..4 row blocks per
    workgroup, 6 / 3 / 2 / 2 groups) and chunk lengths from 4 pages (many chunks, wavefronts with one page or none)
    to 256 (one chunk, up to 11 pages per wavefront: whole groups of three, remainders of one and two)."""
    from paper_2604_26779_amd import binding as sv
    sv.spec_tune_set("attn_row_blocks", row_blocks)
    sv.spec_tune_set("attn_chunk_pages", chunk_pages)
    try:
        ctx = [0, 5, 16, 63, 64, 65, 130, 255, 300, 517, 700]
        ok, max_err, worst = _run_custom_bf16(ctx, k=5, seed=31 + row_blocks, vocab=1000, n_q_heads=16, n_kv_heads=1)
    finally:
        sv.spec_tune_set("attn_row_blocks", 0)
        sv.spec_tune_set("attn_chunk_pages", 0)
    print("row blocks %d, chunk %d pages: logits max abs err %.3e" % (row_blocks, chunk_pages, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("case", ["late_keys_huge", "last_page_large"])
def test_bf16_attention_reference_point_moves(case):
    """The attention keeps the exponentials' reference point of a wavefront where its first page put it and checks
    the exponent range afterwards.  late_keys_huge: keys from position 64 on are 150 times larger, so the scores
    outgrow the first pages' by hundreds of units: the range check fails and the chunk is recomputed with the moving
    reference.  last_page_large: only the keys of the last, partial page are 12 times larger: the masked pages'
    moving reference steps up and rescales the accumulators."""
    if case == "late_keys_huge":
        fn = lambda n: np.where(np.arange(n) >= 64, 150.0, 1.0)
    else:
        fn = lambda n: np.where(np.arange(n) >= 16 * (n // 16), 12.0, 1.0)
    ctx = [70, 200, 333, 519, 1000, 1531]
    for heads in [(8, 2), (16, 1)]:
        ok, max_err, worst = _run_custom_bf16(ctx, k=3, seed=41, vocab=1000, key_scale_fn=fn, n_q_heads=heads[0],
                                              n_kv_heads=heads[1])
        print("%s, Hq/Hkv=%s: logits max abs err %.3e" % (case, heads, max_err))
        assert ok, (max_err, worst)


@pytest.mark.parametrize("B,k,big_from", [(64, 3, 8), (33, 7, 8), (12, 15, 6), (50, 3, 6), (96, 3, 8), (40, 5, 8), (40, 3, 5), (33, 3, 5)])
def test_bf16_large_row_tiles(B, k, big_from):
    """The 192- and 256-row x 256-column GEMM tiles (tuning parameter gemm_big_min_blocks): M = 256 (one 8-block tile),
    264 (9 blocks -> two 6-block tiles, the second half empty), 192 (one 6-block tile), 200 (7 blocks -> one 8-block tile),
    384 (two 6-block tiles), 240, and 160 and 132 (5 row blocks in one 6-block tile); column counts that are not multiples of 256, fused SwiGLU epilogue, split K."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_big_min_blocks"), sv.spec_tune_get("gemm_big_min_tiles")
    sv.spec_tune_set("gemm_big_min_blocks", big_from)
    sv.spec_tune_set("gemm_big_min_tiles", 1)                # the small model has far fewer column tiles than the policy asks for
    try:
        rng = np.random.default_rng(B * 10 + k)
        ctx = [int(c) for c in rng.integers(3, 120, size=B)]
        ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000)
    finally:
        sv.spec_tune_set("gemm_big_min_blocks", before[0])
        sv.spec_tune_set("gemm_big_min_tiles", before[1])
    print("B=%d k=%d (M=%d), big tiles from %d row blocks: logits max abs err %.3e" % (B, k, B * (k + 1), big_from, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("chunk_pages", [64, 128])
def test_bf16_attention_long_chunks_at_their_boundaries(chunk_pages):
    """The chunk lengths the launch policy picks for large batches (64 and 128 pages = 1024 and 2048 tokens): contexts
    one token short of, at and one past a chunk boundary, and new positions that straddle it (k = 3)."""
    from paper_2604_26779_amd import binding as sv
    sv.spec_tune_set("attn_chunk_pages", chunk_pages)
    try:
        edge = chunk_pages * 16
        ctx = [edge - 4, edge - 3, edge - 1, edge, edge + 1, 2 * edge - 2, 2 * edge + 5, 17]
        ok, max_err, worst = _run_custom_bf16(ctx, k=3, seed=50 + chunk_pages, vocab=1000)
    finally:
        sv.spec_tune_set("attn_chunk_pages", 0)
    print("chunk %d pages: logits max abs err %.3e" % (chunk_pages, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("split_rows", [0, 1])
def test_bf16_128_rows_as_one_tile_or_two(split_rows):
    """GEMMs of 97..128 rows run as two 64-row x 256-column tiles per column stripe (the default does so up to 256 rows)
    or as one 128 x 128 tile: both ways, M = 128 and a ragged 101, fused SwiGLU and K-split projections."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_split_rows")
    sv.spec_tune_set("gemm_split_rows", split_rows)
    try:
        for B, k in ((32, 3), (101, 0)):
            rng = np.random.default_rng(B + k)
            ctx = [int(c) for c in rng.integers(3, 150, size=B)]
            ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000)
            print("split rows %d, B=%d k=%d: logits max abs err %.3e" % (split_rows, B, k, max_err))
            assert ok, (max_err, worst)
    finally:
        sv.spec_tune_set("gemm_split_rows", before)


@pytest.mark.parametrize("B,k,w8", [(40, 3, False), (32, 5, False), (64, 3, False), (50, 3, True), (43, 4, False), (33, 3, True)])
@pytest.mark.parametrize("tiles96", [1, 0])
def test_bf16_129_to_256_rows_as_64_row_tiles(B, k, w8, tiles96):
    """GEMMs of 129..256 rows as three or four 64-row x 256-column tiles per column stripe (gemm_split_rows = 2, the default;
    test_bf16_128_rows_as_one_tile_or_two and the 8B-shape sweeps cover the 128 x 128 tiles) instead of two 128 x 128 tiles: M = 160 (the third tile half padding), 192 (no fourth tile), 256, 200, 215 and 132, K-split
    projections; the fused gate/up projection as two 96- or 128-row x 256-column tiles; bf16 and 8-bit matrices."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_split_rows"), sv.spec_tune_get("gemm_tiles_96")
    sv.spec_tune_set("gemm_split_rows", 2)
    sv.spec_tune_set("gemm_tiles_96", tiles96)              # 0: the fused projection in 64-row tiles as well
    try:
        rng = np.random.default_rng(B + k)
        ctx = [int(c) for c in rng.integers(3, 150, size=B)]
        extra = dict(w_dtype="fp8_e4m3") if w8 else {}
        ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1000, **extra)
    finally:
        sv.spec_tune_set("gemm_split_rows", before[0])
        sv.spec_tune_set("gemm_tiles_96", before[1])
    print("64-row tiles, B=%d k=%d (M=%d), 8-bit matrices %s: logits max abs err %.3e" % (B, k, B * (k + 1), w8, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("B,k,w8", [(32, 3, False), (25, 3, True), (13, 7, False), (16, 3, False), (9, 4, True)])
def test_bf16_128x256_tiles_for_single_tile_gemms(B, k, w8):
    """The 128-row x 256-column tile with the wavefronts 1 x 4 (taken by the LM head of large vocabularies), forced here
    onto every plain-epilogue GEMM of the small model: M = 128, 100 and 104 rows (and 64 x 256 tiles: M = 64, 45), column counts 1536, 512 and 1024,
    K split and unsplit, bf16 and 8-bit matrices."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_wide4")
    sv.spec_tune_set("gemm_wide4", 1)
    try:
        rng = np.random.default_rng(B + k)
        ctx = [int(c) for c in rng.integers(3, 150, size=B)]
        extra = dict(w_dtype="fp8_e4m3") if w8 else {}
        ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k, vocab=1024, **extra)
    finally:
        sv.spec_tune_set("gemm_wide4", before)
    print("128 x 256 tiles, B=%d k=%d (M=%d), 8-bit matrices %s: logits max abs err %.3e" % (B, k, B * (k + 1), w8, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("mask", [0, 15, 3])
@pytest.mark.parametrize("B,k,w8", [(9, 2, False), (16, 3, True), (25, 3, False), (32, 3, False), (40, 3, True), (64, 3, False), (96, 3, False)])
def test_bf16_activation_formats_per_projection(mask, B, k, w8):
    """Which projections take one fp16 activation per value instead of hi + lo bf16 pairs is a set of bits read at
    model creation (gemm_f16_inputs; bit 0 QKV, 1 attention output, 2 feed-forward, 3 head; default 12, which every
    other test runs).  Here the other settings - all hi + lo, all fp16, and the default's complement - go through
    every tile shape: M = 27, 64, 100, 128, 160, 256, 384 rows, fused SwiGLU and split K, bf16 and 8-bit matrices."""
    from paper_2604_26779_amd import binding as sv
    before = sv.spec_tune_get("gemm_f16_inputs")
    sv.spec_tune_set("gemm_f16_inputs", mask)
    try:
        rng = np.random.default_rng(B + k)
        ctx = [int(c) for c in rng.integers(3, 150, size=B)]
        extra = dict(w_dtype="fp8_e4m3") if w8 else {}
        ok, max_err, worst = _run_custom_bf16(ctx, k=k, seed=B + k + mask, vocab=1000, **extra)
    finally:
        sv.spec_tune_set("gemm_f16_inputs", before)
    print("fp16-input projections %d, B=%d k=%d (M=%d), 8-bit matrices %s: logits max abs err %.3e" % (mask, B, k, B * (k + 1), w8, max_err))
    assert ok, (max_err, worst)


@pytest.mark.parametrize("workload", ["small_bf16_b5_k3", "tiny_fp32_b4_ctx128_k3"])
def test_bad_and_repeated_sequence_ids_are_dropped_and_the_rest_is_untouched(workload):
    """Batch entries whose sequence id (device memory, invisible to the host's checks) is out of range or names a
    sequence an earlier entry already names are left out of the step: the valid entries' logits still match the
    oracle, their pages and lengths move exactly as the oracle's book says, nothing else changes, and the cache reports
    the fault at the next state query."""
    from paper_2604_26779_amd import binding as sv
    wl, cfg, w_or, kv_or, batch, sess, seq_ids = _setup(workload, prefill="synthetic")
    k, ctx_len = wl["k"], batch["ctx_len"]
    rng = np.random.default_rng(3)
    ids = np.array([seq_ids[0], sess.max_seqs + 50, seq_ids[2], seq_ids[0], -4], dtype=np.int32)      # entries 1, 3, 4 are bad
    good = [0, 2]
    tokens = rng.integers(0, cfg["vocab"], size=(len(ids), k + 1)).astype(np.int32)
    before = sess.state()
    logits = sess.forward(torch.from_numpy(ids).cuda(), torch.from_numpy(tokens).cuda())
    torch.cuda.synchronize()
    assert torch.isfinite(logits[good]).all()
    want, _ = of.verify_forward(cfg, w_or, [[per[b] for b in good] for per in kv_or], tokens[good], ctx_len[good])
    ok, max_err, worst = logits_close(logits[good].cpu().numpy(), want, *TOL[cfg["dtype"]])
    assert ok, (max_err, worst)
    n = np.array([1, 2, 0, 3, 1], dtype=np.int32)
    new_len, slots = sess.commit(torch.from_numpy(ids).cuda(), torch.from_numpy(n).cuda(), k)
    book = _book(batch, sess, seq_ids, ctx_len)
    book.reserve([int(ids[b]) for b in good], k)
    want_len, want_slots = book.commit([int(ids[b]) for b in good], n[good], k)
    got_len, got_slots = new_len.cpu().numpy(), slots.cpu().numpy()
    for j, b in enumerate(good):
        assert got_len[b] == want_len[j] and list(got_slots[b]) == want_slots[j]
    for b in (1, 3, 4):
        assert got_len[b] == -1 and np.all(got_slots[b] == -1)
    with pytest.raises(sv.SpecError) as e:
        sess.state()
    assert e.value.status == sv.SPEC_EINVAL
    _check_state(sess, book, seq_ids)                      # the flag is cleared by the query; every sequence is where the book says
    after = sess.state()
    for s in [s for s in seq_ids if s not in (seq_ids[0], seq_ids[2])]:      # sequences no valid entry named: untouched
        assert after["ctx_len"][s] == before["ctx_len"][s] and after["n_pages"][s] == before["n_pages"][s]
    sess.close()


def test_replay_from_a_longer_cache_state_than_recorded_is_reported():
    """A recorded forward pass is sized for the longest context the host knew at recording time.  Replayed over
    longer contexts it cannot cover them: the cache must say so at the next state query instead of returning logits
    of truncated contexts unmarked."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["small_bf16"]
    weights = {n: t.cuda() for n, t in si.make_weights(cfg, seed=5).items()}
    sess = VerifySession(cfg, weights, max_seqs=2, max_ctx_len=512, n_pages=80)
    before = sv.spec_tune_get("attn_chunk_pages")
    sv.spec_tune_set("attn_chunk_pages", 4)               # one work item per 4 pages: the list is sized from the recorded lengths
    try:
        sess.pool.zero_()
        sess.assign(0, 40, [0, 1, 2])
        sess.assign(1, 20, [3, 4])
        ids = torch.arange(2, dtype=torch.int32, device="cuda")
        tok = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
        snap = torch.empty(sv.spec_kv_state_bytes(sess.kv), dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()
        sess.step_buffers(2, 3)
        with torch.cuda.stream(side):
            sv.spec_kv_snapshot(sess.kv, snap, side)
            sv.spec_graph_capture_begin(side)
            sv.spec_kv_restore(sess.kv, snap, side)
            sess.forward(ids, tok, stream=side)
            graph = sv.spec_graph_capture_end(side)
        torch.cuda.synchronize()
        sv.spec_graph_launch(graph, side)
        side.synchronize()
        sess.state()                                       # replay from the recorded state: no complaint
        sess.assign(0, 300, list(range(10, 29)))           # a much longer context under the same recording
        with torch.cuda.stream(side):
            sv.spec_kv_snapshot(sess.kv, snap, side)
        side.synchronize()
        sv.spec_graph_launch(graph, side)
        side.synchronize()
        with pytest.raises(sv.SpecError) as e:
            sess.state()
        assert e.value.status == sv.SPEC_ESTATE
        sv.spec_graph_destroy(graph)
    finally:
        sv.spec_tune_set("attn_chunk_pages", before)
        sess.close()


def test_long_random_walk_of_the_bookkeeping_against_the_oracle_book():
    """Sixty steps over 300 sequences with a different random subset, order, draft length and accept lengths each
    time, roll-backs to shorter lengths and to zero in between: after every call the lengths and slots the kernels
    report equal the oracle book's, and the whole state (page lists and the free stack, entry by entry) is compared
    every few steps.  More than 256 entries per call take the bookkeeping workgroup through several passes."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["tiny_fp32"]
    S, max_ctx, n_pages = 300, 160, 2600
    rng = np.random.default_rng(2024)
    sess = VerifySession(cfg, si.make_weights(cfg, seed=1, device="cuda"), max_seqs=S, max_ctx_len=max_ctx, n_pages=n_pages)
    sess.pool.normal_()
    book = oracle_commit.KVBook(n_pages, si.PAGE_SIZE)
    order = rng.permutation(n_pages)
    at = 0
    for s in range(S):
        c = int(rng.integers(0, 40))
        need = -(-c // si.PAGE_SIZE)
        pages = [int(p) for p in order[at:at + need]]
        at += need
        sess.assign(s, c, pages)
        book.assign(s, c, pages)
    all_ids = np.arange(S)
    for step in range(60):
        k = int(rng.integers(0, 4))
        room = np.array([s for s in range(S) if book.ctx_len[s] + k + 1 <= max_ctx])
        B = int(rng.integers(1, len(room) + 1))
        ids = rng.permutation(room)[:B].astype(np.int32)
        tokens = torch.randint(0, cfg["vocab"], (B, k + 1), dtype=torch.int32, device="cuda")
        d_ids = torch.from_numpy(ids).cuda()
        logits = sess.forward(d_ids, tokens)
        n = rng.integers(0, k + 1, size=B).astype(np.int32)
        book.reserve([int(s) for s in ids], k)
        new_len, slots = sess.commit(d_ids, torch.from_numpy(n).cuda(), k)
        want_len, want_slots = book.commit([int(s) for s in ids], n, k)
        assert new_len.cpu().numpy().tolist() == want_len and slots.cpu().numpy().tolist() == want_slots, step
        if step % 3 == 2:                                   # roll some back: a little, a lot, or to nothing
            Bt = int(rng.integers(1, S + 1))
            tids = rng.permutation(S)[:Bt].astype(np.int32)
            cur = np.array([book.ctx_len[int(s)] for s in tids])
            kind = rng.integers(0, 3, size=Bt)
            target = np.where(kind == 0, np.maximum(cur - rng.integers(0, 5, size=Bt), 0), np.where(kind == 1, cur // 2, 0)).astype(np.int32)
            out = torch.zeros(Bt, dtype=torch.int32, device="cuda")
            sv.spec_kv_truncate(sess.kv, Bt, torch.from_numpy(tids).cuda(), torch.from_numpy(target).cuda(), 0, out)
            assert out.cpu().numpy().tolist() == book.truncate([int(s) for s in tids], target), step
        if step % 5 == 4 or step == 59:
            assert torch.isfinite(logits).all()
            _check_state(sess, book, all_ids)
    held = sum(len(book.pages[s]) for s in range(S))
    assert held + len(book.free) == n_pages
    print("bookkeeping walk: %d pages held, %d free after 60 steps; longest sequence %d" % (held, len(book.free), max(book.ctx_len[s] for s in range(S))))
    sess.close()
