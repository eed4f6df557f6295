"""GPU parity of the model-free n-gram drafter (spec_ngram_draft / spec_ngram_append) against the CPU oracle:
integer work, bit-exact.  Histories use small vocabularies so that repeated n-grams are common; lengths span
empty, one token, shorter than n_min + 1, and several thousand tokens (many passes of the workgroup's stride)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import forward as of
from oracle import ngram as oracle_ngram
from oracle import sampler as oracle_sampler
from tests.helpers import assert_sampler_parity, logits_close, random_norm_gains

pytestmark = pytest.mark.gpu


def _histories(rng, lengths, cap, vocab):
    hist = rng.integers(0, vocab, size=(len(lengths), cap)).astype(np.int32)      # beyond a row's length: stale tokens
    return hist, np.array(lengths, dtype=np.int32)


@pytest.mark.parametrize("k,n_max,n_min,vocab", [(3, 3, 1, 4), (5, 4, 2, 3), (7, 16, 1, 2), (0, 2, 1, 5), (15, 5, 5, 2),
                                                 (3, 3, 1, 50000)])
def test_ngram_draft_parity(k, n_max, n_min, vocab):
    from paper_2604_26779_amd import binding as sv
    rng = np.random.default_rng(k * 100 + n_max)
    lengths = [0, 1, 2, 3, n_min, n_min + 1, 17, 255, 256, 257, 258, 1000, 4097, 6000] + [int(x) for x in rng.integers(1, 3000, size=20)]
    cap = 6000
    hist, hist_len = _histories(rng, lengths, cap, vocab)
    # a row that is one token repeated (every position matches), one strictly increasing (no match at all)
    hist[15, :] = 1
    hist[16, :] = np.arange(cap)
    n_rows = len(lengths)
    B = n_rows + 2
    seq_ids = np.concatenate([rng.permutation(n_rows), [-1, n_rows]]).astype(np.int32)       # two invalid rows at the end
    want_d, want_c = oracle_ngram.ngram_draft(hist[seq_ids[:n_rows]], hist_len[seq_ids[:n_rows]].clip(1), k, n_max, n_min)
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_drafted = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    sv.spec_ngram_draft(B, k, n_max, n_min, torch.from_numpy(hist).cuda(), torch.from_numpy(hist_len).cuda(),
                        torch.from_numpy(seq_ids).cuda(), tokens, n_drafted)
    torch.cuda.synchronize()
    tokens, n_drafted = tokens.cpu().numpy(), n_drafted.cpu().numpy()
    some_match = 0
    for b in range(n_rows):
        r = seq_ids[b]
        if hist_len[r] == 0:
            assert n_drafted[b] == -1 and np.all(tokens[b] == 0)
            continue
        assert tokens[b, 0] == hist[r, hist_len[r] - 1]
        assert n_drafted[b] == want_c[b], (b, r, hist_len[r], n_drafted[b], want_c[b])
        assert np.array_equal(tokens[b, 1:], want_d[b]), (b, r, hist_len[r])
        some_match += int(want_c[b] > 0)
    assert np.all(n_drafted[n_rows:] == -1) and np.all(tokens[n_rows:] == 0)
    if vocab <= 5 and k > 0 and n_min < 5:
        assert some_match > n_rows // 2
    print("k=%d n=%d..%d vocab=%d: %d of %d rows found an occurrence" % (k, n_min, n_max, vocab, some_match, n_rows))
    # batch entry b = row b when no sequence ids are given
    tokens2 = torch.full((n_rows, k + 1), -5, dtype=torch.int32, device="cuda")
    sv.spec_ngram_draft(n_rows, k, n_max, n_min, torch.from_numpy(hist).cuda(), torch.from_numpy(hist_len).cuda(), None, tokens2, None)
    torch.cuda.synchronize()
    inv = np.argsort(seq_ids[:n_rows])
    assert np.array_equal(tokens2.cpu().numpy(), tokens[:n_rows][inv])


def test_ngram_rollout_history_chain():
    """Six steps of draft -> (forced verdict) -> append on device and in the oracle: the histories, their lengths
    (one row saturates) and every step's drafts stay identical."""
    from paper_2604_26779_amd import binding as sv
    rng = np.random.default_rng(5)
    B, k, cap, vocab = 9, 4, 64, 3
    lengths = [1, 5, 20, 40, 58, 61, 63, 64, 33]
    hist, hist_len = _histories(rng, lengths, cap, vocab)
    d_hist, d_len = torch.from_numpy(hist).cuda(), torch.from_numpy(hist_len).cuda()
    seq_ids = rng.permutation(B).astype(np.int32)
    d_seq = torch.from_numpy(seq_ids).cuda()
    tokens = torch.zeros((B, k + 1), dtype=torch.int32, device="cuda")
    for step in range(6):
        want_d, want_c = oracle_ngram.ngram_draft(hist[seq_ids], hist_len[seq_ids], k, 3, 1)
        c = torch.zeros(B, dtype=torch.int32, device="cuda")
        sv.spec_ngram_draft(B, k, 3, 1, d_hist, d_len, d_seq, tokens, c)
        torch.cuda.synchronize()
        assert np.array_equal(tokens.cpu().numpy()[:, 1:], want_d) and np.array_equal(c.cpu().numpy(), want_c), step
        n = rng.integers(0, k + 1, size=B).astype(np.int32)
        out = np.concatenate([want_d, np.zeros((B, 1), np.int32)], axis=1)
        for b in range(B):
            out[b, n[b]] = rng.integers(0, vocab)                     # the emitted token after the accepted prefix
        sv.spec_ngram_append(B, k, d_hist, d_len, d_seq, torch.from_numpy(out).cuda(), torch.from_numpy(n).cuda())
        h2, l2 = hist[seq_ids].copy(), hist_len[seq_ids].copy()
        oracle_ngram.append_emitted(h2, l2, out, n)
        hist[seq_ids], hist_len[seq_ids] = h2, l2
        torch.cuda.synchronize()
        assert np.array_equal(d_len.cpu().numpy(), hist_len), step
        got = d_hist.cpu().numpy()
        for r in range(B):
            assert np.array_equal(got[r, :hist_len[r]], hist[r, :hist_len[r]]), (step, r)
    assert hist_len.max() == cap


def test_ngram_step_end_to_end():
    """One whole step with the n-gram drafter on the small bf16 model: drafts from histories (bit-exact), verify
    forward (logits tolerance), rejection sampling with point-mass drafts (no q array) and the history update."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = dict(si.MODELS["small_bf16"], vocab=1000)
    B, k, cap = 6, 3, 256
    rng = np.random.default_rng(9)
    ctx_len = np.array([20, 37, 64, 100, 129, 200], dtype=np.int64)
    # histories = the cached context's tokens + the pending token, drawn from 6 distinct tokens so that n-grams repeat
    alphabet = rng.choice(cfg["vocab"], size=6, replace=False)
    hist = np.zeros((B, cap), dtype=np.int32)
    hist_len = (ctx_len + 1).astype(np.int32)
    for b in range(B):
        hist[b, :hist_len[b]] = alphabet[rng.integers(0, 6, size=hist_len[b])]
    weights = random_norm_gains(si.make_weights(cfg, seed=9), 9)
    w_or = si.weights_for_oracle(cfg, weights)
    kv = si.make_logical_kv(cfg, ctx_len, seed=9)
    kv_or = si.kv_for_oracle(kv)
    n_pages = sum(-(-(int(c) + k + 1) // si.PAGE_SIZE) for c in ctx_len) + 8
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=B, max_ctx_len=int(ctx_len.max()) + 64, n_pages=n_pages)
    at = 0
    for b in range(B):
        need = -(-int(ctx_len[b]) // si.PAGE_SIZE)
        pages = list(range(at, at + need))
        at += need
        sess.assign(b, int(ctx_len[b]), pages)
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, pages, kv[l][b][0], kv[l][b][1])
    # oracle side
    drafts, c = oracle_ngram.ngram_draft(hist, hist_len, k, 3, 1)
    tokens_or = np.concatenate([hist[np.arange(B), hist_len - 1][:, None], drafts], axis=1).astype(np.int32)
    logits_or, _ = of.verify_forward(cfg, w_or, kv_or, tokens_or, ctx_len)
    q = np.zeros((B, k, cfg["vocab"]), dtype=np.float32)
    np.put_along_axis(q, drafts[:, :, None].astype(np.int64), 1.0, axis=2)
    seed, step, T = 123, 0, 1.0
    n_or, out_or, pqu, keys = oracle_sampler.reject_sample(logits_or.astype(np.float32), q, drafts, T, seed, step, debug=True)
    # device side
    d_hist, d_len = torch.from_numpy(hist).cuda(), torch.from_numpy(hist_len).cuda()
    d_seq = torch.arange(B, dtype=torch.int32, device="cuda")
    d_tok = torch.zeros((B, k + 1), dtype=torch.int32, device="cuda")
    sv.spec_ngram_draft(B, k, 3, 1, d_hist, d_len, d_seq, d_tok, None)
    logits, n_gpu, out_gpu = sess.step(d_seq, d_tok, None, d_tok[:, 1:].contiguous(), T, seed, step)
    sv.spec_ngram_append(B, k, d_hist, d_len, d_seq, out_gpu, n_gpu)
    torch.cuda.synchronize()
    assert np.array_equal(d_tok.cpu().numpy(), tokens_or)
    ok, max_err, worst = logits_close(logits.cpu().numpy(), logits_or, 2e-2, 1e-2)
    assert ok, (max_err, worst)
    # the sampler decides on the device's logits: compare through the oracle run on those (decisions near a
    # threshold are exempted and counted, as in the sampler's own parity tests)
    assert_sampler_parity(n_gpu.cpu().numpy(), out_gpu.cpu().numpy(), n_or, out_or, pqu, keys, max_exempt_frac=0.5)
    n_np, out_np = n_gpu.cpu().numpy(), out_gpu.cpu().numpy()
    h2, l2 = hist.copy(), hist_len.copy()
    oracle_ngram.append_emitted(h2, l2, out_or, n_or)         # the oracle's own verdict
    got_h, got_l = d_hist.cpu().numpy(), d_len.cpu().numpy()
    for b in range(B):                                        # rows whose verdict was not an exempted near-threshold one
        if n_np[b] == n_or[b] and np.array_equal(out_np[b], out_or[b]):
            assert got_l[b] == l2[b] and np.array_equal(got_h[b], h2[b]), b
        assert got_l[b] == hist_len[b] + n_np[b] + 1
    print("n-gram step: drafted %s, accepted %s, logits max abs err %.3e" % (c.tolist(), n_np.tolist(), max_err))
    sess.close()
