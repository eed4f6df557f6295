"""Full-size parity of the Llama-3-8B-shaped verify step in the launch configurations bench.py times:
B=32, contexts 1024..8192, k=3, and the large rollout batch B=256, contexts 2048..16384, k=7 and k=1
(bf16, shuffled 16-token pages; the large batch on 8 aliased layer pools, which the oracle sees as
layers l and l+8 reading the same cached context).

The CPU oracle cannot run all 32 sequences in a test's time, and a sequence's logits depend only on
its own rows and its own cache, so the logits are checked on sampled sequences (the shortest and
the longest context: fewest and most attention chunks) computed by the oracle one sequence at a
time, within 2e-2 abs + 1e-2 rel.  Inputs are the seeded generator's: weights N(0, 0.02) in bf16,
cache N(0, 1) in bf16 (a real prefill of 150k tokens is out of the oracle's reach), tokens uniform.
The sampler at this vocabulary and batch size is covered on generator-made logits in
test_gpu_sampler.py; the commit is checked here against the oracle's book with seeded accept lengths.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import commit as oracle_commit
from oracle import forward as of
from tests.helpers import logits_close

pytestmark = pytest.mark.gpu

def _check_workload(name, ks, moe_margin=None):
    from paper_2604_26779_amd.workloads import DeviceWorkload
    wl = DeviceWorkload(name)
    cfg, B = wl.cfg, wl.B
    rng = np.random.default_rng(123)
    picks = sorted({int(np.argmin(wl.ctx_len)), int(np.argmax(wl.ctx_len))} | ({3, 17, 40, 99} if moe_margin is not None else set()))
    weights = si.make_weights(cfg, seed=wl.seed, device="cuda")           # the generator's weights again, for the oracle
    w_or = si.weights_for_oracle(cfg, weights)
    del weights
    torch.cuda.empty_cache()
    kv_or = [[tuple(t.float().cpu().numpy() for t in wl.logical_kv(l, b)) for b in picks] for l in range(cfg["n_layers"])]
    seq_ids = wl.seq_ids
    for k in ks:
        wl.restore()
        tokens = np.concatenate([wl.batch["tokens0"][:, None], rng.integers(0, cfg["vocab"], size=(B, k))], axis=1).astype(np.int32)
        logits = wl.sess.forward(seq_ids, torch.from_numpy(tokens).cuda())
        torch.cuda.synchronize()
        assert torch.isfinite(logits).all()
        print(name, "k=%d: oracle on sequences" % k, picks, "contexts", [int(wl.ctx_len[b]) for b in picks], flush=True)
        log = []
        want, new_kv = of.verify_forward(cfg, w_or, kv_or, tokens[picks], wl.ctx_len[picks], route_log=log)
        got = logits[picks].cpu().numpy()
        if moe_margin is not None:
            # rows whose expert choice the oracle decides by less than the margin (and the rows after them in the
            # sequence) may legitimately differ: counted, reported, left out of the comparison
            fragile = np.zeros((len(picks), k + 1), dtype=bool)
            for experts, weight, prob in log:
                srt = np.sort(np.log(prob), axis=-1)[:, ::-1]
                fragile |= ((srt[:, cfg["top_k"] - 1] - srt[:, cfg["top_k"]]) < moe_margin).reshape(len(picks), k + 1)
            keep = ~np.logical_or.accumulate(fragile, axis=1)
            print("  rows exempted for routing margins: %d of %d" % ((~keep).sum(), keep.size), flush=True)
            assert keep.sum() >= keep.size // 2
            got, want = got[keep], want[keep]
        ok, max_err, worst = logits_close(got, want, 2e-2, 1e-2)
        print("  logits max abs err %.3e, |logit| max %.2f" % (max_err, np.abs(want).max()), flush=True)
        assert ok, (max_err, worst)

        # new cache entries of the sampled sequences (last layer) sit where the page table says
        book = oracle_commit.KVBook(wl.sess.n_pages, si.PAGE_SIZE)
        for b in range(B):
            book.assign(b, int(wl.ctx_len[b]), wl.batch["page_lists"][b])
        book.reserve(list(range(B)), k)
        last = cfg["n_layers"] - 1
        for j, b in enumerate(picks):
            K, V = wl.sess.read_logical_kv(last, book.pages[b], int(wl.ctx_len[b]) + k + 1)
            c = int(wl.ctx_len[b])
            assert np.max(np.abs(K[c:].float().cpu().numpy() - new_kv[last][0][j])) < 2e-2 * max(1.0, np.abs(new_kv[last][0][j]).max())
            assert np.max(np.abs(V[c:].float().cpu().numpy() - new_kv[last][1][j])) < 2e-2 * max(1.0, np.abs(new_kv[last][1][j]).max())

        # commit at full batch size with seeded accept lengths against the oracle's book
        n = rng.integers(0, k + 1, size=B).astype(np.int32)
        new_len, slots = wl.sess.commit(seq_ids, torch.from_numpy(n).cuda(), k)
        want_len, want_slots = book.commit(list(range(B)), n, k)
        assert list(new_len.cpu().numpy()) == want_len
        assert slots.cpu().numpy().tolist() == want_slots
        st = wl.sess.state()
        assert list(st["ctx_len"][:B]) == want_len and list(st["free_stack"]) == book.free
    wl.close()
    del wl
    torch.cuda.empty_cache()


def test_llama8b_logits_on_sampled_sequences_and_commit():
    _check_workload("llama8b_b32_ctx1k-8k_k3", [3])


def test_llama8b_large_batch_aliased_pool_k7_and_k1():
    _check_workload("llama8b_b256_ctx2k-16k_k7", [7, 1])


def test_moe_slice_full_size():
    """4 mixture-of-experts layers at 235B-A22B widths (128 experts, top-8), B = 128, contexts 4096..32768, k = 3."""
    _check_workload("moe235b_slice_b128_ctx4k-32k_k3", [3], moe_margin=1e-3)
