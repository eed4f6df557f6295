"""GPU parity of the continuous rollout's slot bookkeeping (spec_rollout_retire + spec_kv_truncate) against the CPU
oracle: slots, queue head, response counters, next-step inputs, page lists and the free stack are integers and must
match bit for bit at every step; the logits of every slot - including slots that were taken over by a waiting
sequence and idle ones - follow the oracle's forward over the caches as the oracle's book keeps them."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import commit as oracle_commit
from oracle import forward as of
from oracle import rollout as oro
from tests.helpers import logits_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,B,n_seqs,k", [(1, 4, 9, 3), (2, 6, 6, 2), (3, 3, 12, 5)])
def test_retire_backfill_chain(seed, B, n_seqs, k):
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["tiny_fp32"]
    rng = np.random.default_rng(seed)
    weights = si.make_weights(cfg, seed=seed)
    w_or = si.weights_for_oracle(cfg, weights)
    ctx0 = rng.integers(0, 40, size=n_seqs).astype(np.int64)
    kv0 = si.make_logical_kv(cfg, ctx0, seed=seed)                       # the waiting sequences' prompts are cached already
    kv_or = si.kv_for_oracle(kv0)
    n_pages = 64
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=n_seqs, max_ctx_len=512, n_pages=n_pages)
    book = oracle_commit.KVBook(n_pages=n_pages, page_size=si.PAGE_SIZE)
    order = [int(p) for p in rng.permutation(n_pages)]
    at = 0
    for s in range(n_seqs):
        need = -(-int(ctx0[s]) // si.PAGE_SIZE)
        pages = order[at:at + need]
        at += need
        sess.assign(s, int(ctx0[s]), pages)
        book.assign(s, int(ctx0[s]), pages)
        for l in range(cfg["n_layers"]):
            sess.write_logical_kv(l, pages, kv0[l][s][0], kv0[l][s][1])
    target = rng.integers(1, 14, size=n_seqs).astype(np.int32)
    first = rng.integers(0, cfg["vocab"], size=n_seqs).astype(np.int32)
    queue = np.arange(B, n_seqs, dtype=np.int32)
    # oracle state
    slot_seq = np.arange(B, dtype=np.int32)
    active = np.ones(B, dtype=np.int32)
    gen = np.zeros(n_seqs, dtype=np.int32)
    tokens = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
    tokens[:, 0] = first[:B]
    head, produced = 0, 0
    kv_cur = [[(kv_or[l][s][0].copy(), kv_or[l][s][1].copy()) for s in range(n_seqs)] for l in range(cfg["n_layers"])]
    ctx = ctx0.copy()
    # device state
    dev = lambda a, dt=torch.int32: torch.from_numpy(np.asarray(a)).to("cuda", dt)
    d_slot, d_active, d_gen = dev(slot_seq), dev(active), dev(gen)
    d_target, d_first, d_queue = dev(target), dev(first), (dev(queue) if len(queue) else None)
    d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_prod = torch.zeros(1, dtype=torch.int64, device="cuda")
    d_tok = dev(tokens)
    d_rel, d_keep = torch.zeros(B, dtype=torch.int32, device="cuda"), torch.zeros(B, dtype=torch.int32, device="cuda")
    steps = 0
    while active.any() and steps < 60:
        steps += 1
        seqs = [int(s) for s in slot_seq]
        kv_slots = [[kv_cur[l][s] for s in seqs] for l in range(cfg["n_layers"])]
        want, new_kv = of.verify_forward(cfg, w_or, kv_slots, tokens, ctx[seqs])
        logits = sess.forward(d_slot, d_tok)
        torch.cuda.synchronize()
        ok, max_err, worst = logits_close(logits.cpu().numpy(), want, 1e-4, 1e-4)
        assert ok, (steps, max_err, worst)
        n = rng.integers(0, k + 1, size=B).astype(np.int32)
        book.reserve(seqs, k)
        book.commit(seqs, n, k)
        d_n = dev(n)
        sess.commit(d_slot, d_n, k)
        for bi, s in enumerate(seqs):                                    # the kept positions join the oracle's caches
            for l in range(cfg["n_layers"]):
                K, V = kv_cur[l][s]
                kv_cur[l][s] = (np.concatenate([K, new_kv[l][0][bi][:n[bi] + 1]]), np.concatenate([V, new_kv[l][1][bi][:n[bi] + 1]]))
            ctx[s] += n[bi] + 1
        # next inputs: what the sampler would have emitted (forced here), fresh drafts; then the slot bookkeeping
        nxt = rng.integers(0, cfg["vocab"], size=(B, k + 1)).astype(np.int32)
        tokens = nxt.copy()
        d_tok.copy_(dev(nxt))
        rel, keep, head, made = oro.retire_and_backfill(slot_seq, active, n, k, gen, target, list(queue), head, first, tokens)
        produced += made
        sv.spec_rollout_retire(B, k, d_slot, d_active, d_n, d_gen, d_target, d_queue, d_head, d_first, d_tok, d_rel, d_keep, d_prod)
        sv.spec_kv_truncate(sess.kv, B, d_rel, d_keep, 0, None)
        book.truncate([int(s) for s in rel], [int(x) for x in keep])
        for b in range(B):
            if keep[b] == 0:
                s = int(rel[b])
                ctx[s] = 0
                for l in range(cfg["n_layers"]):
                    kv_cur[l][s] = (kv_cur[l][s][0][:0], kv_cur[l][s][1][:0])
        torch.cuda.synchronize()
        assert np.array_equal(d_slot.cpu().numpy(), slot_seq) and np.array_equal(d_active.cpu().numpy(), active), steps
        assert np.array_equal(d_gen.cpu().numpy(), gen) and int(d_head.item()) == head and int(d_prod.item()) == produced
        assert np.array_equal(d_tok.cpu().numpy(), tokens) and np.array_equal(d_rel.cpu().numpy(), rel)
        assert np.array_equal(d_keep.cpu().numpy(), keep)
        st = sess.state()
        for s in range(n_seqs):
            assert st["ctx_len"][s] == book.ctx_len[s], (steps, s)
            assert st["n_pages"][s] == len(book.pages[s]), (steps, s)
            assert list(st["page_table"][s][:len(book.pages[s])]) == book.pages[s], (steps, s)
        assert list(st["free_stack"]) == book.free, steps
    assert not active.any() and head == len(queue) and np.array_equal(gen, target) and produced == int(target.sum())
    print("B=%d, %d sequences, k=%d: drained in %d steps, %d tokens" % (B, n_seqs, k, steps, produced))
    sess.close()


def test_compaction_and_shrinking_batch():
    """spec_rollout_compact bit for bit against the oracle (more slots than one pass of the workgroup, none / all
    live), and a whole rollout with the n-gram drafter that compacts and shrinks its batch as slots go idle: every
    sequence still produces exactly its response length and ends with an empty cache."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.draft import ContinuousRollout
    from paper_2604_26779_amd.session import VerifySession
    rng = np.random.default_rng(11)
    for B, k, p_live in ((1, 0, 1.0), (5, 3, 0.5), (300, 2, 0.3), (64, 15, 0.0), (257, 1, 1.0), (600, 4, 0.7)):
        seq = rng.permutation(5000)[:B].astype(np.int32)
        act = (rng.random(B) < p_live).astype(np.int32)
        tok = rng.integers(0, 1 << 20, size=(B, k + 1)).astype(np.int32)
        s2, a2, t2, n = oro.compact_slots(seq, act, tok)
        d_seq, d_act, d_tok = (torch.from_numpy(x).cuda() for x in (seq, act, tok))
        d_n = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        sv.spec_rollout_compact(B, k, d_seq, d_act, d_tok, d_n, torch.empty(B * (k + 3), dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        assert int(d_n.item()) == n and np.array_equal(d_seq.cpu().numpy(), s2) and np.array_equal(d_act.cpu().numpy(), a2)
        assert np.array_equal(d_tok.cpu().numpy(), t2)
    # a rollout that shrinks: 12 slots, 20 sequences, tiny model
    cfg = si.MODELS["tiny_fp32"]
    slots, n_seqs, k = 12, 20, 2
    weights = si.make_weights(cfg, seed=4)
    ctx0 = rng.integers(1, 30, size=n_seqs).astype(np.int64)
    n_pages = 160
    sess = VerifySession(cfg, {n: t.cuda() for n, t in weights.items()}, max_seqs=n_seqs, max_ctx_len=256, n_pages=n_pages)
    sess.pool.normal_()
    at = 0
    for s in range(n_seqs):
        need = -(-int(ctx0[s]) // si.PAGE_SIZE)
        sess.assign(s, int(ctx0[s]), list(range(at, at + need)))
        at += need
    target = rng.integers(1, 25, size=n_seqs).astype(np.int32)
    cap = 128
    hist = torch.from_numpy(rng.integers(0, 5, size=(n_seqs, cap)).astype(np.int32)).cuda()
    hist_len = torch.from_numpy((ctx0 + 1).astype(np.int32)).cuda()
    first = hist[torch.arange(n_seqs, device="cuda"), (hist_len - 1).long()].contiguous()
    roll = ContinuousRollout(sess, slots, k, torch.arange(slots, dtype=torch.int32), torch.from_numpy(target),
                             torch.arange(slots, n_seqs, dtype=torch.int32), first)
    roll.tokens[:, 0] = first[:slots]
    sizes = []
    for chunk in range(40):
        roll.run(hist, hist_len, 4, 1.0, 99, chunk * 4)
        n_live = roll.compact(granule=4)
        sizes.append(roll.B_cur)
        if n_live == 0:
            break
    torch.cuda.synchronize()
    assert n_live == 0 and int(roll.produced.item()) == int(target.sum())
    assert np.array_equal(roll.gen_len.cpu().numpy(), target) and int(roll.queue_head.item()) == n_seqs - slots
    assert sizes[0] == slots and sizes[-1] == 4 and sorted(sizes, reverse=True) == sizes and len(set(sizes)) >= 3
    st = sess.state()
    assert np.all(st["ctx_len"][:n_seqs] == 0) and np.all(st["n_pages"][:n_seqs] == 0) and len(st["free_stack"]) == n_pages
    print("shrinking rollout: batch sizes", sizes, "tokens", int(roll.produced.item()))
    sess.close()


def test_backfilled_slots_get_their_own_pending_pair_and_a_pair_rollout_drains():
    """spec_rollout_pending bit for bit against the oracle on random slot tables (kept, taken-over and idle slots, more
    slots than one workgroup), and a whole continuous rollout with a draft model (tiny pair, slots taken over several
    times): every sequence produces exactly its response length, both caches end empty with every page back on the
    free stacks, and at every step a live slot's draft cache is one position behind its verifier cache."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.draft import ContinuousPairRollout
    from paper_2604_26779_amd.session import VerifySession
    rng = np.random.default_rng(21)
    for B, n_seqs, p_change, p_live in ((1, 3, 1.0, 1.0), (7, 40, 0.5, 0.7), (300, 900, 0.3, 0.5), (513, 600, 0.0, 1.0)):
        before = rng.permutation(n_seqs)[:B].astype(np.int32)
        after = before.copy()
        spare = [s for s in range(n_seqs) if s not in set(before.tolist())]
        for b in range(B):
            if spare and rng.random() < p_change:
                after[b] = spare.pop()
        active = (rng.random(B) < p_live).astype(np.int32)
        prev = rng.integers(0, 1 << 20, size=n_seqs).astype(np.int32)
        first = rng.integers(0, 1 << 20, size=n_seqs).astype(np.int32)
        pending = rng.integers(0, 1 << 20, size=(B, 2)).astype(np.int32)
        want = pending.copy()
        oro.backfill_pending(want, before, after, active, prev, first)
        d = lambda a: torch.from_numpy(a).cuda()
        d_pending = d(pending)
        sv.spec_rollout_pending(B, d(before), d(after), d(active), d(prev), d(first), d_pending)
        torch.cuda.synchronize()
        assert np.array_equal(d_pending.cpu().numpy(), want)

    cfg_t, cfg_d = si.MODELS["tiny_fp32"], si.MODELS["draft_tiny_fp32"]
    slots, n_seqs, k = 5, 13, 3
    ctx0 = rng.integers(2, 40, size=n_seqs).astype(np.int64)
    n_pages = 160
    tsess = VerifySession(cfg_t, {n: t.cuda() for n, t in si.make_weights(cfg_t, seed=5).items()}, max_seqs=n_seqs, max_ctx_len=256,
                          n_pages=n_pages)
    dsess = VerifySession(cfg_d, {n: t.cuda() for n, t in si.make_weights(cfg_d, seed=6).items()}, max_seqs=n_seqs, max_ctx_len=256,
                          n_pages=n_pages)
    tsess.pool.normal_()
    dsess.pool.normal_()
    at = dat = 0
    for s in range(n_seqs):                               # prompts cached: the draft's cache one position behind
        need, dneed = -(-int(ctx0[s]) // si.PAGE_SIZE), -(-int(ctx0[s] - 1) // si.PAGE_SIZE)
        tsess.assign(s, int(ctx0[s]), list(range(at, at + need)))
        dsess.assign(s, int(ctx0[s]) - 1, list(range(dat, dat + dneed)))
        at += need
        dat += dneed
    target = rng.integers(1, 18, size=n_seqs).astype(np.int32)
    prev = torch.from_numpy(rng.integers(0, cfg_t["vocab"], size=n_seqs).astype(np.int32))
    first = torch.from_numpy(rng.integers(0, cfg_t["vocab"], size=n_seqs).astype(np.int32))
    roll = ContinuousPairRollout(tsess, dsess, slots, k, torch.arange(slots, dtype=torch.int32), torch.from_numpy(target),
                                 torch.arange(slots, n_seqs, dtype=torch.int32), prev, first)
    live = torch.zeros(1, dtype=torch.int32, device="cuda")
    steps = 0
    while steps < 200:
        roll.run(1, 1.0, 77, steps, live_out=live)
        steps += 1
        torch.cuda.synchronize()
        ts, ds = tsess.state(), dsess.state()
        slot_seq, active = roll.slot_seq.cpu().numpy(), roll.active.cpu().numpy()
        for b in range(slots):
            s = int(slot_seq[b])
            if active[b]:
                assert ds["ctx_len"][s] == ts["ctx_len"][s] - 1, (steps, b, s)
                assert list(roll.pending[b].cpu().numpy())[1] == int(roll.tokens[b, 0].item())
            else:
                assert ts["ctx_len"][s] == 0 and ds["ctx_len"][s] == 0
        if int(live.item()) == 0:
            break
    assert int(live.item()) == 0 and int(roll.produced.item()) == int(target.sum())
    assert np.array_equal(roll.gen_len.cpu().numpy(), target) and int(roll.queue_head.item()) == n_seqs - slots
    for st in (tsess.state(), dsess.state()):
        assert np.all(st["ctx_len"][:n_seqs] == 0) and np.all(st["n_pages"][:n_seqs] == 0) and len(st["free_stack"]) == n_pages
    print("pair rollout: %d slots, %d sequences, drained in %d steps, %d tokens" % (slots, n_seqs, steps, int(roll.produced.item())))
    tsess.close()
    dsess.close()


def test_hidden_state_pairs_follow_taken_over_slots_and_a_fused_pair_rollout_drains():
    """spec_rollout_pending_hidden bit for bit against the oracle on random slot tables, and a whole continuous rollout
    whose draft model takes the verifier's hidden states (small bf16 pair, slots taken over several times): every
    sequence produces exactly its response length, both caches end empty, at every step a live slot's draft cache is one
    position behind its verifier cache, and a slot that was just taken over carries its new sequence's own hidden states."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.draft import ContinuousPairRollout
    from paper_2604_26779_amd.session import VerifySession
    rng = np.random.default_rng(31)
    for B, n_seqs, d, p_change, p_live in ((1, 3, 8, 1.0, 1.0), (7, 40, 512, 0.5, 0.7), (300, 900, 64, 0.3, 0.5)):
        before = rng.permutation(n_seqs)[:B].astype(np.int32)
        after = before.copy()
        spare = [s for s in range(n_seqs) if s not in set(before.tolist())]
        for b in range(B):
            if spare and rng.random() < p_change:
                after[b] = spare.pop()
        active = (rng.random(B) < p_live).astype(np.int32)
        seq_hidden = rng.standard_normal((n_seqs, 2, d)).astype(np.float32)
        ph = rng.standard_normal((B, 2, d)).astype(np.float32)
        want = ph.copy()
        oro.backfill_pending_hidden(want, before, after, active, seq_hidden)
        dv = lambda a: torch.from_numpy(a).cuda()
        d_ph = dv(ph)
        sv.spec_rollout_pending_hidden(B, dv(before), dv(after), dv(active), dv(seq_hidden), d_ph)
        torch.cuda.synchronize()
        assert np.array_equal(d_ph.cpu().numpy(), want)

    for target_name, draft_name, taps in (("small_bf16", "draft_fused_small_bf16", None), ("small4_bf16", "draft_eagle3_small_bf16", (1, 2, 4)),
                                          ("small4_bf16", "draft_eagle3r_small_bf16", (1, 2, 4))):       # the last: a head over a subset of the tokens
        _drain_fused_pair(rng, target_name, draft_name, taps)


def _drain_fused_pair(rng, target_name, draft_name, taps):
    """taps: the target layers a feature-fed draft is given (then every hidden-state pair is len(taps) * d wide)."""
    from paper_2604_26779_amd.draft import ContinuousPairRollout
    from paper_2604_26779_amd.session import VerifySession
    cfg_t, cfg_d = si.MODELS[target_name], si.MODELS[draft_name]
    slots, n_seqs, k = 4, 10, 3
    ctx0 = rng.integers(2, 60, size=n_seqs).astype(np.int64)
    n_pages = 160
    tsess = VerifySession(cfg_t, {n: t.cuda() for n, t in si.make_weights(cfg_t, seed=5).items()}, max_seqs=n_seqs, max_ctx_len=256,
                          n_pages=n_pages)
    dsess = VerifySession(cfg_d, {n: t.cuda() for n, t in si.make_weights(cfg_d, seed=6).items()}, max_seqs=n_seqs, max_ctx_len=256,
                          n_pages=n_pages)
    tsess.pool.normal_()
    dsess.pool.normal_()
    at = dat = 0
    for s in range(n_seqs):                               # prompts cached: the draft's cache one position behind
        need, dneed = -(-int(ctx0[s]) // si.PAGE_SIZE), -(-int(ctx0[s] - 1) // si.PAGE_SIZE)
        tsess.assign(s, int(ctx0[s]), list(range(at, at + need)))
        dsess.assign(s, int(ctx0[s]) - 1, list(range(dat, dat + dneed)))
        at += need
        dat += dneed
    target = rng.integers(1, 14, size=n_seqs).astype(np.int32)
    prev = torch.from_numpy(rng.integers(0, cfg_t["vocab"], size=n_seqs).astype(np.int32))
    first = torch.from_numpy(rng.integers(0, cfg_t["vocab"], size=n_seqs).astype(np.int32))
    seq_hidden = torch.from_numpy(rng.standard_normal((n_seqs, 2, cfg_t["d_model"] * (len(taps) if taps else 1))).astype(np.float32))
    roll = ContinuousPairRollout(tsess, dsess, slots, k, torch.arange(slots, dtype=torch.int32), torch.from_numpy(target),
                                 torch.arange(slots, n_seqs, dtype=torch.int32), prev, first, seq_hidden=seq_hidden, tap_layers=taps,
                                 token_map=torch.from_numpy(si.make_token_map(cfg_d, seed=7)).cuda() if cfg_d.get("head_vocab", 0) else None)
    live = torch.zeros(1, dtype=torch.int32, device="cuda")
    steps, taken_over = 0, 0
    while steps < 200:
        seq_before = roll.slot_seq.cpu().numpy().copy()
        roll.run(1, 1.0, 78, steps, live_out=live)
        steps += 1
        torch.cuda.synchronize()
        ts, ds = tsess.state(), dsess.state()
        slot_seq, active = roll.slot_seq.cpu().numpy(), roll.active.cpu().numpy()
        for b in range(slots):
            s = int(slot_seq[b])
            if active[b]:
                assert ds["ctx_len"][s] == ts["ctx_len"][s] - 1, (steps, b, s)
                assert int(roll.pending[b, 1].item()) == int(roll.tokens[b, 0].item())
                if s != int(seq_before[b]):
                    assert torch.equal(roll.pending_hidden[b].cpu(), seq_hidden[s])
                    taken_over += 1
                assert torch.isfinite(roll.pending_hidden[b]).all()
                assert 0 <= int(roll.tokens[b, 0].item()) < cfg_t["vocab"]
            else:
                assert ts["ctx_len"][s] == 0 and ds["ctx_len"][s] == 0
        if int(live.item()) == 0:
            break
    assert int(live.item()) == 0 and int(roll.produced.item()) == int(target.sum()) and taken_over == n_seqs - slots
    assert np.array_equal(roll.gen_len.cpu().numpy(), target) and int(roll.queue_head.item()) == n_seqs - slots
    for st in (tsess.state(), dsess.state()):
        assert np.all(st["ctx_len"][:n_seqs] == 0) and np.all(st["n_pages"][:n_seqs] == 0) and len(st["free_stack"]) == n_pages
    print("fused pair rollout (%s): %d slots, %d sequences, drained in %d steps, %d tokens" % (draft_name, slots, n_seqs, steps, int(roll.produced.item())))
    tsess.close()
    dsess.close()
