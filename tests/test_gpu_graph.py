"""A recorded verify step (cache restore + forward + rejection sampling + commit) replayed as a graph must give,
on every replay, exactly what the same calls give when launched one by one - also with other eager work and
synchronisations between the replays.  The headline workload is among the cases because bench.py times its steps as
a replay: the eager launches that the full-size parity tests check and the replayed ones must agree bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["small_bf16_b5_k3", "tiny_fp32_b4_ctx128_k3", "llama8b_b32_ctx1k-8k_k3"])
def test_replayed_step_equals_eager_step(name):
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.workloads import DeviceWorkload
    wl = DeviceWorkload(name)
    wl.make_drafts()
    B, k, T = wl.B, wl.k, wl.wl["temperature"]
    draft = wl.tokens[:, 1:].contiguous()
    buf = wl.sess.step_buffers(B, k)

    def snapshot_outputs():
        torch.cuda.synchronize()
        st = wl.sess.state()
        return (buf["logits"].clone(), buf["accept_len"].clone(), buf["out_tokens"].clone(), buf["new_ctx_len"].clone(),
                buf["commit_slots"].clone(), st["ctx_len"].copy(), st["free_stack"].copy())

    def one_step(stream, step):
        wl.restore(stream)
        wl.sess.step(wl.seq_ids, wl.tokens, wl.q, draft, T, wl.seed, step, stream=stream)

    results = {}
    for step in (7, 8):
        one_step(None, step)
        results[step] = snapshot_outputs()
    assert not torch.equal(results[7][2], results[8][2]) or k == 0          # different random counters, different draws

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        sv.spec_graph_capture_begin(side)
        one_step(side, 7)
        one_step(side, 8)                                                 # two steps in one recording, the second one's results stay
        graph = sv.spec_graph_capture_end(side)
    torch.cuda.synchronize()
    other_tokens = torch.randint(0, wl.cfg["vocab"], (B, k + 1), dtype=torch.int32, device="cuda")
    for rep in range(4):
        for t in buf.values():
            if t.dtype != torch.uint8:
                t.fill_(-3)                                               # stale outputs would show
        torch.cuda.synchronize()
        sv.spec_graph_launch(graph, side)
        side.synchronize()
        got = snapshot_outputs()
        for a, b in zip(got, results[8]):
            if isinstance(a, torch.Tensor):
                assert torch.equal(a, b), ("replay %d differs from the eager step" % rep)
            else:
                assert np.array_equal(a, b), ("replay %d differs from the eager step" % rep)
        # eager work between the replays: another forward on the default stream, a cache state change, a sync
        wl.restore(None)
        wl.sess.forward(wl.seq_ids, other_tokens)
        torch.cuda.synchronize()
    sv.spec_graph_destroy(graph)
    with pytest.raises(sv.SpecError):
        sv.spec_graph_capture_begin(None)                                 # the default stream cannot record
    wl.close()


@pytest.mark.parametrize("name", ["draft_pair_small_b5_k4", "draft_pair_fused_small_b5_k4", "draft_pair_eagle3_small_b5_k4",
                                  "draft_pair_eagle3r_small_b5_k4"])
def test_replayed_pair_rollout_equals_the_eager_one(name):
    """Three consecutive steps of a draft + verify pair (draft loop, verify forward, rejection sampling, commit, roll-back of
    the draft's cache, next inputs - with the draft's hidden-state or feature input and its reduced vocabulary where the
    workload has them) recorded once: every replay, with eager work and synchronisations in between, gives the accept
    lengths, emitted tokens and cache lengths of the same calls launched one by one."""
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.draft import RolloutLoop
    from paper_2604_26779_amd.workloads import DraftPairWorkload
    wl = DraftPairWorkload(name)
    B, k, T, S = wl.B, wl.k, wl.wl["temperature"], 3
    roll = RolloutLoop(wl.sess, wl.dsess, B, k, tap_layers=wl.tap_layers, token_map=wl.token_map)
    acc = torch.zeros((S, B), dtype=torch.int32, device="cuda")
    out = torch.zeros((S, B, k + 1), dtype=torch.int32, device="cuda")

    def begin(stream=None):
        wl.restore(stream)
        roll.start(wl.pending[:, 0].contiguous(), wl.pending[:, 1].contiguous(), wl.pending_hidden)

    def outputs():
        torch.cuda.synchronize()
        return (acc.clone(), out.clone(), wl.sess.state()["ctx_len"].copy(), wl.dsess.state()["ctx_len"].copy(),
                wl.dsess.state()["free_stack"].copy(), roll.pending.clone())

    begin()
    roll.run(wl.seq_ids, S, T, wl.seed, 40, acc, out)
    want = outputs()
    assert int(want[0].sum()) > 0                                         # some drafts were accepted

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        begin(side)
        side.synchronize()
        wl.sess.state(), wl.dsess.state()                                 # the host mirrors are current: no read-back while recording
        sv.spec_graph_capture_begin(side)
        roll.run(wl.seq_ids, S, T, wl.seed, 40, acc, out, stream=side)
        graph = sv.spec_graph_capture_end(side)
    torch.cuda.synchronize()
    for rep in range(3):
        acc.fill_(-3)
        out.fill_(-3)
        with torch.cuda.stream(side):
            begin(side)
            sv.spec_graph_launch(graph, side)
            side.synchronize()
        got = outputs()
        for a, b in zip(got, want):
            same = torch.equal(a, b) if isinstance(a, torch.Tensor) else np.array_equal(a, b)
            assert same, "replay %d differs from the eager rollout" % rep
        begin()                                                           # eager work between the replays
        roll.run(wl.seq_ids, 1, T, wl.seed, 77)
        torch.cuda.synchronize()
    sv.spec_graph_destroy(graph)
    wl.close()


def test_forward_under_capture_never_synchronises():
    """When the host's bounds cannot show that the step fits, an eager call reads the cache state back (a
    synchronisation); a call on a stream that is being captured must not - it reports SPEC_ESTATE with nothing recorded,
    the capture stays valid, and after spec_kv_get_state the same step records and replays."""
    import synth_inputs as si
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS["tiny_fp32"]
    B, k = 2, 3
    sess = VerifySession(cfg, si.make_weights(cfg, seed=1, device="cuda"), max_seqs=B, max_ctx_len=64, n_pages=8)
    sess.pool.normal_()
    for b in range(B):
        sess.assign(b, 5, [b])
    seq = torch.arange(B, dtype=torch.int32, device="cuda")
    tokens = torch.randint(0, cfg["vocab"], (B, k + 1), dtype=torch.int32, device="cuda")
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    for _ in range(3):                                  # eager steps that keep one position each: the bounds drift upwards
        sess.forward(seq, tokens)
        sess.commit(seq, zero, k)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        sv.spec_graph_capture_begin(side)
        with pytest.raises(sv.SpecError) as e:
            sess.forward(seq, tokens, stream=side)
        assert e.value.status == sv.SPEC_ESTATE
        graph = sv.spec_graph_capture_end(side)         # the recording is still alive (and empty)
        sv.spec_graph_destroy(graph)
    st = sess.state()                                   # exact bounds again
    assert list(st["ctx_len"][:B]) == [8, 8]
    with torch.cuda.stream(side):
        sv.spec_graph_capture_begin(side)
        logits = sess.forward(seq, tokens, stream=side)
        graph = sv.spec_graph_capture_end(side)
        sv.spec_graph_launch(graph, side)
        side.synchronize()
    a = logits.clone()
    sess.commit(seq, zero, k)
    sess.state()
    sv.spec_kv_truncate(sess.kv, B, seq, torch.full((B,), 8, dtype=torch.int32, device="cuda"), 0, None)   # back to 8 positions
    b2 = sess.forward(seq, tokens).clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b2)
    sv.spec_graph_destroy(graph)
    sess.close()


@pytest.mark.parametrize("model", ["tiny_fp32", "small_bf16"])
def test_replay_over_a_pool_with_too_few_free_pages_leaves_the_starved_sequences_alone(model):
    """The host checks the page budget when a step is launched; a recorded step replayed after other sequences took the
    free pages meets the shortage on the device.  The entries that needed a page are then left out of the step like
    entries with a bad id (rows not computed, nothing written, commit reports -1 and changes nothing), the others step as
    usual and still equal the eager step, and spec_kv_get_state reports SPEC_ENOMEM once."""
    import synth_inputs as si
    from paper_2604_26779_amd import binding as sv
    from paper_2604_26779_amd.session import VerifySession
    cfg = si.MODELS[model]
    B, k = 3, 3
    sess = VerifySession(cfg, si.make_weights(cfg, seed=2, device="cuda"), max_seqs=4, max_ctx_len=64, n_pages=6)
    sess.pool.normal_()
    ctx = [14, 3, 15]                                   # entries 0 and 2 need a second page for 4 more positions, entry 1 does not
    for b in range(B):
        sess.assign(b, ctx[b], [b])
    seq = torch.arange(B, dtype=torch.int32, device="cuda")
    tokens = torch.randint(0, cfg["vocab"], (B, k + 1), dtype=torch.int32, device="cuda")
    acc = torch.full((B,), k, dtype=torch.int32, device="cuda")
    snap = torch.empty(sv.spec_kv_state_bytes(sess.kv), dtype=torch.uint8, device="cuda")
    sv.spec_kv_snapshot(sess.kv, snap)
    ref = sess.forward(seq, tokens).clone()             # eager, with pages to spare
    torch.cuda.synchronize()
    sv.spec_kv_restore(sess.kv, snap)
    sess.state()                                        # exact bounds on the host: the recording below must not need the device
    side = torch.cuda.Stream()
    buf = sess.step_buffers(B, k)
    with torch.cuda.stream(side):
        sv.spec_graph_capture_begin(side)
        sess.forward(seq, tokens, stream=side)
        sess.commit(seq, acc, k, stream=side)
        graph = sv.spec_graph_capture_end(side)
    free = list(sess.state()["free_stack"])
    assert len(free) == 3
    sess.assign(3, 40, free)                            # another sequence takes every free page
    buf["logits"].fill_(-5.0)
    sv.spec_graph_launch(graph, side)
    side.synchronize()
    with pytest.raises(sv.SpecError) as e:
        sess.state()
    assert e.value.status == sv.SPEC_ENOMEM
    st = sess.state()                                   # the flag is reported once
    assert list(st["ctx_len"][:4]) == [14, 3 + k + 1, 15, 40] and list(st["n_pages"][:4]) == [1, 1, 1, 3]
    assert len(st["free_stack"]) == 0
    assert buf["new_ctx_len"].cpu().tolist() == [-1, 3 + k + 1, -1]
    slots = buf["commit_slots"].cpu().numpy()
    assert np.all(slots[0] == -1) and np.all(slots[2] == -1) and np.all(slots[1] >= 0)
    got = buf["logits"]
    assert torch.equal(got[1], ref[1]) and torch.isfinite(got).all()
    # with pages back, the same recording steps every entry again
    sv.spec_kv_truncate(sess.kv, 1, torch.tensor([3], dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"), 0, None)
    sv.spec_kv_truncate(sess.kv, 1, torch.tensor([1], dtype=torch.int32, device="cuda"), torch.full((1,), 3, dtype=torch.int32, device="cuda"), 0, None)
    sess.state()
    sv.spec_graph_launch(graph, side)
    side.synchronize()
    st = sess.state()
    assert list(st["ctx_len"][:3]) == [c + k + 1 for c in ctx]
    assert torch.equal(buf["logits"], ref)
    sv.spec_graph_destroy(graph)
    sess.close()
