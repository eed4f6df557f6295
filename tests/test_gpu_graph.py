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
