"""GPU test of spec_reject_sample_static, the entry point for callers that cannot allocate: its row statistics live
in a buffer that is part of the loaded library instead of a caller's workspace.  Everything it writes must equal
what spec_reject_sample writes on the same inputs, bit for bit (same kernels, same random streams), on two calls in
a row, the second smaller than the first (the shared buffer then still holds the first call's rows), and the
results must also agree with the C oracle under the sampler's usual rule.  Sizes beyond the built-in buffer are
refused on the host."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import sampler as oracle_sampler
from tests.helpers import assert_sampler_parity

pytestmark = pytest.mark.gpu


def _both(sv, logits, q, draft, temperature, seed, step):
    B, T, V = logits.shape
    k = T - 1
    dev = "cuda"
    d_logits = torch.from_numpy(logits).to(dev)
    d_q = torch.from_numpy(q).to(dev) if k > 0 else None
    d_draft = torch.from_numpy(draft).to(dev) if k > 0 else None
    res = []
    for static in (False, True):
        n = torch.full((B,), -7, dtype=torch.int32, device=dev)
        out = torch.full((B, T), -7, dtype=torch.int32, device=dev)
        dbg = torch.zeros((B, max(k, 1), 3), dtype=torch.float32, device=dev)
        if static:
            sv.spec_reject_sample_static(B, k, V, d_logits, d_q, d_draft, temperature, seed, step, n, out, dbg)
        else:
            ws = torch.empty(sv.spec_sample_workspace_bytes(B, k), dtype=torch.uint8, device=dev)
            sv.spec_reject_sample(B, k, V, d_logits, d_q, d_draft, temperature, seed, step, n, out, dbg, ws)
        torch.cuda.synchronize()
        res.append((n.cpu().numpy(), out.cpu().numpy(), dbg.cpu().numpy()))
    return res


def test_static_scratch_entry_point_equals_the_workspace_one():
    from paper_2604_26779_amd import binding as sv
    seed = 0x0F1E2D3C4B5A6978
    for call, (B, k, V, temperature) in enumerate([(48, 5, 32000, 0.9), (9, 2, 4001, 1.0)]):   # the second is smaller
        logits, q, draft = si.make_sampler_case(B, k, V, seed=77 + call, noise_std=1.0, temperature=temperature)
        (n_ws, out_ws, dbg_ws), (n_st, out_st, dbg_st) = _both(sv, logits, q, draft, temperature, seed, 3 + call)
        assert np.array_equal(n_st, n_ws), call
        assert np.array_equal(out_st, out_ws), call
        assert np.array_equal(dbg_st, dbg_ws, equal_nan=True), call
        n_or, out_or, pqu, keys = oracle_sampler.reject_sample(logits, q, draft, temperature, seed, 3 + call, debug=True)
        stats = assert_sampler_parity(n_st, out_st, n_or, out_or, pqu, keys, exact=True)
        print("static-scratch sampler call %d" % call, dict(B=B, k=k, V=V), stats, flush=True)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    from paper_2604_26779_amd import binding as sv
    B, k, V = 512, 7, 8                                   # 4096 rows: the limit, accepted
    logits, q, draft = si.make_sampler_case(B, k, V, seed=5, noise_std=1.0, temperature=1.0)
    (n_ws, out_ws, _), (n_st, out_st, _) = _both(sv, logits, q, draft, 1.0, 1, 0)
    assert np.array_equal(n_st, n_ws) and np.array_equal(out_st, out_ws)
    one = torch.zeros(16, dtype=torch.int32, device="cuda")
    status = sv.lib().spec_reject_sample_static(513, 7, 8, one.data_ptr(), one.data_ptr(), one.data_ptr(), 1.0, 0, 0,
                                                one.data_ptr(), one.data_ptr(), None, None)
    assert status == sv.SPEC_EINVAL and "4096" in sv.spec_last_error()
