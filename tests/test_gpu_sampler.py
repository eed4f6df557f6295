"""GPU parity of spec_reject_sample against the C oracle on the same seeded inputs.

Accept lengths and emitted tokens must be bit-exact, with no exemption: the kernels take every decision
in fp64 like the oracle.  Trials the oracle flags as close calls (an accept test with |u - P/Q| < 1e-3, a race
whose two best keys differ by less than 1e-4 relative) are counted and printed, and must agree too.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import sampler as oracle_sampler
from tests.helpers import assert_sampler_parity

pytestmark = pytest.mark.gpu


def _run_gpu(logits, q, draft, temperature, seed, step):
    from paper_2604_26779_amd import binding as sv
    B, T, V = logits.shape
    k = T - 1
    dev = "cuda"
    d_logits = torch.from_numpy(logits).to(dev)
    d_q = torch.from_numpy(q).to(dev) if k > 0 else None
    d_draft = torch.from_numpy(draft).to(dev) if k > 0 else None
    n = torch.full((B,), -7, dtype=torch.int32, device=dev)
    out = torch.full((B, T), -7, dtype=torch.int32, device=dev)
    dbg = torch.zeros((B, max(k, 1), 3), dtype=torch.float32, device=dev)
    ws = torch.empty(sv.spec_sample_workspace_bytes(B, k), dtype=torch.uint8, device=dev)
    sv.spec_reject_sample(B, k, V, d_logits, d_q, d_draft, temperature, seed, step, n, out, dbg, ws)
    torch.cuda.synchronize()
    return n.cpu().numpy(), out.cpu().numpy(), dbg.cpu().numpy()


@pytest.mark.parametrize("B,k,V,temperature,noise", [
    (7, 3, 1000, 1.0, 1.0),          # several wavefronts, ragged tail (V % 4 == 0 but V % 1024 != 0)
    (5, 7, 4001, 0.7, 0.5),          # V % 4 != 0, k = 7, temperature != 1
    (3, 0, 50, 1.0, 1.0),            # k = 0: plain sampling from the target
    (64, 1, 257, 1.3, 2.0),
    (32, 3, 128256, 1.0, 1.0),       # the full-size vocabulary and batch of the 8B workload
    (256, 5, 32000, 1.0, 0.3),
    (256, 7, 128256, 1.0, 1.0),      # the large rollout batch at its deepest draft
    (128, 3, 151936, 1.0, 1.0),      # the mixture-of-experts slice's vocabulary and batch
])
def test_parity_on_synthetic_logits(B, k, V, temperature, noise):
    logits, q, draft = si.make_sampler_case(B, k, V, seed=B * 1000 + k, noise_std=noise, temperature=temperature)
    seed, step = 0x1234ABCD5678EF01, 11
    n_or, out_or, pqu, keys = oracle_sampler.reject_sample(logits, q, draft, temperature, seed, step, debug=True)
    n_gpu, out_gpu, dbg = _run_gpu(logits, q, draft, temperature, seed, step)
    stats = assert_sampler_parity(n_gpu, out_gpu, n_or, out_or, pqu, keys, exact=True)
    print("sampler parity", dict(B=B, k=k, V=V), stats, "mean accepted+1 = %.3f" % (n_or.mean() + 1))
    # the debug triples agree with the oracle's where both evaluated the test
    for b in range(B):
        for i in range(min(k, n_or[b] + 1)):
            if n_gpu[b] == n_or[b]:
                assert dbg[b, i, 2] == np.float32(pqu[b, i, 2])                 # identical uniform
                assert abs(dbg[b, i, 0] - pqu[b, i, 0]) <= 1.2e-7 * pqu[b, i, 0] + 1e-40      # the fp64 value rounded to the fp32 debug slot
                assert dbg[b, i, 1] == np.float32(pqu[b, i, 1])


def test_draft_equal_target_and_zero_probability_draft():
    B, k, V = 40, 3, 3000
    rng = np.random.default_rng(5)
    logits = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
    z = logits[:, :k].astype(np.float64)
    z -= z.max(-1, keepdims=True)
    q = np.exp(z)
    q = (q / q.sum(-1, keepdims=True)).astype(np.float32)
    draft = rng.integers(0, V, size=(B, k)).astype(np.int32)
    n_gpu, out_gpu, _ = _run_gpu(logits, q, draft, 1.0, 99, 0)
    n_or, out_or = oracle_sampler.reject_sample(logits, q, draft, 1.0, 99, 0)
    # P/Q is 1 up to the rounding of q to fp32 and u < 1 - 2^-24: the oracle accepts everything, and so must the kernel
    assert np.all(n_or == k)
    n_or2, out_or2, pqu, keys = oracle_sampler.reject_sample(logits, q, draft, 1.0, 99, 0, debug=True)
    stats = assert_sampler_parity(n_gpu, out_gpu, n_or2, out_or2, pqu, keys, exact=True)
    print("draft == target:", stats)
    assert stats["exempt_used"] == 0 and np.all(n_gpu == k)

    # a one-hot draft distribution on a token the target gives zero probability
    logits2 = logits.copy()
    logits2[:, :, 17] = -np.inf
    q2 = np.zeros_like(q)
    q2[:, :, 17] = 1.0
    draft2 = np.full((B, k), 17, dtype=np.int32)
    n_gpu, out_gpu, _ = _run_gpu(logits2, q2, draft2, 1.0, 7, 3)
    n_or, out_or, pqu, keys = oracle_sampler.reject_sample(logits2, q2, draft2, 1.0, 7, 3, debug=True)
    assert np.all(n_gpu == 0) and np.all(n_or == 0)
    assert_sampler_parity(n_gpu, out_gpu, n_or, out_or, pqu, keys, exact=True)
    assert np.all(out_gpu[:, 0] != 17) and np.all(out_gpu[:, 1:] == -1)


def test_out_of_range_draft_is_rejected_and_results_are_deterministic():
    B, k, V = 6, 3, 500
    logits, q, draft = si.make_sampler_case(B, k, V, seed=3)
    draft[2, 1] = V + 5
    draft[4, 0] = -1
    a = _run_gpu(logits, q, draft, 1.0, 5, 5)
    b = _run_gpu(logits, q, draft, 1.0, 5, 5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert a[0][2] <= 1 and a[0][4] == 0
    c = _run_gpu(logits, q, draft, 1.0, 5, 6)
    assert not np.array_equal(a[1], c[1])


def test_argument_errors():
    from paper_2604_26779_amd import binding as sv
    t = torch.zeros(16, dtype=torch.float32, device="cuda")
    i = torch.zeros(16, dtype=torch.int32, device="cuda")
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    for args in [
        (0, 1, 4, t, t, i, 1.0, 0, 0, i, i, None, ws),            # B < 1
        (1, 16, 4, t, t, i, 1.0, 0, 0, i, i, None, ws),           # k > SPEC_MAX_DRAFT
        (1, 1, 4, t, t, i, 0.0, 0, 0, i, i, None, ws),            # temperature 0
        (1, 1, 4, t, t, None, 1.0, 0, 0, i, i, None, ws),         # drafts missing with k > 0
        (1, 1, 4, t, t, i, 1.0, 0, 1 << 30, i, i, None, ws),      # step too large
        (1, 1, 4, t, t, i, 1.0, 0, 0, i, i, None, ws[:4]),        # workspace too small
    ]:
        with pytest.raises(sv.SpecError) as e:
            sv.spec_reject_sample(*args)
        assert e.value.status == sv.SPEC_EINVAL


@pytest.mark.parametrize("B,k,V", [(48, 3, 5000), (16, 5, 128256)])
def test_one_hot_drafts_without_a_q_array(B, k, V):
    """A deterministic drafter (n-gram table): q is one-hot on the drafted token, so the library is given no q at
    all.  Must equal the oracle run on the explicit one-hot array: accept with probability p(x), residual = p
    without x."""
    from paper_2604_26779_amd import binding as sv
    rng = np.random.Generator(np.random.Philox(B + k))
    logits = (rng.standard_normal((B, k + 1, V)) * 3.0).astype(np.float32)
    # drafts: random tokens; for two thirds of them the target is made to favour that token (p(x) around 0.5 .. 0.9)
    draft = rng.integers(0, V, size=(B, k)).astype(np.int32)
    boost = np.where(rng.random((B, k)) < 0.67, np.log(V) + rng.uniform(4.0, 6.5, size=(B, k)), 0.0).astype(np.float32)
    np.put_along_axis(logits[:, :k], draft[:, :, None].astype(np.int64), boost[:, :, None], axis=2)
    q = np.zeros((B, k, V), dtype=np.float32)
    np.put_along_axis(q, draft[:, :, None].astype(np.int64), 1.0, axis=2)
    seed, step = 77, 3
    n_or, out_or, pqu, keys = oracle_sampler.reject_sample(logits, q, draft, 1.0, seed, step, debug=True)
    n = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    out = torch.full((B, k + 1), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(sv.spec_sample_workspace_bytes(B, k), dtype=torch.uint8, device="cuda")
    sv.spec_reject_sample(B, k, V, torch.from_numpy(logits).cuda(), None, torch.from_numpy(draft).cuda(), 1.0, seed, step, n, out, None, ws)
    torch.cuda.synchronize()
    stats = assert_sampler_parity(n.cpu().numpy(), out.cpu().numpy(), n_or, out_or, pqu, keys, exact=True)
    print("one-hot drafts", dict(B=B, k=k, V=V), stats, "mean accepted+1 = %.3f" % (n_or.mean() + 1))
    assert 0 < n_or.mean() < k                      # both outcomes occur
    rejected = n_or < k
    assert np.all(out_or[rejected, n_or[rejected]] != draft[rejected, n_or[rejected]])      # the rejected token is never re-drawn


def test_losslessness_on_the_gpu_first_emitted_token_follows_the_target():
    """The invariant the method rests on (Section 2.1), checked on the kernels themselves rather than through the oracle:
    with drafts drawn from q by spec_draft_sample and verified by spec_reject_sample, the first emitted token of a
    sequence - the kept draft or the token resampled from the residual - is distributed as the target's p, whatever q
    is.  V = 8, k = 3, 10^6 trials (20 steps of 50 000 sequences that share one set of logits), chi-square at 1e-4; the
    mean accept length is compared with its closed form sum_i prod_{j<=i} sum_v min(p_j(v), q_j(v))."""
    from scipy import stats
    from paper_2604_26779_amd import binding as sv
    B, k, V, T = 50_000, 3, 8, 0.9
    rng = np.random.default_rng(77)
    lp = (rng.standard_normal((k + 1, V)) * 1.5).astype(np.float32)            # target logits per row
    lq = (lp[:k] + rng.standard_normal((k, V)) * 1.0).astype(np.float32)       # draft logits: a noisy copy
    soft = lambda z: np.exp(z / np.float32(T) - (z / np.float32(T)).max(-1, keepdims=True)) / np.exp(z / np.float32(T) - (z / np.float32(T)).max(-1, keepdims=True)).sum(-1, keepdims=True)
    p, q = soft(lp.astype(np.float64)), soft(lq.astype(np.float64))
    d_logits = torch.from_numpy(np.broadcast_to(lp, (B, k + 1, V)).copy()).cuda()
    d_qlogits = torch.from_numpy(np.broadcast_to(lq, (B, k, V)).copy()).cuda()
    d_q = torch.zeros((B, k, V), dtype=torch.float32, device="cuda")
    drafts = torch.zeros((B, k), dtype=torch.int32, device="cuda")
    n = torch.zeros(B, dtype=torch.int32, device="cuda")
    out = torch.zeros((B, k + 1), dtype=torch.int32, device="cuda")
    ws = torch.empty(sv.spec_sample_workspace_bytes(B, k), dtype=torch.uint8, device="cuda")
    counts = np.zeros(V)
    acc_sum, steps = 0.0, 20
    for step in range(steps):
        for i in range(k):                                                      # x_i ~ q_i on the draft's random stream
            sv.spec_draft_sample(B, V, d_qlogits.data_ptr() + 4 * i * V, k * V, T, 4242, step, i,
                                 drafts.data_ptr() + 4 * i, k, None, 1, d_q.data_ptr() + 4 * i * V, k * V)
        sv.spec_reject_sample(B, k, V, d_logits, d_q, drafts, T, 4242, step, n, out, None, ws)
        torch.cuda.synchronize()
        counts += np.bincount(out[:, 0].cpu().numpy(), minlength=V)
        acc_sum += float(n.float().mean().item())
    expect = p[0] * B * steps
    chi2 = float(((counts - expect) ** 2 / expect).sum())
    pval = stats.chi2.sf(chi2, df=V - 1)
    beta = np.minimum(p[:k], q).sum(-1)                                         # per-position acceptance probability
    want_n = float(np.cumprod(beta).sum())
    print("GPU losslessness: chi2 %.2f (p-value %.3f) over %d trials; mean accept length %.4f, closed form %.4f" % (chi2, pval, B * steps, acc_sum / steps, want_n))
    assert pval > 1e-4
    assert abs(acc_sum / steps - want_n) < 5e-3
