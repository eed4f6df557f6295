"""Pins for the rejection-sampling oracle: what the cited procedure and mathematics fix.

The paper (Introduction; Section 2.1) fixes only that the procedure preserves the target's output
distribution.  These tests pin the oracle to that property and to closed forms of the standard
procedure, none of which is a retyping of the oracle's own code:
  * published Philox4x32-10 known answers;
  * exact joint distribution of (accept length, emitted tokens) by enumeration at V=4, k=3:
        P(n=j, x_1..x_j, y) = prod_i min(p_i, q_i)(x_i) * max(0, p_{j+1}(y) - q_{j+1}(y))   (j < k)
        P(n=k, x_1..x_k, y) = prod_i min(p_i, q_i)(x_i) * p_{k+1}(y)
    with prefix-dependent p and q tables;
  * losslessness: the first emitted token follows p_1 (chi-square, 10^6 trials);
  * draft == target accepts everything; a draft on a zero-probability token is never accepted;
  * E[n+1] = (1 - beta^(k+1)) / (1 - beta) for identical rows.
"""
import itertools
import os

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax as scipy_softmax

from oracle import commit as oracle_commit
from oracle import sampler


def test_philox_known_answers(golden_dir):
    rows = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            out = sampler.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in out] == w[6:10]
            rows += 1
    assert rows == 3


def test_uniform_ranges_and_fp32_exactness():
    ua = np.array([sampler.uniform_accept(7, 3, b, i) for b in range(200) for i in range(8)])
    uv = np.array([sampler.uniform_vocab(7, 3, b, 0, v) for b in range(4) for v in range(1000)])
    assert ua.min() >= 0.0 and ua.max() < 1.0
    assert uv.min() > 0.0 and uv.max() < 1.0
    assert np.all(ua.astype(np.float32).astype(np.float64) == ua)
    assert np.all(uv.astype(np.float32).astype(np.float64) == uv)
    # counter words are independent streams: different (b,row,v,step,seed) give different draws
    assert sampler.uniform_vocab(7, 3, 0, 0, 5) != sampler.uniform_vocab(7, 3, 0, 1, 5)
    assert sampler.uniform_vocab(7, 3, 0, 0, 5) != sampler.uniform_vocab(7, 4, 0, 0, 5)
    assert sampler.uniform_vocab(7, 3, 0, 0, 5) != sampler.uniform_vocab(8, 3, 0, 0, 5)
    assert sampler.uniform_accept(7, 3, 0, 1) != sampler.uniform_accept(7, 3, 1, 0)
    assert abs(ua.mean() - 0.5) < 0.03 and abs(uv.mean() - 0.5) < 0.03


def _random_tables(rng, V, k, sharp):
    """Prefix-dependent distributions: table[i][prefix tuple] -> probability vector, i = 0..k."""
    tables = []
    for i in range(k + 1):
        t = {}
        for prefix in itertools.product(range(V), repeat=i):
            t[prefix] = scipy_softmax(rng.standard_normal(V) * sharp)
        tables.append(t)
    return tables


def _run_trials(p_tab, q_tab, V, k, N, seed, rng, temperature=1.0):
    """Draw drafts from q autoregressively, build the rows the sampler takes, run the oracle."""
    draft = np.zeros((N, k), dtype=np.int32)
    logits = np.zeros((N, k + 1, V), dtype=np.float32)
    q = np.zeros((N, k, V), dtype=np.float32)
    prefixes = [()] * N
    # group trials by prefix so that table lookups stay cheap
    for i in range(k + 1):
        groups = {}
        for t, pre in enumerate(prefixes):
            groups.setdefault(pre, []).append(t)
        for pre, idx in groups.items():
            idx = np.array(idx)
            logits[idx, i, :] = (np.log(p_tab[i][pre]) * temperature).astype(np.float32)
            if i < k:
                qq = q_tab[i][pre].astype(np.float32)
                q[idx, i, :] = qq
                draft[idx, i] = rng.choice(V, size=len(idx), p=qq.astype(np.float64) / qq.astype(np.float64).sum())
        if i < k:
            prefixes = [pre + (int(draft[t, i]),) for t, pre in enumerate(prefixes)]
    n, out = sampler.reject_sample(logits, q, draft, temperature, seed, 0)
    return draft, n, out


@pytest.mark.parametrize("temperature", [1.0, 0.7])
def test_exact_joint_distribution_by_enumeration(temperature):
    V, k, N = 4, 3, 1_000_000
    rng = np.random.default_rng(11)
    p_tab = _random_tables(rng, V, k, 1.2)
    q_tab = _random_tables(rng, V, k, 1.2)
    # logits handed to the sampler are log(p) * T, so that softmax(logits / T) == p
    draft, n, out = _run_trials(p_tab, q_tab, V, k, N, seed=1234, rng=rng, temperature=temperature)

    # enumerate every outcome (n, emitted tokens) with its exact probability
    expected = {}
    for j in range(k + 1):
        for xs in itertools.product(range(V), repeat=j):
            keep = 1.0
            for i in range(j):
                keep *= min(p_tab[i][xs[:i]][xs[i]], float(np.float32(q_tab[i][xs[:i]][xs[i]])))
            for y in range(V):
                if j < k:
                    last = max(0.0, p_tab[j][xs][y] - float(np.float32(q_tab[j][xs][y])))
                else:
                    last = p_tab[k][xs][y]
                expected[(j,) + xs + (y,)] = keep * last
    assert abs(sum(expected.values()) - 1.0) < 1e-6

    # encode every trial's outcome (n, emitted tokens) as one integer, base V+1 with -1 -> V
    digits = np.where(out < 0, V, out).astype(np.int64)
    code = n.astype(np.int64)
    for i in range(k + 1):
        code = code * (V + 1) + digits[:, i]
    codes, counts = np.unique(code, return_counts=True)

    def encode(cell):
        j, toks = cell[0], list(cell[1:]) + [V] * (k + 1 - len(cell[1:]))
        c = j
        for tkn in toks:
            c = c * (V + 1) + tkn
        return c
    observed = {int(c): int(m) for c, m in zip(codes, counts)}
    by_code = {encode(c): c for c in expected}
    assert set(observed) <= {encode(c) for c, pr in expected.items() if pr > 0}
    observed = {by_code[c]: m for c, m in observed.items()}
    kept_mask = np.arange(k)[None, :] < n[:, None]
    assert np.all(out[:, :k][kept_mask] == draft[kept_mask])           # kept tokens are the drafts
    assert np.all(out[np.arange(k + 1)[None, :] > n[:, None]] == -1)

    # chi-square over cells with a usable expectation, the rest pooled
    cells = [c for c, pr in expected.items() if pr * N >= 10]
    exp = np.array([expected[c] * N for c in cells])
    obs = np.array([observed.get(c, 0) for c in cells], dtype=np.float64)
    rest_e = N - exp.sum()
    rest_o = N - obs.sum()
    if rest_e > 10:
        exp = np.append(exp, rest_e)
        obs = np.append(obs, rest_o)
    chi2 = float(((obs - exp) ** 2 / exp).sum())
    pval = stats.chi2.sf(chi2, df=len(exp) - 1)
    assert pval > 1e-4, (chi2, len(exp))

    # accept-length marginal against its own closed form  P(n >= j) = sum prod min(p_i, q_i)
    for j in range(1, k + 1):
        ge = sum(pr for c, pr in expected.items() if c[0] >= j)
        direct = 0.0
        for xs in itertools.product(range(V), repeat=j):
            t = 1.0
            for i in range(j):
                t *= min(p_tab[i][xs[:i]][xs[i]], q_tab[i][xs[:i]][xs[i]])
            direct += t
        assert abs(ge - direct) < 1e-5
        assert abs((n >= j).mean() - direct) < 5 * np.sqrt(direct * (1 - direct) / N) + 1e-6


def test_losslessness_first_token_follows_target():
    """Chi-square of the first emitted token against p_1 over 10^6 trials, V = 16."""
    V, k, N = 16, 3, 1_000_000
    rng = np.random.default_rng(5)
    base = rng.standard_normal((k + 1, V)) * 1.5
    logits = np.broadcast_to(base.astype(np.float32), (N, k + 1, V)).copy()
    qrow = scipy_softmax(base[:k] + rng.standard_normal((k, V)), axis=-1).astype(np.float32)
    q = np.broadcast_to(qrow, (N, k, V)).copy()
    draft = np.stack([rng.choice(V, size=N, p=qrow[i].astype(np.float64) / qrow[i].astype(np.float64).sum())
                      for i in range(k)], axis=1).astype(np.int32)
    n, out = sampler.reject_sample(logits, q, draft, 1.0, 99, 5)
    p1 = scipy_softmax(base[0].astype(np.float32).astype(np.float64))
    obs = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    chi2 = float(((obs - p1 * N) ** 2 / (p1 * N)).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    # second emitted token, given the first draft was kept, follows p_2 (rows do not depend on the prefix here)
    kept = n >= 1
    p2 = scipy_softmax(base[1].astype(np.float32).astype(np.float64))
    obs2 = np.bincount(out[kept, 1], minlength=V).astype(np.float64)
    chi2 = float(((obs2 - p2 * kept.sum()) ** 2 / (p2 * kept.sum())).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4
    # mean acceptance length, closed form for independent rows: 1 + b1 + b1 b2 + b1 b2 b3
    ps = scipy_softmax(base[:k].astype(np.float32).astype(np.float64), axis=-1)
    beta = np.minimum(ps, qrow.astype(np.float64)).sum(axis=-1)
    alpha = 1 + beta[0] + beta[0] * beta[1] + beta[0] * beta[1] * beta[2]
    assert abs(oracle_commit.mean_acceptance_length(n) - alpha) < 0.01


def test_identical_rows_geometric_acceptance_length():
    """E[n+1] = (1 - beta^(k+1)) / (1 - beta) when every position has the same p and q."""
    V, N = 8, 400_000
    rng = np.random.default_rng(3)
    row = rng.standard_normal(V)
    qrow = scipy_softmax(row + rng.standard_normal(V) * 0.8).astype(np.float32)
    p = scipy_softmax(row.astype(np.float32).astype(np.float64))
    beta = np.minimum(p, qrow.astype(np.float64)).sum()
    for k in (1, 3, 5):
        logits = np.broadcast_to(row.astype(np.float32), (N, k + 1, V)).copy()
        q = np.broadcast_to(qrow, (N, k, V)).copy()
        draft = rng.choice(V, size=(N, k), p=qrow.astype(np.float64) / qrow.astype(np.float64).sum()).astype(np.int32)
        n, _ = sampler.reject_sample(logits, q, draft, 1.0, 2024, k)
        want = (1 - beta ** (k + 1)) / (1 - beta)
        assert abs(oracle_commit.mean_acceptance_length(n) - want) < 0.02, (k, want)


def test_draft_equal_to_target_accepts_everything():
    V, k, N = 64, 3, 5000
    rng = np.random.default_rng(17)
    logits = (rng.standard_normal((N, k + 1, V)) * 2).astype(np.float32)
    q = scipy_softmax(logits[:, :k, :].astype(np.float64), axis=-1).astype(np.float32)
    draft = rng.integers(0, V, size=(N, k)).astype(np.int32)
    n, out = sampler.reject_sample(logits, q, draft, 1.0, 1, 1)
    assert np.all(n == k)
    assert np.all(out[:, :k] == draft)
    # the bonus token follows the last row
    assert np.all((out[:, k] >= 0) & (out[:, k] < V))


def test_draft_on_zero_probability_token_is_never_accepted():
    V, k, N = 12, 3, 300_000
    rng = np.random.default_rng(23)
    row = rng.standard_normal(V).astype(np.float32)
    row[4] = -np.inf                                        # p(4) = 0
    logits = np.broadcast_to(row, (N, k + 1, V)).copy()
    q = np.zeros((N, k, V), dtype=np.float32)
    q[:, :, 4] = 1.0                                        # one-hot draft distribution on token 4
    draft = np.full((N, k), 4, dtype=np.int32)
    n, out = sampler.reject_sample(logits, q, draft, 1.0, 77, 0)
    assert np.all(n == 0)
    assert np.all(out[:, 1:] == -1)
    # residual = max(0, p - q) = p, so the replacement token follows p exactly
    p = scipy_softmax(row.astype(np.float64))
    obs = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    assert obs[4] == 0
    keep = p > 0
    chi2 = float(((obs[keep] - p[keep] * N) ** 2 / (p[keep] * N)).sum())
    assert stats.chi2.sf(chi2, df=keep.sum() - 1) > 1e-4


def test_draft_with_zero_q_and_positive_p_is_accepted():
    """u * 0 < P holds for every u: a token the draft distribution gives no mass is kept if p > 0."""
    V, k = 8, 2
    logits = np.zeros((3, k + 1, V), dtype=np.float32)
    q = np.zeros((3, k, V), dtype=np.float32)
    q[:, :, 0] = 1.0
    draft = np.full((3, k), 5, dtype=np.int32)
    n, _ = sampler.reject_sample(logits, q, draft, 1.0, 1, 0)
    assert np.all(n == k)


def test_temperature_scales_logits():
    """softmax(logits / T): with T = 2 the first emitted token follows scipy's softmax of logits / 2."""
    V, k, N = 10, 1, 400_000
    rng = np.random.default_rng(29)
    row = (rng.standard_normal(V) * 3).astype(np.float32)
    logits = np.broadcast_to(row, (N, k + 1, V)).copy()
    qrow = np.full(V, 1.0 / V, dtype=np.float32)
    q = np.broadcast_to(qrow, (N, k, V)).copy()
    draft = rng.integers(0, V, size=(N, k)).astype(np.int32)
    _, out = sampler.reject_sample(logits, q, draft, 2.0, 31, 2)
    p = scipy_softmax(row.astype(np.float64) / 2.0)
    obs = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    chi2 = float(((obs - p * N) ** 2 / (p * N)).sum())
    assert stats.chi2.sf(chi2, df=V - 1) > 1e-4


def test_debug_outputs_and_determinism():
    logits, q, draft = __import__("synth_inputs").make_sampler_case(6, 3, 500, seed=9)
    a = sampler.reject_sample(logits, q, draft, 1.0, 42, 7, debug=True)
    b = sampler.reject_sample(logits, q, draft, 1.0, 42, 7, debug=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    n, out, pqu, keys = a
    for bb in range(6):
        for i in range(3):
            evaluated = i <= n[bb] and i < 3
            if i < n[bb]:
                assert pqu[bb, i, 2] * pqu[bb, i, 1] < pqu[bb, i, 0]
            elif i == n[bb]:
                assert not (pqu[bb, i, 2] * pqu[bb, i, 1] < pqu[bb, i, 0])
            else:
                assert np.all(np.isnan(pqu[bb, i])) or not evaluated
        assert keys[bb, 0] >= keys[bb, 1]
    c = sampler.reject_sample(logits, q, draft, 1.0, 42, 8)
    assert not np.array_equal(c[1], out)                    # another step word, another draw


def test_amdahl_bound_matches_paper_headline():
    """Section 2.2 bound; with the generation share and acceptance length of Table 1/2 (RL-Zero,
    R_gen = 100.0/151.2, alpha = 3.32) the bound must sit above the measured 1.41x step speedup."""
    bound = oracle_commit.step_speedup_bound(100.0 / 151.2, 3.32)
    assert 1.41 < bound < 1.0 / (1 - 100.0 / 151.2)
    assert abs(oracle_commit.step_speedup_bound(1.0, 2.5) - 2.5) < 1e-12
    assert abs(oracle_commit.step_speedup_bound(0.0, 2.5) - 1.0) < 1e-12
