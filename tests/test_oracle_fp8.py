"""Pins for the 8-bit (E4M3) cache oracle.

The format itself is fixed by its definition (1-4-3 bits, bias 7, no infinities, one NaN, maximum 448), so the pins are:
  * decoding all 256 codes against PyTorch's float8_e4m3fn (a library's independent implementation);
  * encoding against PyTorch's conversion on in-range values, and against brute force over the decode table
    (nearest value, ties to the even mantissa) on values from every binade, the subnormal range and beyond 448;
  * exact midpoints, saturation, sign of zero, round trip of every finite code;
  * in the forward pass: one pass over k+1 positions == k+1 single decodes fed with what the cache returns; a power
    of two in the scale changes nothing; scale -> 0 error bound of half a mantissa step.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import forward as of
from oracle import fp8

ALL = np.arange(256, dtype=np.uint8)
FINITE = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)


def test_decode_table_matches_library():
    lib = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = fp8.decode(ALL)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok])
    assert np.array_equal(np.signbit(lib[ok]), np.signbit(mine[ok]))
    # the definition's landmarks
    assert fp8.decode(0x7E) == 448.0 and fp8.decode(0x01) == 2.0 ** -9 and fp8.decode(0x08) == 2.0 ** -6
    assert fp8.decode(0x38) == 1.0 and fp8.decode(0xB8) == -1.0


def test_every_finite_code_round_trips():
    assert np.array_equal(fp8.encode(fp8.decode(FINITE)), FINITE)


def _brute_force(x):
    """Nearest finite value of the table; of two equally near ones the one whose code is even."""
    vals = fp8.decode(FINITE)
    out = np.empty(len(x))
    for i, xi in enumerate(x):
        d = np.abs(vals - xi)
        best = np.flatnonzero(d == d.min())
        if len(best) > 1:                               # a tie (or +-0): take the even mantissa, keep the sign of x
            best = [j for j in best if FINITE[j] % 2 == 0 and (vals[j] != 0 or np.signbit(vals[j]) == np.signbit(xi))]
        out[i] = vals[best[0]]
    return out


def test_quantise_is_nearest_ties_to_even_brute_force():
    rng = np.random.default_rng(5)
    xs = [rng.normal(size=400) * s for s in (2.0 ** -10, 2.0 ** -7, 0.01, 1.0, 30.0, 300.0, 2000.0)]
    vals = np.sort(np.unique(np.abs(fp8.decode(FINITE))))
    mids = (vals[:-1] + vals[1:]) / 2                    # every exact midpoint, both signs
    xs += [mids, -mids, mids * (1 + 1e-12), mids * (1 - 1e-12), vals, -vals]
    x = np.concatenate(xs)
    assert np.array_equal(fp8.quantise(x), _brute_force(x))
    assert np.array_equal(fp8.decode(fp8.encode(x)), fp8.quantise(x))


def test_encode_matches_library_in_range():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.normal(size=5000) * s for s in (0.003, 0.1, 1.0, 20.0, 120.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.encode(x.astype(np.float64)), lib)


def test_saturation_midpoints_and_zero():
    assert fp8.quantise(1.0e4) == 448.0 and fp8.quantise(-1.0e4) == -448.0
    assert fp8.quantise(464.0) == 448.0 and fp8.quantise(447.9) == 448.0
    assert fp8.quantise(1.0625) == 1.0 and fp8.quantise(1.1875) == 1.25      # ties: to the even mantissa
    assert fp8.quantise(2.0 ** -10) == 0.0 and fp8.quantise(3 * 2.0 ** -10) == 2.0 ** -8
    assert fp8.encode(-0.0) == 0x80 and fp8.encode(0.0) == 0x00
    assert fp8.encode(1.9375 + 0.04) == fp8.encode(2.0) == 0x40               # rounding up into the next binade


def test_relative_error_bound():
    rng = np.random.default_rng(7)
    x = rng.normal(size=20000) * 10.0
    x = x[(np.abs(x) >= 2.0 ** -6) & (np.abs(x) <= 448)]
    assert np.max(np.abs(fp8.quantise(x) - x) / np.abs(x)) <= 2.0 ** -4     # half a step of a 3-bit mantissa


# ------------------------------------------------------------------------------------------ in the forward pass
CFG = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=96, vocab=50,
           rope_theta=1.0e4, rms_eps=1.0e-5, dtype="f64", tied_head=0, kv_dtype="fp8_e4m3")


def _setup(seed=3):
    w = si.weights_for_oracle(CFG, si.make_weights(CFG, seed=seed, std=0.2))
    rng = np.random.default_rng(seed)
    scales = (0.02 * (1 + rng.random((2, 2))), 0.03 * (1 + rng.random((2, 2))))
    ctx_len = np.array([5, 0, 9])
    kv = []
    for l in range(2):
        per_seq = []
        for b, c in enumerate(ctx_len):
            K = fp8.store(rng.normal(size=(c, 2, 16)), scales[0][l][None, :, None])
            V = fp8.store(rng.normal(size=(c, 2, 16)), scales[1][l][None, :, None])
            per_seq.append((K, V))
        kv.append(per_seq)
    tokens = rng.integers(0, 50, size=(3, 4))
    return w, scales, ctx_len, kv, tokens


def test_new_positions_are_stored_before_they_are_attended():
    """k+1 positions in one pass == k+1 single decodes, each fed with what the cache returned for the earlier ones."""
    w, scales, ctx_len, kv, tokens = _setup()
    logits, new_kv = of.verify_forward(CFG, w, kv, tokens, ctx_len, kv_scales=scales)
    cur = [[(K.copy(), V.copy()) for K, V in layer] for layer in kv]
    for i in range(tokens.shape[1]):
        li, nk = of.verify_forward(CFG, w, cur, tokens[:, i:i + 1], ctx_len + i, kv_scales=scales)
        assert np.allclose(li[:, 0], logits[:, i], rtol=0, atol=1e-9)
        for l in range(2):
            for b in range(3):
                assert np.array_equal(nk[l][0][b, 0], new_kv[l][0][b, i])
                cur[l][b] = (np.concatenate([cur[l][b][0], nk[l][0][b]]), np.concatenate([cur[l][b][1], nk[l][1][b]]))
    # what is stored is on the scaled grid
    for l in range(2):
        for which in (0, 1):
            v = new_kv[l][which] / scales[which][l][None, None, :, None]
            assert np.allclose(fp8.quantise(v), v, rtol=1e-12, atol=0)


def test_stored_values_differ_from_unrounded_and_power_of_two_scale_is_neutral():
    w, scales, ctx_len, kv, tokens = _setup()
    logits, new_kv = of.verify_forward(CFG, w, kv, tokens, ctx_len, kv_scales=scales)
    plain, plain_kv = of.verify_forward(dict(CFG, kv_dtype=None), w, kv, tokens, ctx_len)
    assert np.max(np.abs(logits - plain)) > 1e-4                         # the rounding is really applied
    rel = np.abs(new_kv[0][0] - plain_kv[0][0]) / np.maximum(np.abs(plain_kv[0][0]), 1e-300)
    big = np.abs(plain_kv[0][0]) >= scales[0][0][None, None, :, None] * 2.0 ** -6
    assert np.max(rel[big]) <= 2.0 ** -4
    # a factor 4 in every scale moves the grid with the data (no saturation, no subnormals at these magnitudes
    # except for values that are subnormal already: compare where the stored value is a normal number)
    s4 = (scales[0] * 4, scales[1] * 4)
    _, kv4 = of.verify_forward(CFG, w, [[(K, V) for K, V in layer] for layer in kv], tokens, ctx_len, kv_scales=s4)
    normal = np.abs(new_kv[0][0]) >= s4[0][0][None, None, :, None] * 2.0 ** -6
    assert np.array_equal(kv4[0][0][normal], new_kv[0][0][normal])


def test_8bit_matrices_reach_the_oracle_as_codes_and_scales():
    """The generator's 8-bit matrices (a library cast of w / scale, scale = row absmax / 448) reach the oracle as bytes
    plus scales; the oracle's own decode * scale is checked against the library's cast back and against the draws the
    codes came from (half a mantissa step; the row maximum itself is exact), and the forward pass with them against
    the forward pass on the dequantised matrices given as plain fp64 arrays."""
    cfg = dict(si.MODELS["small_bf16_w8"])
    w8 = si.make_weights(cfg, seed=4)
    w16 = si.make_weights(dict(cfg, w_dtype=None), seed=4)
    names = [n for n in w16]
    assert list(w8)[:len(names)] == names and all(n.endswith(".scale") for n in list(w8)[len(names):])
    w_or = si.weights_for_oracle(cfg, w8)
    for name, key in (("l0.wq", "wq"), ("l1.wd", "wd"), ("l0.wg", "wg")):
        layer = int(name[1])
        mine = of.matrix(w_or["layers"][layer], key)
        lib = w8[name].to(torch.float64).numpy() * w8[name + ".scale"].to(torch.float64).numpy()[:, None]
        assert np.array_equal(mine, lib)
        orig = w16[name].to(torch.float64).numpy()
        scale = w8[name + ".scale"].numpy().astype(np.float64)
        big = np.abs(orig) >= scale[:, None] * 2.0 ** -6
        assert np.max(np.abs(mine - orig)[big] / np.abs(orig)[big]) <= 2.0 ** -4 * (1 + 1e-6)
        assert np.allclose(np.abs(mine).max(axis=1), np.abs(orig).max(axis=1), rtol=1e-6)
    # the forward pass: codes + scales in, against the same matrices dequantised beforehand
    plain = {"embed": w_or["embed"], "final_norm": w_or["final_norm"], "head": of.matrix(w_or, "head"),
             "layers": [{k: (of.matrix(lw, k) if k.startswith("w") else lw[k]) for k in lw if not k.endswith("_scale")}
                        for lw in w_or["layers"]]}
    ctx_len = np.array([3, 0])
    kv = si.kv_for_oracle(si.make_logical_kv(dict(cfg, kv_dtype=None), ctx_len, seed=5))
    tokens = np.array([[1, 2, 3], [4, 5, 6]])
    a, _ = of.verify_forward(cfg, w_or, kv, tokens, ctx_len)
    b, _ = of.verify_forward(dict(cfg, w_dtype=None), plain, kv, tokens, ctx_len)
    assert np.array_equal(a, b)
    # ... and given as the library's cast times the scale (what the full-size tests hand over): fp32 products
    c, _ = of.verify_forward(dict(cfg, w_dtype=None), si.weights_for_oracle(cfg, w8, library_decode=True), kv, tokens, ctx_len)
    assert np.allclose(a, c, rtol=0, atol=1e-5)


def test_weight_count_with_8bit_matrices():
    from paper_2604_26779_amd import binding as sv
    import ctypes
    for name in ("small_bf16", "small_bf16_w8", "small_bf16_w8kv8"):
        cfg = si.MODELS[name]
        d = sv.make_desc(cfg)
        assert sv.lib().spec_model_weight_count(ctypes.byref(d)) == len(si.make_weights(cfg, seed=1))
