"""CPU oracle for an 8-bit floating-point KV cache (E4M3).

TEST INFRASTRUCTURE ONLY (see the package docstring).

What it follows.  The paper's large-scale projections assume FP8 serving (Section 4, simulator set-up) and say
nothing more about it; this build's reading: the cache stores keys (after rotation) and values as 8-bit
floating-point numbers of the OCP "E4M3" kind with one fp32 scale per (layer, kv head) for keys and one for values,
    code = encode(x / scale),   value read back = decode(code) * scale,
and, as with the other storage types, the k+1 new positions are encoded before any row attends to them.

The format, written out from its definition: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
  exponent field 0      : +-(m / 8) * 2^-6            (zero and the subnormals, spacing 2^-9)
  exponent field 1..15  : +-(1 + m / 8) * 2^(e - 7)
  there are no infinities; S.1111.111 is the only NaN, so the largest finite magnitude is S.1111.110 = 448.
encode rounds to the nearest representable value, ties to the one with an even mantissa, and saturates at +-448
(the paper does not say; saturation is the choice that keeps an outlier finite).  NaN inputs are not handled.
"""
import numpy as np

MAX_FINITE = 448.0


def decode(code):
    """uint8 codes -> fp64 values (NaN for 0x7f / 0xff)."""
    code = np.asarray(code).astype(np.int64)
    sign = np.where((code >> 7) & 1, -1.0, 1.0)
    e = (code >> 3) & 15
    m = (code & 7).astype(np.float64)
    sub = (m / 8.0) * 2.0 ** -6
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    val = sign * np.where(e == 0, sub, nor)
    return np.where((e == 15) & ((code & 7) == 7), np.nan, val)


def quantise(x):
    """fp64 values -> the nearest E4M3 values (fp64), ties to even, saturating."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    # the binade of |x| fixes the spacing of representable values around it: 2^(e-3) with 3 mantissa bits,
    # never finer than the subnormal spacing 2^-9
    _, ex = np.frexp(a)                                     # a = f * 2^ex, f in [0.5, 1)  ->  floor(log2 a) = ex - 1
    e = np.maximum(ex - 1, -6)
    step = np.exp2((e - 3).astype(np.float64))
    q = np.rint(a / step) * step                            # rint: halves go to the even multiple
    q = np.minimum(q, MAX_FINITE)
    return np.copysign(q, x)


def encode(x):
    """fp64 values -> uint8 codes of quantise(x) (the sign of zero is kept)."""
    x = np.asarray(x, dtype=np.float64)
    q = np.abs(quantise(x))
    _, ex = np.frexp(q)
    e = ex - 1
    normal = q >= 2.0 ** -6
    e_field = np.where(normal, e + 7, 0).astype(np.int64)
    m_field = np.where(normal, np.rint((q / np.exp2(np.where(normal, e, 0).astype(np.float64)) - 1.0) * 8.0),
                       np.rint(q * 2.0 ** 9)).astype(np.int64)
    sign = np.signbit(x).astype(np.int64)
    return ((sign << 7) | (e_field << 3) | m_field).astype(np.uint8)


def store(x, scale):
    """What a cache with this scale returns for x: decode(encode(x / scale)) * scale, in fp64."""
    scale = np.asarray(scale, dtype=np.float64)
    return quantise(np.asarray(x, dtype=np.float64) / scale) * scale


def cache_values(kv_codes, scales):
    """kv_codes[layer][b] = (K codes, V codes), uint8 [ctx, Hkv, dh]; scales = (k_scale [L, Hkv], v_scale [L, Hkv]).
    Returns the same nesting with what the cache returns, decode(code) * scale, in fp64."""
    ks, vs = (np.asarray(a, dtype=np.float64) for a in scales)
    return [[(decode(K) * ks[l][None, :, None], decode(V) * vs[l][None, :, None]) for (K, V) in per_seq]
            for l, per_seq in enumerate(kv_codes)]
