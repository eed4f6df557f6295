"""ctypes access to the C rejection-sampling oracle (``reject_sample.c``).

TEST INFRASTRUCTURE ONLY (see the package docstring).  ``build()`` compiles the C file with
gcc into ``oracle/liboracle_sampler.so``; nothing here is tuned for speed.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reject_sample.c")
_LIB = os.path.join(_HERE, "liboracle_sampler.so")
_lib = None


def build(force=False):
    """Compile the C oracle.  Rebuilds when the source is newer than the library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_philox4x32_10.argtypes = [ctypes.c_void_p] * 3
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_uniform_accept.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_int]
        lib.oracle_uniform_accept.restype = ctypes.c_double
        lib.oracle_uniform_vocab.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int]
        lib.oracle_uniform_vocab.restype = ctypes.c_double
        lib.oracle_reject_sample.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_reject_sample.restype = ctypes.c_int
        lib.oracle_uniform_draft.argtypes = lib.oracle_uniform_vocab.argtypes
        lib.oracle_uniform_draft.restype = ctypes.c_double
        lib.oracle_draft_sample.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_float,
                                            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int,
                                            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_draft_sample.restype = ctypes.c_int
        _lib = lib
    return _lib


def philox4x32_10(counter, key):
    """Raw Philox4x32-10 block: 4 counter words and 2 key words in, 4 words out."""
    ctr = np.ascontiguousarray(counter, dtype=np.uint32)
    ky = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(ctr.ctypes.data, ky.ctypes.data, out.ctypes.data)
    return out


def uniform_accept(seed, step, b, row):
    return _load().oracle_uniform_accept(seed, step, b, row)


def uniform_vocab(seed, step, b, row, v):
    return _load().oracle_uniform_vocab(seed, step, b, row, v)


def reject_sample(logits, q, draft, temperature, seed, step, debug=False):
    """Rejection-sample one verify step.

    logits [B,k+1,V] fp32, q [B,k,V] fp32 probabilities, draft [B,k] int32.
    Returns (accept_len [B], out_tokens [B,k+1]) and, with ``debug``, also
    pqu [B,k,3] (P, Q, u of each evaluated accept test, NaN elsewhere) and
    keys [B,2] (winning and runner-up key of the categorical draw).
    """
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, k1, V = logits.shape
    k = k1 - 1
    q = np.ascontiguousarray(q, dtype=np.float32).reshape(B, k, V)
    draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(B, k)
    accept_len = np.zeros(B, dtype=np.int32)
    out_tokens = np.zeros((B, k + 1), dtype=np.int32)
    pqu = np.zeros((B, k, 3), dtype=np.float64)
    keys = np.zeros((B, 2), dtype=np.float64)
    rc = _load().oracle_reject_sample(B, k, V, logits.ctypes.data, q.ctypes.data, draft.ctypes.data,
                                      float(temperature), int(seed), int(step),
                                      accept_len.ctypes.data, out_tokens.ctypes.data,
                                      pqu.ctypes.data, keys.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_reject_sample: invalid arguments")
    if debug:
        return accept_len, out_tokens, pqu, keys
    return accept_len, out_tokens


def uniform_draft(seed, step, b, row, v):
    return _load().oracle_uniform_draft(seed, step, b, row, v)


def draft_sample(logits, temperature, seed, step, row, debug=False):
    """The draft model's proposal for draft position ``row``: logits [B,V] fp32 ->
    (tokens [B] int32 drawn from q, q [B,V] fp32 = softmax(logits/T)); with ``debug`` also keys [B,2]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, V = logits.shape
    tokens = np.zeros(B, dtype=np.int32)
    q = np.zeros((B, V), dtype=np.float32)
    keys = np.zeros((B, 2), dtype=np.float64)
    rc = _load().oracle_draft_sample(B, V, logits.ctypes.data, float(temperature), int(seed), int(step), int(row),
                                     tokens.ctypes.data, q.ctypes.data, keys.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_draft_sample: invalid arguments")
    if debug:
        return tokens, q, keys
    return tokens, q


def draft_sample_mapped(logits, token_map, v_full, temperature, seed, step, row, debug=False):
    """The proposal of a draft model whose output head covers a subset of the target's vocabulary (the reduced draft
    vocabulary of the EAGLE-3 design: the head holds the V_d most useful tokens, token_map [V_d] gives their ids in the
    target's vocabulary, strictly increasing).  logits [B, V_d] -> (tokens [B] as target ids, q [B, v_full] fp32): the
    draft's own softmax and draw (``draft_sample``), q laid out over the target's vocabulary with zeros outside the
    subset - the form the verifier takes."""
    token_map = np.asarray(token_map, dtype=np.int64)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    assert logits.shape[1] == token_map.shape[0] and np.all(np.diff(token_map) > 0) and 0 <= token_map[0] and token_map[-1] < v_full
    out = draft_sample(logits, temperature, seed, step, row, debug=debug)
    x_d, q_d = out[0], out[1]
    q = np.zeros((logits.shape[0], int(v_full)), dtype=np.float32)
    q[:, token_map] = q_d
    tokens = token_map[x_d].astype(np.int32)
    return (tokens, q, out[2]) if debug else (tokens, q)
