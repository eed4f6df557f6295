"""Pins of the n-gram drafting oracle: hand-worked cases, a library routine (str.rfind on the history written as
a string finds the most recent occurrence of a substring), and invariants that a wrong bound, a wrong preference
(earliest instead of most recent, shorter instead of longer) or an off-by-one in the continuation would break."""
import numpy as np
import pytest

from oracle import ngram


def test_hand_worked_cases():
    # history a b c a b c a b : ending (n=3) "c a b" occurs at j=2 (followed by c a b ...); most recent with room
    h = [1, 2, 3, 1, 2, 3, 1, 2]
    d, c, n, j = ngram.ngram_draft_one(h, 4, 3, 1)
    assert (n, j) == (3, 2) and c == 3 and list(d) == [3, 1, 2, 2]      # 3 tokens follow j+n=5, the 4th slot repeats
    # the occurrence may overlap the ending: a a a a, n=2: ending "a a" at j=1 (j+n = 3 <= L-1 = 3)
    d, c, n, j = ngram.ngram_draft_one([7, 7, 7, 7], 2, 2, 1)
    assert (n, j, c) == (2, 1, 1) and list(d) == [7, 7]
    # longer match preferred over a more recent shorter one: ... x y z ... y z ... z | ending x? no: build explicitly
    h = [5, 6, 7, 9, 0, 6, 7, 8, 0, 5, 6, 7]
    # ending n=3 "5 6 7" occurs at j=0 (followed by 9); n=2 "6 7" occurs more recently at j=5 (followed by 8)
    d, c, n, j = ngram.ngram_draft_one(h, 2, 3, 1)
    assert (n, j) == (3, 0) and list(d) == [9, 0]
    d, c, n, j = ngram.ngram_draft_one(h, 2, 2, 1)
    assert (n, j) == (2, 5) and list(d) == [8, 0]
    # no occurrence at all, history of one token, n_min larger than what fits
    d, c, n, j = ngram.ngram_draft_one([1, 2, 3, 4], 3, 3, 1)
    assert c == 0 and j == -1 and list(d) == [4, 4, 4]
    d, c, n, j = ngram.ngram_draft_one([9], 2, 3, 1)
    assert c == 0 and list(d) == [9, 9]
    d, c, n, j = ngram.ngram_draft_one([4, 4], 2, 3, 2)
    assert c == 0 and list(d) == [4, 4]
    # k = 0: nothing to draft
    d, c, n, j = ngram.ngram_draft_one([1, 2, 1], 0, 2, 1)
    assert d.shape == (0,) and c == 0 and (n, j) == (1, 0)


@pytest.mark.parametrize("seed", range(6))
def test_against_rfind(seed):
    rng = np.random.default_rng(seed)
    for _ in range(300):
        L = int(rng.integers(1, 60))
        vocab = int(rng.integers(2, 6))
        h = rng.integers(0, vocab, size=L)
        k = int(rng.integers(1, 6))
        n_max = int(rng.integers(1, 6))
        n_min = int(rng.integers(1, n_max + 1))
        d, c, n, j = ngram.ngram_draft_one(h, k, n_max, n_min)
        text = "".join(chr(ord("a") + int(t)) for t in h)
        want = None
        for nn in range(n_max, n_min - 1, -1):
            if nn > L - 1:
                continue
            at = text.rfind(text[L - nn:], 0, L - 1)        # occurrence must end at or before index L-2
            if at >= 0:
                want = (nn, at)
                break
        if want is None:
            assert c == 0 and j == -1 and np.all(d == h[-1])
        else:
            assert (n, j) == want
            cont = list(h[j + n:j + n + k])
            assert c == len(cont) and 1 <= c <= k
            assert list(d[:c]) == [int(t) for t in cont] and np.all(d[c:] == cont[-1])


def test_batch_and_append():
    hist = np.zeros((2, 8), dtype=np.int32)
    hist[0, :5] = [1, 2, 3, 1, 2]
    hist[1, :3] = [4, 5, 6]
    hist_len = np.array([5, 3], dtype=np.int32)
    drafts, c = ngram.ngram_draft(hist, hist_len, 2, 2, 1)
    assert list(drafts[0]) == [3, 1] and c[0] == 2           # ending "1 2" at j=0 -> 3 1
    assert list(drafts[1]) == [6, 6] and c[1] == 0
    out = np.array([[3, 1, 9], [7, 0, 0]], dtype=np.int32)
    ngram.append_emitted(hist, hist_len, out, np.array([2, 0]))
    assert list(hist_len) == [8, 4] and list(hist[0]) == [1, 2, 3, 1, 2, 3, 1, 9] and list(hist[1, :4]) == [4, 5, 6, 7]
    ngram.append_emitted(hist, hist_len, out, np.array([1, 0]))       # row 0 is full: nothing more fits
    assert list(hist_len) == [8, 5] and list(hist[0]) == [1, 2, 3, 1, 2, 3, 1, 9]
