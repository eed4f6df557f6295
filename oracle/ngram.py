"""CPU oracle for model-free n-gram drafting: the drafts of a step are copied from the sequence's own
history, from behind the most recent earlier occurrence of its current ending.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What it follows.  The paper compares against n-gram drafting as a model-free baseline (Section 3.1 set-up;
Section 3.2, Table 2) and gives no algorithm.  The reading taken here (prompt-lookup drafting):

  * the history h[0..L-1] of a sequence is every token it holds so far, the last one being the token the
    verifier emitted last (the first input of the coming step);
  * for n = n_max down to n_min: the ending e = h[L-n..L-1] is searched in h at start positions j with
    j + n <= L - 1, so that at least one token follows the occurrence and the occurrence is not the ending
    itself (it may overlap it); the longest n with an occurrence wins, and among its occurrences the most
    recent one (largest j);
  * the drafts are the tokens behind it, h[j+n], h[j+n+1], ..., at most k and at most up to h[L-1];
    `n_drafted` says how many there are.  The remaining draft slots, which the verifier still scores, repeat
    the last drafted token; without any occurrence n_drafted = 0 and every slot holds h[L-1].
A drafted token is a point mass (the verifier's one-hot draft distribution: accept x with probability p(x)).
"""
import numpy as np


def ngram_draft_one(hist, k, n_max, n_min):
    """hist: 1-D int sequence (L >= 1).  Returns (drafts [k] int32, n_drafted, n_matched, j)."""
    h = [int(t) for t in hist]
    L = len(h)
    assert L >= 1 and k >= 0 and 1 <= n_min <= n_max
    for n in range(n_max, n_min - 1, -1):
        if n > L - 1:                                   # no room for an occurrence with a token behind it
            continue
        ending = h[L - n:]
        for j in range(L - 1 - n, -1, -1):              # most recent first
            if h[j:j + n] == ending:
                cont = h[j + n:j + n + k]
                n_drafted = len(cont)
                drafts = cont + [cont[-1]] * (k - n_drafted) if k > 0 else []
                return np.array(drafts, dtype=np.int32), n_drafted, n, j
    return np.full(k, h[L - 1], dtype=np.int32), 0, 0, -1


def ngram_draft(hist, hist_len, k, n_max, n_min):
    """hist [B, cap] int32, hist_len [B].  Returns (drafts [B, k] int32, n_drafted [B] int32)."""
    B = len(hist_len)
    drafts = np.zeros((B, k), dtype=np.int32)
    n_drafted = np.zeros(B, dtype=np.int32)
    for b in range(B):
        d, c, _, _ = ngram_draft_one(hist[b][:int(hist_len[b])], k, n_max, n_min)
        drafts[b] = d
        n_drafted[b] = c
    return drafts, n_drafted


def append_emitted(hist, hist_len, out_tokens, accept_len):
    """After a verify step: the accepted drafts and the token the verifier emitted (out_tokens[b][0..n]) join
    the history.  In place; a history that would overflow its row keeps what fits and its length saturates."""
    cap = hist.shape[1]
    for b in range(len(hist_len)):
        n = int(accept_len[b])
        for i in range(n + 1):
            if hist_len[b] < cap:
                hist[b, hist_len[b]] = out_tokens[b, i]
                hist_len[b] += 1
    return hist, hist_len
