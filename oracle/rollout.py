"""CPU oracle for the slot bookkeeping of a continuous rollout: sequences that have produced their whole response
leave their batch slot, waiting sequences take the slot over, slots without a successor idle.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What it follows.  The paper's rollouts generate responses of very different lengths (long-tailed; Section 2.2 and
the discussion of generation time in Section 4), so a fixed set of batch slots drains unevenly: the decode phase
keeps running while fewer and fewer slots hold a live sequence.  The paper describes no mechanism; the reading
taken here is the usual continuous-batching one, on the decode phase only:

  * a slot b holds sequence slot_seq[b]; gen_len[s] counts the response tokens of s, target_len[s] is where its
    response ends (a synthetic stand-in for the end-of-sequence token);
  * after a speculation step with accept length n the sequence has produced n+1 more tokens, of which only those
    up to target_len count (the rest lie behind the end of the response and are dropped);
  * a sequence that reached its target is retired: its whole cache is released (keep_len 0).  The next waiting
    sequence of `queue` (already prefilled: it holds its prompt's cache) takes the slot, and its first input token
    replaces the slot's next-step input.  Slots are served in batch order.  With the queue exhausted the slot goes
    idle: it keeps the retired sequence id, produces nothing, and whatever later steps write for it is released
    again after every step (keep_len 0);
  * keep_len for a live, unfinished sequence is KEEP_ALL (nothing to release).
"""
import numpy as np

KEEP_ALL = 2 ** 30


def retire_and_backfill(slot_seq, active, accept_len, k, gen_len, target_len, queue, head, first_token, tokens):
    """Arrays are updated in place (slot_seq, active [B]; gen_len [n_seqs]; tokens [B, k+1]).

    Returns (release_seq [B], keep_len [B], head, produced): what to hand to the cache roll-back
    (``KVBook.truncate(release_seq, keep_len)``), the new queue head, and the tokens counted this step.
    """
    B = len(slot_seq)
    release_seq = np.zeros(B, dtype=np.int32)
    keep_len = np.zeros(B, dtype=np.int32)
    produced = 0
    for b in range(B):
        s = int(slot_seq[b])
        release_seq[b] = s
        if not active[b]:
            keep_len[b] = 0
            continue
        n = min(max(int(accept_len[b]), 0), k)
        made = min(n + 1, int(target_len[s]) - int(gen_len[s]))
        made = max(made, 0)
        gen_len[s] += made
        produced += made
        if gen_len[s] >= target_len[s]:
            keep_len[b] = 0
            if head < len(queue):
                nxt = int(queue[head])
                head += 1
                slot_seq[b] = nxt
                tokens[b, 0] = first_token[nxt]
            else:
                active[b] = 0
        else:
            keep_len[b] = KEEP_ALL
    return release_seq, keep_len, head, produced


def compact_slots(slot_seq, active, tokens):
    """Live slots move to the front, in their order; idle ones follow, in theirs (a stable partition), so that a
    step over the first `n_live` slots covers every live sequence.  Returns (slot_seq, active, tokens, n_live) as
    new arrays."""
    slot_seq, active, tokens = np.asarray(slot_seq), np.asarray(active), np.asarray(tokens)
    live = [b for b in range(len(active)) if active[b]]
    idle = [b for b in range(len(active)) if not active[b]]
    order = live + idle
    return slot_seq[order].copy(), active[order].copy(), tokens[order].copy(), len(live)


def backfill_pending(pending, slot_seq_before, slot_seq, active, prev_token, first_token):
    """With a draft model the step also carries, per slot, the pair of tokens the draft has not cached yet: the last
    input the target has cached and the last emitted token (``oracle/draft.py``).  A slot that a waiting sequence has
    just taken over starts from that sequence's own pair: the last token of its prompt (cached by the target, not by
    the draft, whose cache is one position behind) and its first input token.  pending [B, 2] is updated in place;
    slots that kept their sequence, and idle ones, are left alone.  Returns the slots that changed."""
    changed = []
    for b in range(len(slot_seq)):
        s = int(slot_seq[b])
        if active[b] and s != int(slot_seq_before[b]):
            pending[b, 0] = prev_token[s]
            pending[b, 1] = first_token[s]
            changed.append(b)
    return changed


def backfill_pending_hidden(pending_hidden, slot_seq_before, slot_seq, active, seq_hidden):
    """A draft model that takes the verifier's hidden states (the paper's Section 2.3 drafting paths) also carries, per
    slot, the hidden states of the positions before its two pending tokens (``oracle/draft.py: next_pending_hidden``).
    A waiting sequence brings its own: seq_hidden[s] [2, d], left by whatever prefilled it - the verifier's hidden state
    of the position before the last prompt token and of the last prompt token's own position.  A slot that sequence s
    has just taken over gets them; every other slot is left alone.  pending_hidden [B, 2, d] is updated in place.
    Returns the slots that changed (the same ones ``backfill_pending`` changes)."""
    changed = []
    for b in range(len(slot_seq)):
        s = int(slot_seq[b])
        if active[b] and s != int(slot_seq_before[b]):
            pending_hidden[b, 0, :] = seq_hidden[s, 0, :]
            pending_hidden[b, 1, :] = seq_hidden[s, 1, :]
            changed.append(b)
    return changed
