"""Pins of the slot bookkeeping oracle: a hand-worked drain, and invariants over random rollouts that a wrong
order (slots not served in batch order), a double admission, counting behind the end of a response or a missed
release would break."""
import numpy as np

from oracle import commit as oracle_commit
from oracle import rollout as oro


def test_hand_worked_drain():
    k = 3
    slot_seq = np.array([0, 1, 2], dtype=np.int32)
    active = np.array([1, 1, 1], dtype=np.int32)
    gen = np.zeros(6, dtype=np.int32)
    target = np.array([2, 5, 9, 3, 4, 1], dtype=np.int32)
    queue = [3, 4]
    first = np.array([10, 11, 12, 13, 14, 15], dtype=np.int32)
    tokens = np.zeros((3, k + 1), dtype=np.int32)
    # step 1: accept 1, 3, 0 -> seq 0 made min(2, 2) = 2 and retires (slot 0 <- seq 3), seq 1 made 4, seq 2 made 1
    rel, keep, head, made = oro.retire_and_backfill(slot_seq, active, [1, 3, 0], k, gen, target, queue, 0, first, tokens)
    assert list(slot_seq) == [3, 1, 2] and list(active) == [1, 1, 1] and head == 1 and made == 7
    assert list(rel) == [0, 1, 2] and list(keep) == [0, oro.KEEP_ALL, oro.KEEP_ALL] and tokens[0, 0] == 13
    assert list(gen[:3]) == [2, 4, 1]
    # step 2: accept 3, 3, 3 -> seq 3 made min(4, 3) = 3 retires (slot 0 <- seq 4); seq 1 made min(4, 1) = 1 retires:
    # the queue is empty by then, slot 1 idles; seq 2 made 4
    rel, keep, head, made = oro.retire_and_backfill(slot_seq, active, [3, 3, 3], k, gen, target, queue, head, first, tokens)
    assert list(slot_seq) == [4, 1, 2] and list(active) == [1, 0, 1] and head == 2 and made == 8
    assert list(rel) == [3, 1, 2] and list(keep) == [0, 0, oro.KEEP_ALL] and tokens[0, 0] == 14
    # step 3: the idle slot is released again and counts nothing, whatever its accept length says
    rel, keep, head, made = oro.retire_and_backfill(slot_seq, active, [0, 3, 0], k, gen, target, queue, head, first, tokens)
    assert list(rel) == [4, 1, 2] and list(keep) == [oro.KEEP_ALL, 0, oro.KEEP_ALL] and made == 2 and list(active) == [1, 0, 1]


def test_random_rollouts_invariants():
    rng = np.random.default_rng(3)
    for trial in range(40):
        B, k = int(rng.integers(1, 9)), int(rng.integers(0, 6))
        n_seqs = B + int(rng.integers(0, 12))
        target = rng.integers(1, 30, size=n_seqs).astype(np.int32)
        first = rng.integers(100, 200, size=n_seqs).astype(np.int32)
        ctx0 = rng.integers(0, 50, size=n_seqs)
        book = oracle_commit.KVBook(n_pages=400, page_size=16)
        for s in range(n_seqs):
            need = -(-int(ctx0[s]) // 16)
            book.assign(s, int(ctx0[s]), list(reversed(book.free[len(book.free) - need:])))
        n_free0 = len(book.free) + sum(len(p) for p in book.pages.values())
        slot_seq = np.arange(B, dtype=np.int32)
        active = np.ones(B, dtype=np.int32)
        queue = list(range(B, n_seqs))
        gen = np.zeros(n_seqs, dtype=np.int32)
        tokens = np.zeros((B, k + 1), dtype=np.int32)
        head, total, admitted = 0, 0, []
        for step in range(200):
            if not active.any():
                break
            seqs = [int(s) for s in slot_seq]
            book.reserve(seqs, k)
            n = rng.integers(0, k + 1, size=B)
            book.commit(seqs, n, k)
            before = slot_seq.copy()
            rel, keep, head2, made = oro.retire_and_backfill(slot_seq, active, n, k, gen, target, queue, head, first, tokens)
            admitted += queue[head:head2]
            # slots served in batch order: the admitted sequences land in increasing slot index
            changed = [b for b in range(B) if slot_seq[b] != before[b]]
            assert [int(slot_seq[b]) for b in changed] == queue[head:head2]
            assert all(tokens[b, 0] == first[slot_seq[b]] for b in changed)
            head = head2
            total += made
            book.truncate([int(s) for s in rel], [int(x) for x in keep])
            for b in range(B):                               # retired and idle sequences hold nothing
                if keep[b] == 0:
                    assert book.ctx_len[int(rel[b])] == 0 and book.pages[int(rel[b])] == []
        assert not active.any() and head == len(queue) and admitted == queue
        assert np.array_equal(gen, target) and total == int(target.sum())
        assert len(book.free) + sum(len(p) for p in book.pages.values()) == n_free0       # no page lost or doubled
        assert all(book.pages[s] == [] for s in range(n_seqs))


def test_compact_slots():
    slot_seq = np.array([7, 3, 9, 1, 4], dtype=np.int32)
    active = np.array([0, 1, 0, 1, 1], dtype=np.int32)
    tokens = np.arange(10, dtype=np.int32).reshape(5, 2)
    s2, a2, t2, n = oro.compact_slots(slot_seq, active, tokens)
    assert n == 3 and list(s2) == [3, 1, 4, 7, 9] and list(a2) == [1, 1, 1, 0, 0]
    assert t2.tolist() == [[2, 3], [6, 7], [8, 9], [0, 1], [4, 5]]
    rng = np.random.default_rng(0)
    for _ in range(50):
        B = int(rng.integers(1, 40))
        seq = rng.permutation(100)[:B].astype(np.int32)
        act = (rng.random(B) < 0.5).astype(np.int32)
        tok = rng.integers(0, 1000, size=(B, 4)).astype(np.int32)
        s2, a2, t2, n = oro.compact_slots(seq, act, tok)
        assert n == act.sum() and np.all(a2[:n] == 1) and np.all(a2[n:] == 0)
        assert sorted(s2.tolist()) == sorted(seq.tolist())                    # a permutation ...
        assert list(s2[:n]) == [int(s) for s, a in zip(seq, act) if a]        # ... that keeps the live ones in order
        for b in range(B):                                                    # rows travel with their slot
            src = int(np.where(seq == s2[b])[0][0])
            assert np.array_equal(t2[b], tok[src])


def test_backfill_pending_touches_only_slots_taken_over():
    """A slot taken over by a waiting sequence starts from that sequence's own (last prompt token, first input) pair;
    slots that kept their sequence and idle slots keep what they had.  Checked on a retire step built so that all
    three kinds of slot occur, against the definition spelled out per slot."""
    rng = np.random.default_rng(3)
    B, n_seqs, k = 5, 8, 2
    slot_seq = np.arange(B, dtype=np.int32)
    active = np.array([1, 1, 1, 1, 0], dtype=np.int32)                 # slot 4 idle already
    gen = np.zeros(n_seqs, dtype=np.int32)
    target = np.array([1, 9, 2, 1, 5, 7, 7, 7], dtype=np.int32)         # slots 0, 2, 3 finish with n = 1
    queue = [5, 6]                                                      # two successors for three finishing slots
    first = rng.integers(0, 100, size=n_seqs).astype(np.int32)
    prev = rng.integers(100, 200, size=n_seqs).astype(np.int32)
    tokens = rng.integers(0, 100, size=(B, k + 1)).astype(np.int32)
    pending = rng.integers(200, 300, size=(B, 2)).astype(np.int32)
    before = slot_seq.copy()
    old_pending = pending.copy()
    oro.retire_and_backfill(slot_seq, active, np.ones(B, dtype=np.int32), k, gen, target, queue, 0, first, tokens)
    assert list(slot_seq) == [5, 1, 6, 3, 4] and list(active) == [1, 1, 1, 0, 0]
    changed = oro.backfill_pending(pending, before, slot_seq, active, prev, first)
    assert changed == [0, 2]
    for b in range(B):
        if b in (0, 2):
            assert list(pending[b]) == [prev[slot_seq[b]], first[slot_seq[b]]]
            assert pending[b, 1] == tokens[b, 0]                        # the same first input the verifier gets
        else:
            assert list(pending[b]) == list(old_pending[b])


def test_backfill_pending_hidden_follows_the_token_pairs():
    """The hidden-state pairs change for exactly the slots whose token pairs change, and to the new sequence's own two
    states; checked against the definition spelled out per slot on the same retire step as above, plus random tables."""
    rng = np.random.default_rng(4)
    B, n_seqs, d = 5, 8, 6
    before = np.arange(B, dtype=np.int32)
    after = np.array([5, 1, 6, 3, 4], dtype=np.int32)
    active = np.array([1, 1, 1, 0, 0], dtype=np.int32)
    seq_hidden = rng.standard_normal((n_seqs, 2, d)).astype(np.float32)
    ph = rng.standard_normal((B, 2, d)).astype(np.float32)
    old = ph.copy()
    pend = np.zeros((B, 2), dtype=np.int32)
    assert oro.backfill_pending_hidden(ph, before, after, active, seq_hidden) == [0, 2] == \
        oro.backfill_pending(pend, before, after, active, np.zeros(n_seqs, np.int32), np.zeros(n_seqs, np.int32))
    for b in range(B):
        want = seq_hidden[after[b]] if b in (0, 2) else old[b]
        assert np.array_equal(ph[b], want)
    for trial in range(50):                                            # idle slots and kept slots never change
        B, n_seqs = int(rng.integers(1, 40)), 60
        before = rng.permutation(n_seqs)[:B].astype(np.int32)
        after = np.where(rng.random(B) < 0.4, rng.permutation(n_seqs)[:B], before).astype(np.int32)
        active = (rng.random(B) < 0.6).astype(np.int32)
        seq_hidden = rng.standard_normal((n_seqs, 2, d)).astype(np.float32)
        ph = rng.standard_normal((B, 2, d)).astype(np.float32)
        old = ph.copy()
        changed = oro.backfill_pending_hidden(ph, before, after, active, seq_hidden)
        for b in range(B):
            moved = bool(active[b]) and after[b] != before[b]
            assert (b in changed) == moved
            assert np.array_equal(ph[b], seq_hidden[after[b]] if moved else old[b])
