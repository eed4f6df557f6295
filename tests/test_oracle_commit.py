"""Pins for the KV bookkeeping oracle: exhaustive small cases against a set-based model.

The paper does not describe the cache (Section 2.1-2.2 only imply one); the reading under test is:
positions ctx..ctx+k are written speculatively, ctx..ctx+n stay, the new length is ctx+n+1, pages
wholly beyond the new length are released.  The independent model below works on sets of
logical positions instead of page counters.
"""
import numpy as np

from oracle.commit import KVBook, mean_acceptance_length

P = 16


def test_exhaustive_lengths_slots_and_released_pages():
    for k in (1, 3, 5, 7):
        for ctx in list(range(0, 2 * P + 2)) + [5 * P - 1, 5 * P]:
            for n in range(k + 1):
                book = KVBook(n_pages=40, page_size=P)
                pages = list(range(20, 20 + -(-ctx // P)))
                book.assign(0, ctx, pages)
                free_before = set(book.free)
                book.reserve([0], k)
                held = list(book.pages[0])
                # set-based model: pages needed to hold positions 0..ctx+k
                positions = set(range(ctx + k + 1))
                assert len(held) == len({p // P for p in positions})
                assert held[:len(pages)] == pages
                new_len, slots = book.commit([0], [n], k)
                assert new_len == [ctx + n + 1]
                kept_positions = set(range(ctx + n + 1))
                kept_pages = {p // P for p in kept_positions}
                assert len(book.pages[0]) == len(kept_pages)
                for i in range(k + 1):
                    if i <= n:
                        pos = ctx + i
                        assert slots[0][i] == held[pos // P] * P + pos % P
                    else:
                        assert slots[0][i] == -1
                # pages are conserved: free + held partitions the pool
                assert set(book.free) | set(book.pages[0]) == set(range(40))
                assert len(book.free) + len(book.pages[0]) == 40
                assert set(book.free) >= free_before - set(held)


def test_reserve_pops_in_batch_order_and_release_pushes_back():
    book = KVBook(n_pages=10, page_size=P)
    book.assign("a", 16, [7])
    book.assign("b", 15, [2])
    # free stack pops ascending over the remaining pages: 0, 1, 3, ...
    book.reserve(["a", "b"], 3)
    assert book.pages["a"] == [7, 0]            # 16+4 = 20 positions -> 2 pages
    assert book.pages["b"] == [2, 1]            # 15+4 = 19 positions -> 2 pages
    new_len, slots = book.commit(["a", "b"], [0, 3], 3)
    assert new_len == [17, 19]
    assert book.pages["a"] == [7, 0] and book.pages["b"] == [2, 1]
    assert slots[0] == [0 * P + 0, -1, -1, -1]
    assert slots[1] == [2 * P + 15, 1 * P + 0, 1 * P + 1, 1 * P + 2]
    # a sequence whose tail page becomes unused gives it back; the next reserve reuses it first
    book2 = KVBook(n_pages=4, page_size=P)
    book2.assign(0, 14, [3])
    book2.reserve([0], 3)                       # 18 positions -> second page = 0
    assert book2.pages[0] == [3, 0]
    book2.commit([0], [0], 3)                   # new length 15 -> one page
    assert book2.pages[0] == [3] and book2.free[-1] == 0


def test_acceptance_length_counts_every_produced_token():
    assert mean_acceptance_length([0, 3, 1]) == (1 + 4 + 2) / 3
    assert mean_acceptance_length(np.array([3, 3])) == 4.0     # k = 3 fully accepted: k + 1 tokens
