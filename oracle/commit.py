"""CPU oracle for the KV bookkeeping around a verify step (page reservation and commit).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python lists, no arithmetic tricks.

What it follows.  The paper (Section 2.1-2.2) verifies drafts against the target's cache in the
decode phase and keeps what the rejection procedure accepts; it does not describe the cache.
Reading of this build: the k+1 input positions are written speculatively at logical positions
ctx .. ctx+k; after sampling, with n accepted drafts, the positions ctx .. ctx+n stay (the last
emitted token and the n kept drafts) and the new length is ctx + n + 1.  The token drawn by the
rejection procedure has no cache entry yet: it is input 0 of the next step.  Pages that lie
wholly beyond the new length go back to the free stack.

Page stack convention: the free pages form a stack; reserving pops from the top, releasing
pushes on the top; sequences are processed in batch order, a sequence's pages are released
from its last logical page downwards.  A fresh pool of n pages pops 0, 1, 2, ...
"""


class KVBook:
    def __init__(self, n_pages, page_size):
        self.page_size = int(page_size)
        self.free = list(range(int(n_pages) - 1, -1, -1))      # top of stack = end of list
        self.ctx_len = {}
        self.pages = {}

    def assign(self, seq, ctx_len, page_ids):
        """Install a sequence with an explicit (possibly fragmented) page list."""
        need = -(-int(ctx_len) // self.page_size)
        page_ids = [int(p) for p in page_ids]
        if len(page_ids) != need:
            raise ValueError("page list does not cover the context exactly")
        for p in page_ids:
            self.free.remove(p)
        self.ctx_len[seq] = int(ctx_len)
        self.pages[seq] = page_ids

    def reserve(self, seq_ids, k):
        """Before the forward pass: make room for positions ctx .. ctx+k of every sequence."""
        for seq in seq_ids:
            need = -(-(self.ctx_len[seq] + k + 1) // self.page_size)
            while len(self.pages[seq]) < need:
                self.pages[seq].append(self.free.pop())

    def slot(self, seq, pos):
        """Pool slot (page * page_size + offset) of a logical position."""
        return self.pages[seq][pos // self.page_size] * self.page_size + pos % self.page_size

    def commit(self, seq_ids, accept_len, k):
        """After sampling.  Returns (new_ctx_len [B], commit_slots [B][k+1])."""
        new_len, slots = [], []
        for b, seq in enumerate(seq_ids):
            ctx = self.ctx_len[seq]
            n = int(accept_len[b])
            if not 0 <= n <= k:
                raise ValueError("accept_len out of range")
            slots.append([self.slot(seq, ctx + i) if i <= n else -1 for i in range(k + 1)])
            new = ctx + n + 1
            keep = -(-new // self.page_size)
            while len(self.pages[seq]) > keep:
                self.free.append(self.pages[seq].pop())
            self.ctx_len[seq] = new
            new_len.append(new)
        return new_len, slots

    def truncate(self, seq_ids, new_len):
        """Roll sequences back to new_len[b] cached positions (never forwards): the draft model's cache
        after a verify step keeps only what the verifier kept.  Pages wholly beyond go back to the stack,
        in batch order, last logical page first.  Returns the lengths now in force."""
        out = []
        for b, seq in enumerate(seq_ids):
            new = int(new_len[b])
            if new < 0:
                raise ValueError("negative length")
            new = min(new, self.ctx_len[seq])
            keep = -(-new // self.page_size)
            while len(self.pages[seq]) > keep:
                self.free.append(self.pages[seq].pop())
            self.ctx_len[seq] = new
            out.append(new)
        return out


def mean_acceptance_length(accept_len):
    """Tokens produced per speculation step, the paper's acceptance length (Section 2.2): mean(n + 1)."""
    return sum(int(n) + 1 for n in accept_len) / float(len(accept_len))


def step_speedup_bound(gen_share, alpha):
    """Amdahl bound on the step-level speedup (Section 2.2): 1 / (R_gen/alpha + 1 - R_gen)."""
    return 1.0 / (gen_share / alpha + (1.0 - gen_share))
