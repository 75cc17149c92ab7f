"""Integer mirror of the paged-KV bookkeeping -- TEST INFRASTRUCTURE ONLY.

Pages hold `page_size` tokens.  A sequence of length n owns ceil(n/page_size)
pages.  The free list is a stack initialised so that the first pop returns
page 0; a verify step allocates, in batch order and ascending position, the
pages that positions len..len+k need; commit keeps ceil((len+1+a)/page_size)
pages and rollback ceil(len/page_size), returning the others to the stack from
the highest page position down, sequences in batch order.  ("Accepted tokens
advance generation", Fig. 3 right: everything else is discarded.)
"""


class PageTableMirror:
    def __init__(self, num_pages, page_size=16):
        self.page_size = page_size
        self.free = list(range(num_pages - 1, -1, -1))   # pop() -> 0 first
        self.pages = {}      # seq_id -> list of page ids
        self.len = {}        # seq_id -> committed length
        self.spec = {}       # seq_id -> rows written speculatively

    def _need(self, n):
        return (n + self.page_size - 1) // self.page_size

    def _grow(self, sid, n_tokens):
        pl = self.pages.setdefault(sid, [])
        while len(pl) < self._need(n_tokens):
            pl.append(self.free.pop())

    def _shrink(self, sid, n_tokens):
        pl = self.pages[sid]
        while len(pl) > self._need(n_tokens):
            self.free.append(pl.pop())

    def prefill(self, seq_ids, lens):
        for sid, n in zip(seq_ids, lens):
            self.len[sid] = 0
            self._grow(sid, n)
            self.len[sid] = int(n)

    def verify(self, seq_ids, draft_lens):
        for sid, k in zip(seq_ids, draft_lens):
            self._grow(sid, self.len[sid] + 1 + int(k))
            self.spec[sid] = 1 + int(k)

    def commit(self, seq_ids, accept_lens):
        for sid, a in zip(seq_ids, accept_lens):
            self.len[sid] += 1 + int(a)
            self._shrink(sid, self.len[sid])
            self.spec.pop(sid, None)

    def rollback(self, seq_ids):
        for sid in seq_ids:
            self._shrink(sid, self.len[sid])
            self.spec.pop(sid, None)

    def release(self, seq_ids):
        for sid in seq_ids:
            self._shrink(sid, 0)
            del self.pages[sid], self.len[sid]
