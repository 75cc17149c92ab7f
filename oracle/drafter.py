"""Brute-force definition of the suffix-match drafter (Sec. 4.1.2 of the paper).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else).  Shares no code with the product.

No index: rollouts are kept as lists, a match is found by comparing slices, continuations are counted by scanning.
  * window: the last `max_epochs` epochs of rollouts;
  * match: per epoch, the longest suffix of the context (at most max_match tokens) that occurs inside one rollout; the epoch
    with the longest match wins, the newest among equals;
  * draft: repeatedly the token that follows the matched string most often in that epoch (smallest token among equals),
    the matched string growing by that token; stops when nothing follows.
"""


class BruteDrafter:
    def __init__(self, max_epochs):
        self.max_epochs = max_epochs
        self.epochs = [[]]

    def new_epoch(self):
        self.epochs.append([])
        self.epochs = self.epochs[-self.max_epochs:]

    def add(self, tokens):
        self.epochs[-1].append(list(tokens))

    @staticmethod
    def _occurrences(rollouts, s):
        """(rollout index, end position) of every occurrence of the list s."""
        n = len(s)
        return [(r, p + n) for r, seq in enumerate(rollouts) for p in range(len(seq) - n + 1) if seq[p:p + n] == s]

    def _match_len(self, rollouts, ctx, max_match):
        for length in range(min(len(ctx), max_match), 0, -1):
            if self._occurrences(rollouts, list(ctx[len(ctx) - length:])):
                return length
        return 0

    def propose(self, ctx, max_match, min_match, k):
        ctx = list(ctx)
        best_len, best = 0, None
        for rollouts in reversed(self.epochs):
            length = self._match_len(rollouts, ctx, max_match)
            if length > best_len:
                best_len, best = length, rollouts
        draft = []
        if best is None or best_len < min_match:
            return best_len, draft
        s = ctx[len(ctx) - best_len:]
        while len(draft) < k:
            follow = {}
            for r, end in self._occurrences(best, s):
                if end < len(best[r]):
                    follow[best[r][end]] = follow.get(best[r][end], 0) + 1
            if not follow:
                break
            t = min(follow, key=lambda x: (-follow[x], x))
            draft.append(t)
            s = s + [t]
        return best_len, draft
