"""Pins of the brute-force drafter (oracle/drafter.py, Sec. 4.1.2) against hand-worked examples and a library routine
(Python's own substring search on byte strings for the longest match)."""
import numpy as np

from oracle.drafter import BruteDrafter


def test_hand_worked_examples():
    d = BruteDrafter(max_epochs=2)
    a, b, c, dd, x = 1, 2, 3, 4, 9
    d.add([a, b, c, a, b, dd])
    # context ends in "a b": matches twice, followed once by c and once by d -> the smaller token, then what follows "a b c"
    assert d.propose([x, a, b], 8, 1, 3) == (2, [c, a, b])
    # "x" never occurs: no match, no draft; a one-token match is refused when two are asked for
    assert d.propose([a, x], 8, 1, 3) == (0, [])
    assert d.propose([x, b], 8, 2, 3) == (1, [])
    # the end of a rollout is never proposed, and a match never runs over two rollouts
    d.add([dd, a])
    assert d.propose([b, dd], 8, 1, 4) == (2, [])            # "b d" ends the first rollout; "d a" starts another one
    assert d.propose([dd, dd], 8, 1, 4) == (1, [a])          # "d d" does not occur across the boundary; "d" is followed by a
    # frequency decides: after "a", b follows twice and nothing else
    assert d.propose([a], 8, 1, 1) == (1, [b])
    # max_match caps how much of the context is looked at
    assert d.propose([c, a, b], 2, 1, 1)[0] == 2 and d.propose([c, a, b], 8, 1, 1)[0] == 3


def test_window_keeps_the_most_recent_epochs_and_prefers_the_newest_on_ties():
    d = BruteDrafter(max_epochs=2)
    d.add([1, 2, 3])
    d.new_epoch()
    d.add([1, 2, 4])
    assert d.propose([1, 2], 8, 1, 1) == (2, [4])            # both epochs match two tokens: the newest one drafts
    assert d.propose([0, 2, 3], 8, 1, 1) == (2, [])          # only the old epoch has "2 3" (and nothing follows it there)
    d.new_epoch()                                            # the first epoch leaves the window
    d.add([7, 7])
    assert d.propose([2, 3], 8, 1, 1) == (0, [])
    assert d.propose([1, 2], 8, 1, 1) == (2, [4])


def test_longest_match_equals_pythons_substring_search():
    rng = np.random.default_rng(3)
    for _ in range(200):
        d = BruteDrafter(max_epochs=1)
        rollouts = [rng.integers(0, 4, size=rng.integers(1, 30)).tolist() for _ in range(rng.integers(1, 4))]
        for r in rollouts:
            d.add(r)
        ctx = rng.integers(0, 4, size=rng.integers(0, 12)).tolist()
        want = 0
        for length in range(len(ctx), 0, -1):
            if any(bytes(ctx[len(ctx) - length:]) in bytes(r) for r in rollouts):
                want = length
                break
        assert d.propose(ctx, 64, 1, 0)[0] == want
