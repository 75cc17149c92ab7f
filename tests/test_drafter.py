"""The suffix-tree drafter behind include/das_drafter.h against the brute-force definition (oracle/drafter.py): same match
lengths and same drafts on random corpora, degenerate repeats, several epochs with the window sliding.  Host code: no GPU."""
import time

import numpy as np
import pytest

from oracle.drafter import BruteDrafter
from paper_2511_13841_amd.drafter import Drafter, DrafterError


def _compare(dr, br, ctx, max_match, min_match, k):
    ml, draft = dr.propose(ctx, k, max_match=max_match, min_match=min_match)
    want_ml, want = br.propose(ctx, max_match, min_match, k)
    assert ml == want_ml, (ctx, ml, want_ml)
    assert draft.tolist() == want, (ctx, draft.tolist(), want)


@pytest.mark.parametrize("alphabet,seed", [(2, 0), (3, 1), (5, 2), (50, 3)])
def test_random_corpora_match_the_brute_force(alphabet, seed):
    rng = np.random.default_rng(seed)
    for _ in range(40):
        dr, br = Drafter(max_epochs=1), BruteDrafter(1)
        for _ in range(rng.integers(1, 5)):
            r = rng.integers(0, alphabet, size=rng.integers(1, 60))
            dr.add(r)
            br.add(r.tolist())
        for _ in range(30):
            ctx = rng.integers(0, alphabet, size=rng.integers(0, 20))
            _compare(dr, br, ctx, int(rng.integers(1, 24)), int(rng.integers(0, 3)), int(rng.integers(0, 9)))
        dr.free()


def test_contexts_cut_out_of_the_corpus_and_degenerate_repeats():
    rng = np.random.default_rng(9)
    dr, br = Drafter(max_epochs=1), BruteDrafter(1)
    rolls = [[7] * 40, [7, 8] * 15, rng.integers(0, 3, size=80).tolist(), [1, 2, 3, 4, 5, 1, 2, 3, 4, 6, 1, 2, 3, 9]]
    for r in rolls:
        dr.add(r)
        br.add(r)
    for r in rolls:
        for a in range(0, len(r), 3):
            for b in range(a + 1, min(len(r), a + 12)):
                _compare(dr, br, [99] + r[a:b], 16, 1, 6)          # a context that ends inside the corpus
    _compare(dr, br, [7] * 60, 64, 1, 10)                           # longer than any run of 7s
    _compare(dr, br, [], 8, 0, 4)
    dr.free()


def test_epochs_slide_out_of_the_window():
    rng = np.random.default_rng(4)
    dr, br = Drafter(max_epochs=3), BruteDrafter(3)
    for epoch in range(7):
        if epoch:
            dr.new_epoch()
            br.new_epoch()
        for _ in range(3):
            r = rng.integers(0, 4, size=rng.integers(5, 40))
            dr.add(r)
            br.add(r.tolist())
        for _ in range(40):
            _compare(dr, br, rng.integers(0, 4, size=rng.integers(1, 15)), 12, 1, 5)
        assert dr.size()["epochs"] == min(epoch + 1, 3)
    dr.free()


def test_linear_time_construction_and_bad_arguments():
    rng = np.random.default_rng(1)
    dr = Drafter(max_epochs=2)
    t0 = time.time()
    for _ in range(40):
        dr.add(rng.integers(0, 50000, size=5000))                   # 200k tokens, large alphabet
    dr.add(np.tile(np.arange(7), 3000))                             # 21k tokens of a short period: deep repeats
    build = time.time() - t0
    sz = dr.size()
    assert sz["tokens"] == 200000 + 40 + 21000 + 1 and sz["nodes"] < 2 * sz["tokens"]
    t0 = time.time()
    for _ in range(2000):
        dr.propose(rng.integers(0, 50000, size=64), 8, max_match=32)
    ml, draft = dr.propose(np.tile(np.arange(7), 6), 8, max_match=32)
    assert ml == 32 and draft.tolist() == [0, 1, 2, 3, 4, 5, 6, 0]
    assert build < 20 and time.time() - t0 < 5
    with pytest.raises(DrafterError):
        dr.add([1, -2, 3])
    with pytest.raises(DrafterError):
        dr.add([])
    dr.free()
