"""Pins of the oracle's speculative round: losslessness (abstract, Sec. 5.1,
Sec. 6 of the paper), its boundary cases, the rejection-sampling rule the
paper cites, the page bookkeeping invariants and the drafter statistics."""
import itertools
import numpy as np
import pytest

import das_inputs as di
import oracle
from oracle import greedy_accept, stochastic_accept, softmax_weights, inverse_cdf


def _start(om, shape, seed, n=24, cap=400):
    s = om.new_seq(cap)
    prompt = di.prompts([n], shape.vocab, seed)[0]
    s.pending = int(np.argmax(om.prefill(s, prompt)))
    return s, prompt


def _ar_reference(om, shape, seed, n_tokens, n=24):
    s, _ = _start(om, shape, seed, n)
    first = s.pending
    return [first] + om.ar_greedy(s, n_tokens - 1)


@pytest.mark.parametrize("drafter", ["random", "all_right", "all_wrong", "p0.7", "mixed_k"])
def test_speculative_greedy_is_token_identical_to_plain_decoding(tiny_oracle, tiny_shape, drafter):
    """32 rounds of config 1: whatever the drafts, the emitted stream equals
    one-token-at-a-time greedy decoding."""
    om, V = tiny_oracle, tiny_shape.vocab
    ref = _ar_reference(om, tiny_shape, seed=21, n_tokens=32 * 9 + 10)
    s, _ = _start(om, tiny_shape, seed=21)
    rng = np.random.default_rng(77)
    emitted = [s.pending]
    accepted_total = 0
    for rnd in range(32):
        k = 4 if drafter != "mixed_k" else int(rng.integers(0, 9))
        future = ref[len(emitted):len(emitted) + k]
        if drafter == "random":
            d = rng.integers(0, V, size=k, dtype=np.int32)
        elif drafter == "all_right":
            d = np.array(future, np.int32)
        elif drafter == "all_wrong":
            d = (np.array(future, np.int32) + 1) % V
        else:
            d = di.make_drafts(future, k, 0.7, V, rng)
        a, nxt, _ = om.verify_greedy(s, d)
        if drafter == "all_right":
            assert a == k
        if drafter == "all_wrong":
            assert a == 0
        om.commit(s, a, nxt, d)
        emitted += [int(t) for t in d[:a]] + [nxt]
        accepted_total += a
    assert emitted == ref[:len(emitted)]
    assert s.tokens + [s.pending] == list(di.prompts([24], V, 21)[0]) + emitted
    if drafter == "p0.7":
        assert accepted_total > 32        # the drafter does get tokens accepted


def test_boundary_cases(tiny_oracle, tiny_shape):
    om = tiny_oracle
    ref = _ar_reference(om, tiny_shape, seed=5, n_tokens=12)
    # k = 0 is a plain decode step
    s, _ = _start(om, tiny_shape, seed=5)
    a, nxt, lg = om.verify_greedy(s, [])
    assert (a, nxt) == (0, ref[1]) and lg.shape[0] == 1
    # all-correct draft: a = k and next is the AR token after the draft
    a, nxt, _ = om.verify_greedy(s, ref[1:6])
    assert (a, nxt) == (5, ref[6])
    # first token wrong: a = 0, next = AR next, whatever follows
    bad = [(ref[1] + 1) % tiny_shape.vocab] + ref[2:6]
    a, nxt, _ = om.verify_greedy(s, bad)
    assert (a, nxt) == (0, ref[1])
    # third wrong
    bad = ref[1:3] + [(ref[3] + 5) % tiny_shape.vocab] + ref[4:6]
    a, nxt, _ = om.verify_greedy(s, bad)
    assert (a, nxt) == (2, ref[3])


def _emitted_by_plain_decoding(next_token, n):
    """n tokens of one-token-at-a-time greedy decoding from a next-token table (a deterministic 'model'
    whose choice depends on the last token only)."""
    out, x = [], 0
    for _ in range(n):
        x = next_token[x]
        out.append(x)
    return out


def test_greedy_accept_emits_the_plain_decoding_stream_for_every_draft_string():
    """Losslessness on a toy target (the next token is a function of the last token, alphabet of 3): for EVERY
    draft string of length <= 3, what a round emits -- the accepted drafts, then the target's own token -- is a prefix
    of the stream plain decoding produces, it is as long as the longest draft prefix that agrees with that stream
    plus one, and rounds chained with arbitrary drafts reproduce the stream.  The expected values come from the
    plain stream, not from the acceptance rule."""
    for table in itertools.product(range(3), repeat=3):
        stream = _emitted_by_plain_decoding(table, 12)
        for k in range(4):
            for d in itertools.product(range(3), repeat=k):
                # rows [pending = 0, d_1..d_k]: the target's token after row j follows the row's own input token
                g = [table[t] for t in (0,) + d]
                a, nxt = greedy_accept(g, d)
                agree = 0
                while agree < k and d[agree] == stream[agree]:
                    agree += 1
                assert a == agree
                assert list(d[:a]) + [nxt] == stream[:a + 1]
        # chained rounds with a fixed awkward draft pattern
        rng = np.random.default_rng(sum(table))
        emitted, last = [], 0
        while len(emitted) < 9:
            d = tuple(int(x) for x in rng.integers(0, 3, size=int(rng.integers(0, 4))))
            g = [table[t] for t in (last,) + d]
            a, nxt = greedy_accept(g, d)
            emitted += list(d[:a]) + [nxt]
            last = nxt
        assert emitted == stream[:len(emitted)]


def test_verify_greedy_breaks_logit_ties_towards_the_lowest_index(tiny_oracle, tiny_shape):
    """The oracle's own decision path on planted ties: rows of logits with the maximum at two and at three
    columns must yield the lowest of them as the target's token (hand-written rows, through oracle.verify_greedy's
    argmax + greedy_accept, with the model forward replaced by the planted logits)."""
    rows = np.array([[0.0, 2.0, 2.0, 1.0, -1.0],
                     [3.0, 0.5, 3.0, 3.0, 0.0],
                     [-4.0, -4.0, -4.0, -4.0, -4.0]], dtype=np.float32)

    class Planted(type(tiny_oracle)):
        def __init__(self):      # no weights: only the decision logic of the parent class is exercised
            pass

        def verify_logits(self, seq, drafts):
            return rows[: len(drafts) + 1]

        def close(self):
            pass

    om = Planted()
    assert om.verify_greedy(None, [])[:2] == (0, 1)               # tie between columns 1 and 2 -> 1
    assert om.verify_greedy(None, [1])[:2] == (1, 0)              # draft 1 accepted; next row ties at 0, 2, 3 -> 0
    assert om.verify_greedy(None, [2])[:2] == (0, 1)              # the HIGHER tied column is not the target's token
    assert om.verify_greedy(None, [1, 0])[:2] == (2, 0)           # all-equal row -> column 0


# ----------------------------------------------------------------------------- rejection sampling

def test_inverse_cdf_definition():
    w = np.array([0.0, 1.0, 0.0, 3.0, 0.0])
    assert inverse_cdf(w, 0.0) == 1
    assert inverse_cdf(w, 0.2499) == 1
    assert inverse_cdf(w, 0.25) == 3          # cumulative must EXCEED u*Z
    assert inverse_cdf(w, 0.999999) == 3
    assert inverse_cdf(np.array([1.0, 1.0, 0.0]), 1.0) == 1     # clamp to last non-zero weight


def test_softmax_weights_hand_values():
    """Pins of the target weights w_v = exp(l_v/tau - max) from outside the oracle: logits tau*[0, ln 2, ln 4] give
    p = (1/7, 2/7, 4/7) at every temperature; the same logits at another temperature give p ~ 2^(v/tau'); a large
    common offset changes nothing (the maximum is subtracted before exp); the largest weight is exactly 1."""
    for tau in (1.0, 0.6, 2.5):
        l = tau * np.log(np.array([1.0, 2.0, 4.0]))
        w, Z = softmax_weights(l, tau)
        np.testing.assert_allclose(w / Z, [1 / 7, 2 / 7, 4 / 7], rtol=1e-12)
        assert w.max() == 1.0 and abs(Z - 1.75) < 1e-12
        w2, Z2 = softmax_weights(l + 1000.0, tau)                  # exp(1000) overflows unless the max is subtracted
        np.testing.assert_allclose(w2 / Z2, [1 / 7, 2 / 7, 4 / 7], rtol=1e-9)
    # the same logits [0, ln 2, ln 4] read at tau = 0.5: p ~ (1, 4, 16); at tau = 2: p ~ (1, sqrt 2, 2)
    l = np.log(np.array([1.0, 2.0, 4.0]))
    w, Z = softmax_weights(l, 0.5)
    np.testing.assert_allclose(w / Z, np.array([1.0, 4.0, 16.0]) / 21.0, rtol=1e-12)
    w, Z = softmax_weights(l, 2.0)
    np.testing.assert_allclose(w / Z, np.array([1.0, np.sqrt(2.0), 2.0]) / (3.0 + np.sqrt(2.0)), rtol=1e-12)
    # lowering the temperature sharpens: the top token's probability grows
    l = np.array([0.3, -1.2, 2.0, 0.0])
    tops = [softmax_weights(l, t)[0][2] / softmax_weights(l, t)[1] for t in (2.0, 1.0, 0.6, 0.2)]
    assert tops == sorted(tops) and tops[-1] > 0.99


def test_stochastic_accept_probability_is_the_target_probability():
    """Draft d is accepted iff u < p_target(d) with p = softmax(l / tau) written out here: the acceptance threshold
    of the oracle's rule, found by bisection on u, equals exp(l_d/tau) / sum exp(l/tau) for every token."""
    rng = np.random.default_rng(3)
    for tau in (1.0, 0.6):
        l = rng.standard_normal(9) * 2.0
        p = np.exp(l / tau) / np.exp(l / tau).sum()
        logits = np.stack([l, l])
        for d in range(9):
            lo, hi = 0.0, 1.0
            for _ in range(50):
                mid = 0.5 * (lo + hi)
                if stochastic_accept(logits, [d], tau, [mid, 0.0], [0.5, 0.5])[0] == 1:
                    lo = mid
                else:
                    hi = mid
            assert abs(lo - p[d]) < 1e-9, (tau, d, lo, p[d])


def test_residual_distribution_by_enumeration():
    """After a rejection the emitted token follows max(0, p - delta_d) renormalised = p with d removed: the measure of
    u_sample that yields each token, found on a fine grid, against the closed form written out here; and the
    mixture p(d)[x=d] + (1-p(d)) r(x) is p(x) again (the rule is lossless)."""
    rng = np.random.default_rng(0)
    M = 4000
    grid = (np.arange(M) + 0.5) / M
    for tau in (1.0, 0.6):
        V = 7
        l = rng.standard_normal(V) * 1.5
        p = np.exp(l / tau) / np.exp(l / tau).sum()
        d = 3
        logits = np.stack([l, l])
        hist = np.zeros(V)
        for u in grid:
            a, nxt = stochastic_accept(logits, [d], tau, [0.999999, 0.0], [u, 0.5])      # u_accept ~ 1: rejected
            assert a == 0
            hist[nxt] += 1
        r = p.copy(); r[d] = 0.0; r /= r.sum()
        np.testing.assert_allclose(hist / M, r, atol=1.5 / M)
        mix = (1 - p[d]) * (hist / M)
        mix[d] += p[d]
        np.testing.assert_allclose(mix, p, atol=2.0 / M)


def _first_token_hist(logits, drafts, tau, n, seed):
    rng = np.random.default_rng(seed)
    V = logits.shape[1]
    hist = np.zeros(V)
    k = len(drafts)
    for _ in range(n):
        ua, us = rng.random(k + 1), rng.random(k + 1)
        a, nxt = stochastic_accept(logits, drafts, tau, ua, us)
        first = drafts[0] if a >= 1 else nxt
        hist[first] += 1
    return hist


@pytest.mark.parametrize("tau", [1.0, 0.6])
def test_first_emitted_token_follows_target_distribution_chi_square(tau):
    from scipy.stats import chi2
    rng = np.random.default_rng(4)
    V, k, n = 24, 3, 120000
    logits = rng.standard_normal((k + 1, V)) * 1.5
    drafts = [int(np.argmax(logits[0])), 5, 7]          # a likely first draft: both branches are exercised
    hist = _first_token_hist(logits, drafts, tau, n, seed=99)
    p = np.exp(logits[0] / tau) / np.exp(logits[0] / tau).sum()      # the target distribution, written out
    stat = float(((hist - n * p) ** 2 / (n * p)).sum())
    assert chi2.sf(stat, V - 1) > 1e-3, stat
    # a planted mistake (no renormalised residual: resample from p itself) must fail the same test
    bad = hist.copy()
    pd = p[drafts[0]]
    wrong = pd * np.eye(V)[drafts[0]] + (1 - pd) * p
    stat_wrong = float(((n * wrong - n * p) ** 2 / (n * p)).sum())
    assert chi2.sf(stat_wrong, V - 1) < 1e-6


def test_two_token_joint_by_enumeration():
    """Joint of the first two emitted tokens by enumerating the uniforms on a
    midpoint grid (the outcome is piecewise constant in them): token 1 ~ p_0;
    given the first draft was accepted, token 2 ~ p_1; a rejected round emits
    one token and never the rejected draft."""
    rng = np.random.default_rng(8)
    V, tau, M = 6, 1.0, 250
    logits = rng.standard_normal((3, V))
    d = [2, 4]
    p0 = np.exp(logits[0] / tau) / np.exp(logits[0] / tau).sum()
    p1 = np.exp(logits[1] / tau) / np.exp(logits[1] / tau).sum()
    grid = (np.arange(M) + 0.5) / M
    first = np.zeros(V)
    second = np.zeros(V)
    for ua in grid:
        for us in grid:
            a, nxt = stochastic_accept(logits, d, tau, [ua, 0.99, 0.5], [us, 0.5, 0.5])
            if a == 0:
                assert nxt != d[0]
                first[nxt] += 1
            else:
                first[d[0]] += 1
            a, nxt = stochastic_accept(logits, d, tau, [0.0, ua, 0.5], [0.5, us, 0.5])   # first draft accepted
            assert a >= 1
            second[d[1] if a == 2 else nxt] += 1
            if a == 1:
                assert nxt != d[1]
    np.testing.assert_allclose(first / first.sum(), p0, atol=2.0 / M)
    np.testing.assert_allclose(second / second.sum(), p1, atol=2.0 / M)


def test_k0_is_plain_inverse_cdf_sampling():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((1, 40))
    for u in [0.0, 0.1, 0.5, 0.93, 0.999999]:
        a, nxt = stochastic_accept(logits, [], 0.8, [0.3], [u])
        cdf = np.cumsum(np.exp(logits[0].astype(np.float64) / 0.8))
        assert a == 0 and nxt == int(np.searchsorted(cdf, u * cdf[-1], side="right"))


def test_accept_uses_strict_less_than_and_forced_accept():
    logits = np.zeros((2, 4))           # p = 1/4 each
    assert stochastic_accept(logits, [1], 1.0, [0.0, 0.0], [0.0, 0.0])[0] == 1      # u = 0 always accepts
    assert stochastic_accept(logits, [1], 1.0, [0.25, 0.0], [0.0, 0.0])[0] == 0     # u = p rejects
    # residual never returns the rejected token
    for u in np.linspace(0, 0.999, 50):
        a, nxt = stochastic_accept(logits, [1], 1.0, [0.9, 0.0], [u, 0.0])
        assert a == 0 and nxt != 1


# ----------------------------------------------------------------------------- page bookkeeping

def test_page_mirror_invariants():
    rng = np.random.default_rng(6)
    total = 200
    pt = oracle.PageTableMirror(total, 16)
    ids = list(range(5))
    lens = [int(x) for x in rng.integers(1, 70, size=5)]
    pt.prefill(ids, lens)
    assert pt.pages[0][0] == 0                      # first page handed out is page 0

    def check():
        owned = [p for sid in pt.pages for p in pt.pages[sid]]
        assert len(owned) == len(set(owned))
        assert len(owned) + len(pt.free) == total
        assert not set(owned) & set(pt.free)
    check()
    for sid in ids:
        assert len(pt.pages[sid]) == -(-pt.len[sid] // 16)
    for _ in range(60):
        ks = [int(x) for x in rng.integers(0, 33, size=5)]
        pt.verify(ids, ks)
        check()
        for sid, k in zip(ids, ks):
            assert len(pt.pages[sid]) == -(-(pt.len[sid] + 1 + k) // 16)
        if rng.random() < 0.3:
            before = {sid: pt.len[sid] for sid in ids}
            snapshot = {sid: list(pt.pages[sid][:-(-pt.len[sid] // 16)]) for sid in ids}
            pt.rollback(ids)
            assert before == pt.len
            assert snapshot == pt.pages
        else:
            acc = [int(rng.integers(0, k + 1)) for k in ks]
            old = dict(pt.len)
            pt.commit(ids, acc)
            for sid, a in zip(ids, acc):
                assert pt.len[sid] == old[sid] + 1 + a
        for sid in ids:
            assert len(pt.pages[sid]) == -(-pt.len[sid] // 16)
        check()
    pt.release(ids)
    assert sorted(pt.free) == list(range(total))


def test_rollback_then_reverify_and_commit_equals_fresh_prefill(tiny_oracle, tiny_shape):
    om = tiny_oracle
    s, prompt = _start(om, tiny_shape, seed=31)
    d = np.array([1, 2, 3, 4], np.int32)
    a1, n1, l1 = om.verify_greedy(s, d)
    # rollback = nothing committed; an identical verify gives identical outputs
    a2, n2, l2 = om.verify_greedy(s, d)
    assert (a1, n1) == (a2, n2)
    np.testing.assert_array_equal(l1, l2)
    ref = _ar_reference(om, tiny_shape, seed=31, n_tokens=8)
    a, nxt, _ = om.verify_greedy(s, ref[1:4])
    om.commit(s, a, nxt, ref[1:4])
    # state after commit == a fresh sequence prefilled with the same tokens
    fresh = om.new_seq(400)
    lg = om.prefill(fresh, np.array(s.tokens, np.int32))
    assert int(np.argmax(lg)) == s.pending
    after = om.forward(s, s.len, [s.pending])[0]
    after_fresh = om.forward(fresh, fresh.len, [s.pending])[0]
    np.testing.assert_allclose(after, after_fresh, atol=1e-5)


def test_mean_accept_length_matches_closed_form():
    """Synthetic drafter statistics: E[a] = p'(1-p'^k)/(1-p')."""
    rng = np.random.default_rng(12)
    V, k, p, n = 50, 6, 0.7, 40000
    future = np.arange(100, 100 + k) % V
    tot = 0
    for _ in range(n):
        d = di.make_drafts(future, k, p, V, rng)
        a, _ = greedy_accept(list(future) + [0], d)
        tot += a
    mean = tot / n
    want = di.expected_accept_len(p, k, V)
    # per-trial variance of a is below k^2/4
    assert abs(mean - want) < 3 * (k / 2) / np.sqrt(n)
