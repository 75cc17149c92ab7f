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


def test_greedy_accept_rule_brute_force():
    """All draft strings over a 3-letter alphabet, k <= 3, against the literal
    definition: emit what step-by-step decoding emits."""
    for k in range(4):
        for g in itertools.product(range(3), repeat=k + 1):
            for d in itertools.product(range(3), repeat=k):
                a, nxt = greedy_accept(g, d)
                # literal: walk while the draft agrees with the target's choice
                j = 0
                while j < k and d[j] == g[j]:
                    j += 1
                assert (a, nxt) == (j, g[j])
                assert 0 <= a <= k


def test_argmax_ties_take_lowest_index():
    g = np.argmax(np.array([[0.0, 2.0, 2.0, 1.0]]), axis=1)
    assert g[0] == 1


# ----------------------------------------------------------------------------- rejection sampling

def test_inverse_cdf_definition():
    w = np.array([0.0, 1.0, 0.0, 3.0, 0.0])
    assert inverse_cdf(w, 0.0) == 1
    assert inverse_cdf(w, 0.2499) == 1
    assert inverse_cdf(w, 0.25) == 3          # cumulative must EXCEED u*Z
    assert inverse_cdf(w, 0.999999) == 3
    assert inverse_cdf(np.array([1.0, 1.0, 0.0]), 1.0) == 1     # clamp to last non-zero weight


def test_rejection_identity_is_exact():
    """p(d)[x=d] + (1-p(d)) r(x) = p(x) for the point-mass drafter."""
    rng = np.random.default_rng(0)
    for _ in range(20):
        V = int(rng.integers(3, 12))
        p = rng.dirichlet(np.ones(V))
        d = int(rng.integers(0, V))
        r = p.copy(); r[d] = 0.0; r /= r.sum()
        mix = (1 - p[d]) * r
        mix[d] += p[d]
        np.testing.assert_allclose(mix, p, atol=1e-12)


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
    w, Z = softmax_weights(logits[0], tau)
    p = w / Z
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
    p0 = softmax_weights(logits[0], tau)[0]; p0 = p0 / p0.sum()
    p1 = softmax_weights(logits[1], tau)[0]; p1 = p1 / p1.sum()
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
        w, _ = softmax_weights(logits[0], 0.8)
        assert a == 0 and nxt == inverse_cdf(w, u)


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
