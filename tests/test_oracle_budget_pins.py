"""Pins of the budget-model oracle (oracle/budget.py) against what the paper and the mathematics fix (Sec. 4.2.1).

The oracle contains the definitions (Eq. 3-5) and brute force only; the checks below come from outside it: limits and
slopes the paper states, a one-request optimum derived by hand from Eq. 3-5, agreement of two different brute-force
scans, and the observations the paper draws from the model."""
import math

from oracle import budget as ob


def test_accept_curve_limits_stated_by_the_paper():
    req = (1000.0, 0.8, 0.6)
    assert ob.accepted(req, 0.0) == 0.0
    assert abs(ob.accepted(req, 1e9) - 0.6 * 1000.0) < 1e-9                 # A -> k l as p -> inf (Sec. 4.2.1)
    # linear regime for p << l (appendix): A ~ alpha p when k = 1, slope k alpha in general
    for k in (1.0, 0.5):
        p = 1e-3
        assert abs(ob.accepted((1000.0, 0.8, k), p) / p - 0.8 * k) < 1e-6
    # monotone and concave in p
    a = [ob.accepted(req, p) for p in (0, 100, 200, 300)]
    assert a[1] - a[0] > a[2] - a[1] > a[3] - a[2] > 0


def test_forward_passes_and_latency_follow_eq_4_and_5_on_a_hand_example():
    # one request, numbers worked by hand: l = 100, alpha = 1, k = 1, p = 100 ln 2  ->  A = 50, 50 tokens left
    reqs = [(100.0, 1.0, 1.0), (20.0, 1.0, 1.0)]
    p = [100.0 * math.log(2.0), 0.0]
    assert abs(ob.forward_passes(reqs, p) - 50.0) < 1e-9                     # the short request (20 left) does not bind
    assert abs(ob.latency(reqs, p, 3.0, 0.01, 7.0) - (3.0 * 50.0 + 0.01 * 100.0 * math.log(2.0) + 7.0)) < 1e-9
    assert abs(ob.forward_passes(reqs, [0.0, 0.0]) - 100.0) < 1e-12          # no speculation: the longest length


def test_least_budget_is_tight_and_the_printed_closed_form_is_tight_only_for_full_capacity():
    for req in [(500.0, 0.7, 1.0), (500.0, 0.7, 0.6), (80.0, 1.5, 0.9)]:
        l, alpha, k = req
        n = l * (1 - k) + 0.4 * l * k                                        # reachable: above the floor l (1 - k)
        p = ob.least_budget(req, n)
        assert abs((l - ob.accepted(req, p)) - n) < 1e-6 * l                 # constraint of Eq. 6 holds with equality
        printed = -(l / alpha) * math.log(1.0 - k * (1.0 - n / l))           # Eq. 7 as printed
        left = l - ob.accepted(req, printed)
        if k == 1.0:
            assert abs(left - n) < 1e-6 * l
        else:
            assert left > n + 1e-3 * l                                        # too small a budget: constraint violated
    assert ob.least_budget((500.0, 0.7, 0.6), 500.0 * 0.4) == math.inf       # the floor l (1 - k) itself is never reached
    assert ob.least_budget((500.0, 0.7, 0.6), 600.0) == 0.0                   # short requests skip speculation


def test_single_request_optimum_matches_the_hand_derivation():
    # one request: J(N) = c_base N - c_tok (l/alpha) ln(1 - (1 - N/l)/k); dJ/dN = 0  =>  N* = l (1 - k + c_tok / (alpha c_base))
    for (l, alpha, k, c_base, c_tok) in [(2000.0, 0.9, 0.8, 10.0, 0.02), (300.0, 1.3, 1.0, 5.0, 0.5), (1000.0, 0.5, 0.5, 8.0, 0.1)]:
        n_star = l * (1 - k + c_tok / (alpha * c_base))
        assert l * (1 - k) < n_star < l
        n, j = ob.scan_forward_passes([(l, alpha, k)], c_base, c_tok, steps=10000)
        assert abs(n - n_star) <= 2 * l / 10000
        j_star = ob.latency_at([(l, alpha, k)], n_star, c_base, c_tok)
        assert -1e-9 <= j - j_star < 1e-6 * j_star                                # the hand-derived point is the minimum
    # speculation never pays when a proposed token costs more than the pass it saves: c_tok / (alpha k) >= c_base
    n, _ = ob.scan_forward_passes([(300.0, 1.0, 0.9)], 1.0, 2.0, steps=4000)
    assert n == 300.0


def test_scan_over_forward_passes_agrees_with_brute_force_over_the_budget_plane():
    reqs = [(400.0, 1.0, 0.9), (250.0, 0.8, 0.7)]
    c_base, c_tok = 6.0, 0.05
    n, j = ob.scan_forward_passes(reqs, c_base, c_tok, steps=8000)
    jb, p1, p2 = ob.scan_budget_plane(reqs, c_base, c_tok, p_top=1600.0, steps=400)
    assert j <= jb + 1e-9                                                     # no point of the plane beats the tight budgets
    assert jb - j < 0.01 * j                                                  # and the plane's best point is close to them
    assert abs(p1 - ob.least_budget(reqs[0], n)) < 3 * 1600.0 / 400 + 8.0
    assert abs(ob.forward_passes(reqs, (p1, p2)) - n) < 5.0


def test_observations_the_paper_draws_from_the_model():
    c_base, c_tok = 1.0, 0.02
    reqs = [(4000.0, 1.0, 0.8), (3900.0, 1.0, 0.8), (1500.0, 1.0, 0.8), (200.0, 1.0, 0.8)]
    n, _ = ob.scan_forward_passes(reqs, c_base, c_tok, steps=4000)
    p = [ob.least_budget(r, n) for r in reqs]
    assert p[0] > p[2] > 0.0 and abs(p[0] - p[1]) < 0.1 * p[0]               # longer requests get more; similar lengths, similar budgets
    assert p[3] == 0.0 and reqs[3][0] <= n                                    # a short generation skips speculation
    weak = [(l, a, 0.3) for l, a, _ in reqs]
    nw, jw = ob.scan_forward_passes(weak, c_base, c_tok, steps=4000)
    _, js = ob.scan_forward_passes(reqs, c_base, c_tok, steps=4000)
    assert nw > n and jw > js                                                 # a weak drafter bounds the gain
    # base-cost-dominant regime: the optimum drives the pass count towards its floor
    nb, _ = ob.scan_forward_passes(reqs, 1000.0, c_tok, steps=4000)
    assert nb < n and nb < 1.05 * 4000.0 * 0.2 + 40


def test_length_class_policy_counts():
    assert [ob.length_class(x, 100, 1000) for x in (0, 99, 100, 999, 1000, 5000)] == [0, 0, 1, 1, 2, 2]
    assert ob.class_init([5, 3, 1]) == 0 and ob.class_init([2, 7, 7]) == 2 and ob.class_init([0, 0, 0]) == 2
    hist_len = [50, 60, 70, 150, 400, 2000, 3000, 120, 90]
    hist_init = [0, 0, 0, 0, 0, 0, 1, 1, 1]
    # initial class short, nothing observed yet: most such requests ended short
    assert ob.class_update(hist_len, hist_init, 100, 1000, 0, 0) == 0
    # having already produced 130 tokens, the survivors are 150, 400 (medium) and 2000 (long): medium
    assert ob.class_update(hist_len, hist_init, 100, 1000, 130, 0) == 1
    # at 500 tokens only the long one is left
    assert ob.class_update(hist_len, hist_init, 100, 1000, 500, 0) == 2
    # no comparable history reached this length: the class of the observed length itself
    assert ob.class_update(hist_len, hist_init, 100, 1000, 2500, 0) == 2 and ob.class_update([], [], 100, 1000, 150, 1) == 1
