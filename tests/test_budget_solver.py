"""The host-side budget solver behind include/das_budget.h against the plain definitions and brute force of oracle/budget.py
(Sec. 4.2.1, Eq. 3-9; Sec. 4.2.2).  Host arithmetic only: runs without a GPU."""
import math

import numpy as np
import pytest

from oracle import budget as ob
from paper_2511_13841_amd import budget as pb

BATCHES = [
    ([(4000.0, 1.0, 0.8), (3900.0, 1.0, 0.8), (1500.0, 1.0, 0.8), (200.0, 1.0, 0.8)], 10.0, 0.02),
    ([(400.0, 1.0, 0.9), (250.0, 0.8, 0.7)], 6.0, 0.05),
    ([(2000.0, 0.9, 1.0)], 10.0, 0.02),
    ([(300.0 + 37.0 * i, 0.6 + 0.05 * (i % 5), 0.5 + 0.04 * (i % 9)) for i in range(64)], 12.0, 0.03),
]


def test_definitions_equal_the_plain_ones():
    rng = np.random.default_rng(5)
    for reqs, c_base, c_tok in BATCHES:
        p = rng.uniform(0, 3000, size=len(reqs))
        for r, pi in zip(reqs, p):
            assert abs(pb.accepted(r, pi) - ob.accepted(r, pi)) <= 1e-12 * r[0]
        assert abs(pb.forward_passes(reqs, p) - ob.forward_passes(reqs, p)) <= 1e-9
        assert abs(pb.latency(reqs, p, c_base, c_tok, 3.5) - ob.latency(reqs, p, c_base, c_tok, 3.5)) <= 1e-9 * (1 + c_base * 4000)


def test_tight_budgets_equal_the_least_budgets_found_by_bisection():
    for reqs, _, _ in BATCHES:
        floor = max(l * (1 - k) for l, _, k in reqs)
        top = max(l for l, _, _ in reqs)
        for frac in (0.05, 0.5, 0.95, 1.0):
            n = floor + frac * (top - floor)
            p = pb.tight(reqs, n)
            for r, pi in zip(reqs, p):
                assert abs(pi - ob.least_budget(r, n)) <= 1e-6 * (1 + pi)
            assert abs(ob.forward_passes(reqs, p) - n) <= 1e-6 * n or n >= top       # every active constraint tight
        with pytest.raises(pb.BudgetError):
            pb.tight(reqs, floor if floor > 0 else -1.0)


def test_printed_closed_form_coincides_only_at_full_capacity():
    full = [(2000.0, 0.9, 1.0), (500.0, 1.2, 1.0)]
    assert np.allclose(pb.tight(full, 300.0), pb.tight_printed(full, 300.0), rtol=1e-12)
    part = [(2000.0, 0.9, 0.7)]
    n = 1000.0
    assert pb.tight_printed(part, n)[0] < pb.tight(part, n)[0]                       # the printed budget is too small ...
    assert ob.forward_passes(part, pb.tight_printed(part, n)) > n + 1.0               # ... and leaves more than n tokens


def test_slope_is_the_derivative_of_the_latency_along_the_tight_budgets():
    for reqs, c_base, c_tok in BATCHES:
        floor = max(l * (1 - k) for l, _, k in reqs)
        top = max(l for l, _, _ in reqs)
        for frac in (0.2, 0.6, 0.9):
            n = floor + frac * (top - floor)
            h = 1e-4 * top
            if any(abs(l - n) < 2 * h for l, _, _ in reqs):
                continue                                                               # kink where a request drops out
            num = (ob.latency_at(reqs, n + h, c_base, c_tok) - ob.latency_at(reqs, n - h, c_base, c_tok)) / (2 * h)
            assert abs(pb.slope(reqs, c_base, c_tok, n) - num) <= 1e-4 * (abs(num) + c_base)


def test_solver_finds_the_minimum_the_scan_finds():
    for reqs, c_base, c_tok in BATCHES:
        n_star, p_star = pb.solve(reqs, c_base, c_tok)
        top = max(l for l, _, _ in reqs)
        n_scan, j_scan = ob.scan_forward_passes(reqs, c_base, c_tok, steps=4000)
        j_star = ob.latency(reqs, p_star, c_base, c_tok)
        assert j_star <= j_scan + 1e-9 * j_scan                                        # at least as good as any grid point
        assert abs(n_star - n_scan) <= 2 * top / 4000 + 1e-6
        assert abs(ob.forward_passes(reqs, p_star) - n_star) <= 1e-6 * n_star
        for (l, _, _), pi in zip(reqs, p_star):
            assert (pi == 0.0) == (l <= n_star)                                        # short requests skip speculation
    # one request: the optimum derived by hand from Eq. 3-5
    l, alpha, k, c_base, c_tok = 1000.0, 0.5, 0.5, 8.0, 0.1
    n_star, _ = pb.solve([(l, alpha, k)], c_base, c_tok)
    assert abs(n_star - l * (1 - k + c_tok / (alpha * c_base))) <= 1e-6 * l


def test_no_speculation_when_it_cannot_pay():
    reqs = [(300.0, 1.0, 0.9), (100.0, 1.0, 0.9)]
    n_star, p_star = pb.solve(reqs, 1.0, 2.0)                                          # c_tok / (alpha k) > c_base
    assert n_star == 300.0 and not p_star.any()


def test_draft_lens_and_error_codes():
    assert pb.draft_lens([0.0, 900.0, 5100.0, 40000.0], 1000.0, 16).tolist() == [0, 0, 4, 16]
    with pytest.raises(pb.BudgetError):
        pb.solve([(100.0, 1.0, 1.2)], 1.0, 0.1)                                        # k outside (0, 1]
    with pytest.raises(pb.BudgetError):
        pb.accepted((100.0, -1.0, 0.5), 1.0)


def test_length_class_policy_equals_plain_counting():
    rng = np.random.default_rng(11)
    fl = np.round(512 * (1 - rng.random(400)) ** (-1 / 1.5)).clip(1, 32768)
    ini = rng.integers(0, 3, size=400)
    for t_m, t_l in [(1024, 8192), (700, 700)]:
        for x in (0, 100, 1024, 5000, 8192, 40000):
            assert pb.length_class(x, t_m, t_l) == ob.length_class(x, t_m, t_l)
        for partial in (0, 600, 1500, 9000, 50000):
            for c in range(3):
                assert pb.class_update(fl, ini, t_m, t_l, partial, c) == ob.class_update(fl, ini, t_m, t_l, partial, c)
    for counts in ([5, 3, 1], [2, 7, 7], [0, 0, 0], [4, 4, 1]):
        assert pb.class_init(counts) == ob.class_init(counts)
