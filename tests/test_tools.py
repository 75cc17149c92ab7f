"""Host-side helpers of the measurement tools (no GPU): the line fit of the forward-latency model
(Sec. 4.2.1, Eq. 1), the closed form for a chain draft's emitted tokens, and the length-class budgets."""
import numpy as np

import das_inputs as di
from paper_2511_13841_amd.latency_model import expected_emitted, fit_line
from paper_2511_13841_amd.rollout_makespan import class_budgets, target_lengths


def test_fit_line_recovers_an_exact_line_and_reports_r2():
    x = np.array([128, 256, 640, 1152, 2176, 4224], float)
    a, b, r2 = fit_line(x, 3.5 + 0.004 * x)
    assert abs(a - 3.5) < 1e-9 and abs(b - 0.004) < 1e-12 and abs(r2 - 1.0) < 1e-12
    rng = np.random.default_rng(0)
    a, b, r2 = fit_line(x, 3.5 + 0.004 * x + rng.normal(0, 0.5, x.size))
    assert abs(b - 0.004) < 5e-4 and 0.9 < r2 < 1.0


def test_expected_emitted_is_the_mean_of_the_accept_length_distribution():
    # accept length a < k with probability q^a (1-q), a = k with probability q^k; a+1 tokens are emitted
    for p, k, V in [(0.7, 4, 2048), (0.6, 16, 151936), (0.8, 0, 100), (0.0, 8, 16)]:
        q = p + (1 - p) / V
        mean = sum((a + 1) * q ** a * (1 - q) for a in range(k)) + (k + 1) * q ** k
        assert abs(expected_emitted(p, k, V) - mean) < 1e-12
        assert abs(expected_emitted(p, k, V) - 1.0 - di.expected_accept_len(p, k, V)) < 1e-9


def test_uniform_budget_recipes_parse_any_k():
    import dataclasses
    wl = dataclasses.replace(di.WORKLOADS["c3"], budgets="k7")
    assert di.max_budget(wl) == 7 and (di.draft_budgets(wl, [5, 6, 7]) == 7).all()
    assert di.max_budget(di.WORKLOADS["c3"]) == 16 and di.max_budget(di.WORKLOADS["c5"]) == 32


def test_length_classes_and_long_tail():
    lens = target_lengths(300, 512, 7)
    assert lens.min() >= 4 and lens.max() == 512 and np.median(lens) < 128          # a tail, clipped at the cap
    b = class_budgets(lens, 4, 8)
    assert sorted(set(b.tolist())) == [0, 4, 8] and np.bincount(b // 4).tolist() == [100, 100, 100]
    assert lens[b == 8].min() >= lens[b == 4].max() >= lens[b == 4].min() >= lens[b == 0].max()
