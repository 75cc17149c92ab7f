"""Plain definitions of the paper's speculative-token budget model (Sec. 4.2.1) and a brute-force minimiser.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else).  Shares no code with the product.

Everything is written from the definitions, with no closed form for the optimum:
  A_i(p)   = k_i l_i (1 - exp(-alpha_i p / l_i))                      Eq. 3
  N_fwd(p) = max_i (l_i - A_i(p_i))                                   Eq. 4
  J(p)     = c_base N_fwd(p) + c_tok sum_i p_i + C                    Eq. 5
The least budget that brings request i down to N remaining tokens is found by bisection on p in Eq. 3 itself, and
J is minimised by scanning N (and, for two requests, by scanning the (p_1, p_2) plane directly).
A request is a tuple (l, alpha, k).
"""
import math


def accepted(req, p):
    l, alpha, k = req
    return k * l * (1.0 - math.exp(-alpha * p / l))


def forward_passes(reqs, p):
    return max(l - accepted((l, a, k), pi) for (l, a, k), pi in zip(reqs, p))


def latency(reqs, p, c_base, c_tok, c_other=0.0):
    return c_base * forward_passes(reqs, p) + c_tok * sum(p) + c_other


def least_budget(req, n_fwd, p_max=1e9):
    """Smallest p >= 0 with l - A(p) <= n_fwd, by bisection on Eq. 3; math.inf if no p reaches it."""
    l, alpha, k = req
    if l <= n_fwd:
        return 0.0
    if n_fwd <= l - k * l:          # A(p) -> k l only as p -> inf (the limit the paper states): l - k l is never reached
        return math.inf
    lo, hi = 0.0, p_max
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if l - accepted(req, mid) <= n_fwd:
            hi = mid
        else:
            lo = mid
    return hi


def latency_at(reqs, n_fwd, c_base, c_tok):
    """J when every request gets the least budget that leaves it at most n_fwd tokens."""
    return c_base * n_fwd + c_tok * sum(least_budget(r, n_fwd) for r in reqs)


def scan_forward_passes(reqs, c_base, c_tok, steps=20000):
    """(N, J) minimising latency_at over a uniform grid of N in (0, max l]."""
    top = max(l for l, _, _ in reqs)
    best = (top, latency_at(reqs, top, c_base, c_tok))
    for s in range(1, steps):
        n = top * s / steps
        j = latency_at(reqs, n, c_base, c_tok)
        if j < best[1]:
            best = (n, j)
    return best


def scan_budget_plane(reqs, c_base, c_tok, p_top, steps=400):
    """Brute force over a (p_1, p_2) grid for two requests: (J, p_1, p_2) of the best grid point."""
    assert len(reqs) == 2
    best = (math.inf, 0.0, 0.0)
    for a in range(steps + 1):
        for b in range(steps + 1):
            p = (p_top * a / steps, p_top * b / steps)
            j = latency(reqs, p, c_base, c_tok)
            if j < best[0]:
                best = (j, p[0], p[1])
    return best


# ---- length classes (Sec. 4.2.2): 0 short, 1 medium, 2 long

def length_class(length, t_medium, t_long):
    return 2 if length >= t_long else 1 if length >= t_medium else 0


def class_init(counts):
    """Most frequent class among comparable past requests; ties to the longer class."""
    return max(range(3), key=lambda c: (counts[c], c))


def class_update(hist_final_len, hist_init, t_medium, t_long, partial_len, init_cls):
    """argmax_c P(c | partial length, initial class) from past requests with that initial class that reached at least
    the partial length; never below the class of the partial length itself; that class if no past request qualifies."""
    counts = [0, 0, 0]
    for fl, ini in zip(hist_final_len, hist_init):
        if ini == init_cls and fl >= partial_len:
            counts[length_class(fl, t_medium, t_long)] += 1
    floor_cls = length_class(partial_len, t_medium, t_long)
    if sum(counts) == 0:
        return floor_cls
    return max(class_init(counts), floor_cls)
