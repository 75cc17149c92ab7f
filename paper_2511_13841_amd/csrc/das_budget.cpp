// Length-aware speculative-token budget (Sec. 4.2 of the paper): host arithmetic behind include/das_budget.h.
#include "../../include/das_budget.h"

#include <algorithm>
#include <cmath>
#include <limits>

namespace {

bool ok_request(const das_request &q) {
    return q.length > 0.0 && q.alpha > 0.0 && q.cap > 0.0 && q.cap <= 1.0 && std::isfinite(q.length) && std::isfinite(q.alpha);
}
bool ok_batch(const das_request *r, int32_t n) {
    if (!r || n < 1) return false;
    for (int32_t i = 0; i < n; ++i)
        if (!ok_request(r[i])) return false;
    return true;
}
// tokens left after p proposed (l - A(p), Eq. 3)
double remaining(const das_request &q, double p) { return q.length * (1.0 - q.cap + q.cap * std::exp(-q.alpha * p / q.length)); }

// dJ/dN for the tight budgets; requests with l_i <= N do not speculate
double slope(const das_request *r, int32_t n, double c_base, double c_tok, double N) {
    double s = 0.0;
    for (int32_t i = 0; i < n; ++i)
        if (r[i].length > N) s += 1.0 / (r[i].alpha * (r[i].cap - 1.0 + N / r[i].length));
    return c_base - c_tok * s;
}

}  // namespace

extern "C" int das_budget_accepted(const das_request *r, double p, double *accepted) {
    if (!r || !accepted || !ok_request(*r) || !(p >= 0.0)) return DAS_BUDGET_ERR_INVALID;
    *accepted = r->length - remaining(*r, p);
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_forward_passes(const das_request *r, int32_t n, const double *p, double *n_fwd) {
    if (!ok_batch(r, n) || !p || !n_fwd) return DAS_BUDGET_ERR_INVALID;
    double m = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        if (!(p[i] >= 0.0)) return DAS_BUDGET_ERR_INVALID;
        m = std::max(m, remaining(r[i], p[i]));
    }
    *n_fwd = m;
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_latency(const das_request *r, int32_t n, const double *p, double c_base, double c_tok, double c_other,
                                  double *latency) {
    double nf = 0.0;
    if (!latency) return DAS_BUDGET_ERR_INVALID;
    const int rc = das_budget_forward_passes(r, n, p, &nf);
    if (rc != DAS_BUDGET_OK) return rc;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += p[i];
    *latency = c_base * nf + c_tok * sum + c_other;
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_tight(const das_request *r, int32_t n, double n_fwd, double *p_out) {
    if (!ok_batch(r, n) || !p_out || !(n_fwd > 0.0)) return DAS_BUDGET_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i)
        if (r[i].length > n_fwd && !(n_fwd > r[i].length * (1.0 - r[i].cap))) return DAS_BUDGET_ERR_RANGE;
    for (int32_t i = 0; i < n; ++i) {
        const das_request &q = r[i];
        p_out[i] = q.length > n_fwd ? -(q.length / q.alpha) * std::log(1.0 - (1.0 - n_fwd / q.length) / q.cap) : 0.0;
    }
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_tight_printed(const das_request *r, int32_t n, double n_fwd, double *p_out) {
    if (!ok_batch(r, n) || !p_out || !(n_fwd > 0.0)) return DAS_BUDGET_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i) {
        const das_request &q = r[i];
        p_out[i] = q.length > n_fwd ? -(q.length / q.alpha) * std::log(1.0 - q.cap * (1.0 - n_fwd / q.length)) : 0.0;
    }
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_slope(const das_request *r, int32_t n, double c_base, double c_tok, double n_fwd, double *out) {
    if (!ok_batch(r, n) || !out || !(n_fwd > 0.0) || !(c_base >= 0.0) || !(c_tok >= 0.0)) return DAS_BUDGET_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i)
        if (r[i].length > n_fwd && !(n_fwd > r[i].length * (1.0 - r[i].cap))) return DAS_BUDGET_ERR_RANGE;
    *out = slope(r, n, c_base, c_tok, n_fwd);
    return DAS_BUDGET_OK;
}

extern "C" int das_budget_solve(const das_request *r, int32_t n, double c_base, double c_tok, double *n_fwd, double *p_out) {
    if (!ok_batch(r, n) || !n_fwd || !p_out || !(c_base >= 0.0) || !(c_tok > 0.0)) return DAS_BUDGET_ERR_INVALID;
    double hi = 0.0, lo = 0.0;           // J is defined on (lo, hi]: lo = largest floor l_i (1 - k_i), hi = longest request
    for (int32_t i = 0; i < n; ++i) {
        hi = std::max(hi, r[i].length);
        lo = std::max(lo, r[i].length * (1.0 - r[i].cap));
    }
    double N = hi;
    // dJ/dN rises from -inf at lo (or from c_base - c_tok sum 1/(alpha N/l) > -inf when every k_i = 1 and lo = 0) to its
    // value just below hi; a root exists iff that value is positive, otherwise J falls all the way and p = 0 is optimal
    const double just_below = std::nextafter(hi, 0.0);
    if (slope(r, n, c_base, c_tok, just_below) > 0.0) {
        double a = lo, b = just_below;   // slope(a+) < 0 < slope(b)
        for (int it = 0; it < 200; ++it) {
            const double m = 0.5 * (a + b);
            if (!(m > a) || !(m < b)) break;
            if (slope(r, n, c_base, c_tok, m) > 0.0) b = m; else a = m;
        }
        N = b;
    }
    *n_fwd = N;
    return das_budget_tight(r, n, N, p_out);
}

extern "C" int das_budget_draft_lens(const double *p, int32_t n, double n_fwd, int32_t k_max, int32_t *k_out) {
    if (!p || !k_out || n < 1 || !(n_fwd > 0.0) || k_max < 0) return DAS_BUDGET_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i)
        if (!(p[i] >= 0.0)) return DAS_BUDGET_ERR_INVALID;
    for (int32_t i = 0; i < n; ++i) {
        const double per_pass = std::floor(p[i] / n_fwd + 0.5);
        const double k = p[i] > 0.0 ? per_pass - 1.0 : 0.0;
        k_out[i] = (int32_t)std::min<double>(k_max, std::max(0.0, k));
    }
    return DAS_BUDGET_OK;
}

extern "C" int das_length_class(double length, double t_medium, double t_long, int32_t *cls) {
    if (!cls || !(length >= 0.0) || !(t_medium <= t_long)) return DAS_BUDGET_ERR_INVALID;
    *cls = length >= t_long ? 2 : length >= t_medium ? 1 : 0;
    return DAS_BUDGET_OK;
}

extern "C" int das_length_class_init(const int64_t *counts, int32_t *cls) {
    if (!counts || !cls || counts[0] < 0 || counts[1] < 0 || counts[2] < 0) return DAS_BUDGET_ERR_INVALID;
    int32_t best = 0;
    for (int32_t c = 1; c < 3; ++c)
        if (counts[c] >= counts[best]) best = c;
    *cls = best;
    return DAS_BUDGET_OK;
}

extern "C" int das_length_class_update(const double *hist_final_len, const int32_t *hist_init, int32_t n_hist, double t_medium,
                                       double t_long, double partial_len, int32_t init_cls, int32_t *cls) {
    if (!cls || n_hist < 0 || (n_hist > 0 && (!hist_final_len || !hist_init)) || !(partial_len >= 0.0) || !(t_medium <= t_long) ||
        init_cls < 0 || init_cls > 2)
        return DAS_BUDGET_ERR_INVALID;
    int64_t counts[3] = {0, 0, 0};
    for (int32_t i = 0; i < n_hist; ++i) {
        if (hist_init[i] != init_cls || !(hist_final_len[i] >= partial_len)) continue;
        int32_t c = 0;
        das_length_class(hist_final_len[i], t_medium, t_long, &c);
        ++counts[c];
    }
    int32_t floor_cls = 0;
    das_length_class(partial_len, t_medium, t_long, &floor_cls);
    if (counts[0] + counts[1] + counts[2] == 0) { *cls = floor_cls; return DAS_BUDGET_OK; }
    int32_t best = 0;
    das_length_class_init(counts, &best);
    *cls = std::max(best, floor_cls);
    return DAS_BUDGET_OK;
}
