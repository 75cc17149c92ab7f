/*
 * das_budget.h -- host-side C ABI of the length-aware speculative-token budget (Sec. 4.2 of the paper).
 *
 * Everything here is plain host arithmetic: no device, no model.  All pointers are host memory owned by the caller.
 * Every call returns DAS_BUDGET_OK (0) or a negative code and writes nothing on failure.
 *
 * Model (Sec. 4.2.1).  Request i has a target generation length l_i > 0, an accept efficiency alpha_i > 0 and a
 * drafter capacity factor k_i in (0, 1].  With p_i tokens proposed in total it gets A_i(p_i) = k_i l_i (1 - exp(-alpha_i p_i / l_i))
 * tokens accepted (Eq. 3); l_i - A_i remain; the batch needs N_fwd = max_i (l_i - A_i(p_i)) forward passes (Eq. 4); the rollout
 * latency is J(p) = c_base N_fwd + c_tok sum_i p_i + C (Eq. 5).
 *
 * Reading used for the optimum.  Minimising J under the constraints of Eq. 6 makes the constraint of every request with
 * l_i > N_fwd tight: l_i (1 - k_i + k_i exp(-alpha_i p_i / l_i)) = N_fwd, i.e.
 *     p_i(N_fwd) = -(l_i / alpha_i) ln(1 - (1 - N_fwd / l_i) / k_i),   defined for N_fwd > l_i (1 - k_i),   0 for N_fwd >= l_i.
 * The closed form printed as Eq. 7, -(l_i / alpha_i) ln(1 - k_i (1 - N_fwd / l_i)), satisfies that equation only for k_i = 1;
 * it is kept as das_budget_tight_printed for comparison.  With the tight form J(N_fwd) is convex with
 *     dJ/dN = c_base - c_tok sum_{i: l_i > N} 1 / (alpha_i (k_i - 1 + N / l_i))            (the counterpart of Eq. 9)
 * and das_budget_solve finds its root by bisection; if dJ/dN < 0 up to max_i l_i, speculation does not pay and p = 0.
 */
#ifndef DAS_BUDGET_H
#define DAS_BUDGET_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DAS_BUDGET_OK            0
#define DAS_BUDGET_ERR_INVALID  (-1)   /* null pointer, n < 1, or a parameter outside its domain */
#define DAS_BUDGET_ERR_RANGE    (-2)   /* N_fwd at or below a request's floor l_i (1 - k_i): no finite budget reaches it */

typedef struct {
    double length;   /* l_i     > 0 */
    double alpha;    /* alpha_i > 0 */
    double cap;      /* k_i in (0, 1] */
} das_request;

/* Eq. 3: tokens accepted out of p >= 0 proposed. */
int das_budget_accepted(const das_request *r, double p, double *accepted);
/* Eq. 4: forward passes the batch needs under budgets p[n]. */
int das_budget_forward_passes(const das_request *r, int32_t n, const double *p, double *n_fwd);
/* Eq. 5: rollout latency under budgets p[n]; c_other is the paper's C. */
int das_budget_latency(const das_request *r, int32_t n, const double *p, double c_base, double c_tok, double c_other, double *latency);
/* Budgets that make every constraint of Eq. 6 tight at a given N_fwd (see the header comment); p_out[n]. */
int das_budget_tight(const das_request *r, int32_t n, double n_fwd, double *p_out);
/* The same with the closed form as printed (Eq. 7). */
int das_budget_tight_printed(const das_request *r, int32_t n, double n_fwd, double *p_out);
/* dJ/dN at n_fwd for the tight budgets (counterpart of Eq. 9). */
int das_budget_slope(const das_request *r, int32_t n, double c_base, double c_tok, double n_fwd, double *slope);
/* Minimiser of J: writes N_fwd* and the budgets p*[n]. */
int das_budget_solve(const das_request *r, int32_t n, double c_base, double c_tok, double *n_fwd, double *p_out);
/* Per-round chain lengths from total budgets: request i processes p_i tokens over about N_fwd passes, one of them per pass
 * its own (non-speculative) token, so k_i = round(p_i / N_fwd) - 1 clamped to [0, k_max]; 0 where p_i = 0. */
int das_budget_draft_lens(const double *p, int32_t n, double n_fwd, int32_t k_max, int32_t *k_out);

/* ---- length-class policy (Sec. 4.2.2): 0 = Short (no speculation), 1 = Medium, 2 = Long ---- */
/* Class of a (final or predicted) length given the two thresholds t_medium <= t_long. */
int das_length_class(double length, double t_medium, double t_long, int32_t *cls);
/* Initial class from history: the class that most comparable past requests fell into (counts[3]; ties go to the longer class). */
int das_length_class_init(const int64_t *counts, int32_t *cls);
/* Runtime update: argmax_c P(c | observed partial length, initial class), P estimated from past requests with the same
 * initial class that reached at least the observed length (hist_final_len[n_hist], hist_init[n_hist]); if none did, the
 * class of the observed length itself (never below it); ties go to the longer class. */
int das_length_class_update(const double *hist_final_len, const int32_t *hist_init, int32_t n_hist, double t_medium, double t_long,
                            double partial_len, int32_t init_cls, int32_t *cls);

#ifdef __cplusplus
}
#endif
#endif /* DAS_BUDGET_H */
