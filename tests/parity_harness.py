"""GPU-vs-oracle comparison protocol shared by the `-m gpu` parity tests.

Per verify step, same inputs on both sides:
 (1) logits: max |delta| <= 3e-2 * max |oracle logit| over the step;
 (2) every row whose oracle top-1/top-2 margin exceeds 0.1 must have the same
     greedy token; accept_len / next_token must be bit-exact when every
     decision row 0..a_oracle clears the margin, otherwise the sequence-step
     is flagged (counted, mismatch allowed);
 (3) teacher forcing: the ORACLE's decision is committed on both sides, so one
     flipped near-tie cannot desynchronise the run;
 (4) committed length, pending token and page lists are compared bit-exactly
     with the integer mirror every step.
"""
import numpy as np

LOGIT_RTOL = 3e-2
MARGIN = 0.1


def top2_margin(logits):
    part = np.partition(logits, -2, axis=1)
    return part[:, -1] - part[:, -2]


class StepReport:
    def __init__(self):
        self.steps = 0
        self.rows = 0
        self.flagged_rows = 0
        self.flagged_decisions = 0
        self.decisions = 0
        self.mismatched_flagged = 0
        self.max_rel_logit_err = 0.0

    def __repr__(self):
        return (f"steps={self.steps} rows={self.rows} flagged_rows={self.flagged_rows} decisions={self.decisions} "
                f"flagged_decisions={self.flagged_decisions} mismatched_flagged={self.mismatched_flagged} "
                f"max_rel_logit_err={self.max_rel_logit_err:.3e}")


def compare_greedy_step(rep, gpu_logits, gpu_g, gpu_accept, gpu_next, oracle_logits, oracle_accept, oracle_next, drafts):
    """One sequence of one step.  Raises AssertionError on a parity violation."""
    scale = float(np.abs(oracle_logits).max())
    err = float(np.abs(gpu_logits.astype(np.float64) - oracle_logits.astype(np.float64)).max())
    rep.max_rel_logit_err = max(rep.max_rel_logit_err, err / scale)
    assert err <= LOGIT_RTOL * scale, f"logit error {err:.4g} > {LOGIT_RTOL}*{scale:.4g}"
    margin = top2_margin(oracle_logits)
    g_o = np.argmax(oracle_logits, axis=1)
    clear = margin > MARGIN
    rep.rows += len(margin)
    rep.flagged_rows += int((~clear).sum())
    assert np.array_equal(np.asarray(gpu_g)[clear], g_o[clear]), "greedy token differs on a row with margin > 0.1"
    rep.decisions += 1
    if clear[: oracle_accept + 1].all():
        assert (int(gpu_accept), int(gpu_next)) == (int(oracle_accept), int(oracle_next)), \
            f"decision differs: gpu ({gpu_accept},{gpu_next}) oracle ({oracle_accept},{oracle_next})"
    else:
        rep.flagged_decisions += 1
        if (int(gpu_accept), int(gpu_next)) != (int(oracle_accept), int(oracle_next)):
            rep.mismatched_flagged += 1
    # whatever the ties, the GPU's own decision must follow from its own greedy tokens
    a = 0
    while a < len(drafts) and int(drafts[a]) == int(gpu_g[a]):
        a += 1
    assert (int(gpu_accept), int(gpu_next)) == (a, int(gpu_g[a])), "accept kernel disagrees with the row argmaxes"


def check_bookkeeping(dm, mirror, seq_ids, pendings):
    for sid, pend in zip(seq_ids, pendings):
        st = dm.debug_seq(sid)
        assert st["ctx_len"] == mirror.len[sid], (sid, st, mirror.len[sid])
        assert st["pending"] == int(pend)
        assert st["pages"] == mirror.pages[sid], (sid, st["pages"], mirror.pages[sid])
    assert dm.debug_free_pages() == len(mirror.free)


def check_sampled_token(w, u, v, eps):
    """The GPU's token v must satisfy u*Z in [prefix(v-1) - eps*Z, prefix(v) + eps*Z] under the oracle's weights."""
    cs = np.cumsum(w)
    Z = cs[-1]
    lo = cs[v - 1] if v > 0 else 0.0
    assert w[v] > 0.0, "sampled a zero-weight token"
    assert lo - eps * Z <= u * Z <= cs[v] + eps * Z, (v, u * Z, lo, cs[v], eps * Z)


def compare_stochastic_step(gpu_logits, gpu_accept, gpu_next, oracle_logits, drafts, tau, u_accept, u_sample):
    """One sequence of one stochastic step.  Returns True when the decision was compared exactly, False when it
    was flagged (a uniform within e^{+-0.1} of an accept probability on the way to the oracle's decision)."""
    from oracle import softmax_weights, stochastic_accept
    err = float(np.abs(gpu_logits.astype(np.float64) - oracle_logits.astype(np.float64)).max())
    assert err <= LOGIT_RTOL * float(np.abs(oracle_logits).max())
    a, _ = stochastic_accept(oracle_logits, drafts, tau, u_accept, u_sample)
    k = len(drafts)
    for j in range(min(a + 1, k)):
        w, Z = softmax_weights(oracle_logits[j], tau)
        pd = w[int(drafts[j])] / Z
        if pd * np.exp(-0.1) <= float(u_accept[j]) <= pd * np.exp(0.1):
            return False
    assert int(gpu_accept) == a, (int(gpu_accept), a)
    w, _ = softmax_weights(oracle_logits[a], tau)
    if a < k:
        w = w.copy()
        w[int(drafts[a])] = 0.0
        assert int(gpu_next) != int(drafts[a])
    check_sampled_token(w, float(u_sample[a]), int(gpu_next), np.exp(2 * err / tau) - 1 + 1e-6)
    return True
