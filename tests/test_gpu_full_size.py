"""Parity at the benchmark's full sizes, in the launch configuration bench.py times, over several rounds.

The whole batch of a config runs verification rounds on the GPU (full model, full batch, full context lengths; the
contexts are the keyed synthetic KV that das_kv_synth writes on the device).  The oracle recomputes SAMPLED sequences
one by one from the same inputs (same bf16 weights widened to fp32, same synthetic KV, same drafts): sequences of a
verify step are independent, so a sampled sequence inside the full ragged batch must equal the oracle's stand-alone
result.  Per round:
  * the drafts of a sampled sequence are the oracle's own greedy continuation with every position kept with the
    config's acceptance probability (so accepted prefixes longer than one occur) -- the oracle decodes ahead only up
    to the first position the drafter gets wrong, since nothing behind it can be accepted; the other sequences get
    random drafts;
  * logits, row argmaxes and decisions of the sampled sequences are compared under the usual protocol;
  * the ORACLE's decision is committed for the sampled sequences (teacher forcing), the GPU's own for the others;
  * committed length, pending token, page list of EVERY sequence of the batch and the free-page count are compared
    with the integer mirror.
Config 4 includes its longest sequence (above 60k tokens) in the sample.  The stochastic config also checks every
token the GPU sampled in the batch against fp64 prefix sums of the GPU's own logits (the window under the oracle's
weights is wide at this logit error).
"""
import numpy as np
import pytest

import das_inputs as di
import oracle
from conftest import progress
from parity_harness import StepReport, compare_greedy_step, compare_stochastic_step, check_bookkeeping

pytestmark = pytest.mark.gpu

ROUNDS = 3


@pytest.fixture(scope="module")
def weights():
    cache = {}

    def get(model):
        if model not in cache:
            cache.clear()                                   # one big model at a time in host memory
            shape = di.MODELS[model]
            blob = di.weights_bf16(shape, seed=0)
            cache[model] = (blob, oracle.OracleModel(shape, di.bf16_to_f32(blob)))
        return cache[model]
    return get


def _oracle_seq(om, shape, seed, sid, ctx, pending, room):
    s = om.new_seq(ctx + room)
    for layer in range(shape.n_layers):
        s.kv(layer, 0)[:ctx] = di.bf16_to_f32(di.kv_synth(seed, sid, layer, 0, 0, ctx, shape.n_kv_heads, shape.head_dim))
        s.kv(layer, 1)[:ctx] = di.bf16_to_f32(di.kv_synth(seed, sid, layer, 1, 0, ctx, shape.n_kv_heads, shape.head_dim))
    s.len, s.pending = ctx, int(pending)
    return s


def _sample_ids(name, ctx, ks):
    order = np.argsort(ctx, kind="stable")
    picks = [int(order[0]), int(order[-1])]                                        # shortest, LONGEST
    if name != "c4":                                                               # (every c4 sequence is long and has k = 16)
        picks.append(int(order[len(order) // 2]))
        picks.append(int(max(range(len(ctx)), key=lambda i: (ks[i], -ctx[i]))))    # the largest budget (shortest such)
    if name == "c5":
        picks.append(int(min(range(len(ctx)), key=lambda i: (ks[i], ctx[i]))))     # and a sequence without drafts
    return sorted(set(picks))


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_size_rounds_against_oracle_on_sampled_sequences(name, weights):
    import paper_2511_13841_amd as das
    wl = di.WORKLOADS[name]
    shape = di.MODELS[wl.model]
    blob, om = weights(wl.model)
    ctx = di.context_lengths(wl).astype(np.int64)
    B = wl.batch
    kmax = di.max_budget(wl)
    grow = ROUNDS * (kmax + 1) + kmax + 2
    pages = int(sum(-(-(int(c) + grow) // 16) for c in ctx)) + 8
    Tmax = B * (kmax + 1)
    progress(f"{name}: B={B} kv_tokens={int(ctx.sum())} pages={pages} longest={int(ctx.max())}")
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=-(-(int(ctx.max()) + grow + 16) // 16) * 16, max_rows=max(Tmax, 256),
                                     max_draft=max(kmax, 1), num_pages=pages), blob)
    mirror = oracle.PageTableMirror(pages)
    rng = np.random.default_rng(wl.seed)
    pend = rng.integers(0, shape.vocab, size=B, dtype=np.int32)
    ids = list(range(B))
    for i in ids:
        dm.seq_create(i, int(ctx[i]), int(pend[i]))
        dm.kv_synth(i, wl.seed, i)
    mirror.prefill(ids, [int(c) for c in ctx])
    picks = _sample_ids(name, ctx, di.draft_budgets(wl, ctx))
    if name == "c4":
        assert max(int(ctx[i]) for i in picks) > 60000
    seqs = {i: _oracle_seq(om, shape, wl.seed, i, int(ctx[i]), pend[i], grow) for i in picks}
    rep = StepReport()
    exact = flagged = sampled_checked = 0
    accepted_sampled = 0
    for rnd in range(ROUNDS):
        ks = di.draft_budgets(wl, ctx)
        T = int((ks + 1).sum())
        drafts = [rng.integers(0, shape.vocab, size=int(k), dtype=np.int32) for k in ks]
        for i in picks:
            if wl.mode == "greedy" and ks[i] > 0:
                # the synthetic drafter on the oracle's continuation: positions are right with probability p; behind
                # the first wrong one the chain cannot be accepted, so the oracle decodes ahead only that far
                wrong = np.nonzero(rng.random(int(ks[i])) >= wl.accept_p)[0]
                n_true = int(wrong[0]) if wrong.size else int(ks[i])
                s = seqs[i]
                n0, p0, t0 = s.len, s.pending, list(s.tokens)
                progress(f"  oracle decodes {n_true} tokens ahead for sequence {i} (ctx {n0})")
                drafts[i][:n_true] = om.ar_greedy(s, n_true)
                s.len, s.pending, s.tokens = n0, p0, t0
        row0 = np.concatenate([[0], np.cumsum(ks + 1)])
        sampling = None
        if wl.mode == "stochastic":
            keys = np.repeat(np.arange(B), ks + 1)
            pos = np.concatenate([np.arange(ctx[i], ctx[i] + ks[i] + 1) for i in ids])
            ua = di.uniforms(wl.seed, keys, pos, 0)
            us = di.uniforms(wl.seed, keys, pos, 1)
            ua = np.where(rng.random(ua.size) < wl.accept_p, 0.0, ua).astype(np.float32)      # controlled mode: forced acceptances
            sampling = (wl.temperature, ua, us)
        progress(f"round {rnd}: rows={T}")
        acc, nx = dm.verify_step(ids, ctx, drafts, sampling)
        mirror.verify(ids, [int(k) for k in ks])
        gg = None
        if sampling is None:
            gg = dm.debug_row_argmax()
            if rnd == 0:
                # that was the production path: row maxima gathered inside the LM-head GEMM, no logits in memory.  The
                # same step with the logits written out and scanned must take the same decisions, bit for bit.
                with pytest.raises(das.DasError):
                    dm.debug_logits(0, 1)
                dm.kv_rollback(ids)
                mirror.rollback(ids)
                dm.keep_logits(True)
                acc2, nx2 = dm.verify_step(ids, ctx, drafts, sampling)
                mirror.verify(ids, [int(k) for k in ks])
                assert np.array_equal(gg, dm.debug_row_argmax()) and np.array_equal(acc, acc2) and np.array_equal(nx, nx2)
        elif rnd == 0:
            # production path of a sampling pass first (no logits kept), then the same step in inspection mode:
            # identical decisions
            dm.kv_rollback(ids)
            mirror.rollback(ids)
            dm.keep_logits(True)
            acc2, nx2 = dm.verify_step(ids, ctx, drafts, sampling)
            mirror.verify(ids, [int(k) for k in ks])
            assert np.array_equal(acc, acc2) and np.array_equal(nx, nx2)
        c_acc, c_nx = [int(a) for a in acc], [int(t) for t in nx]
        for i in picks:
            n = int(ks[i]) + 1
            glog = dm.debug_logits(int(row0[i]), n)
            s = seqs[i]
            progress(f"  oracle for sequence {i}: ctx={s.len} k={int(ks[i])}")
            if sampling is None:
                a, t, lo = om.verify_greedy(s, drafts[i])
                compare_greedy_step(rep, glog, gg[row0[i]:row0[i] + n], acc[i], nx[i], lo, a, t, drafts[i])
                accepted_sampled += a
            else:
                sl = slice(int(row0[i]), int(row0[i]) + n)
                a, t, lo = om.verify_stochastic(s, drafts[i], wl.temperature, ua[sl], us[sl])
                ok = compare_stochastic_step(glog, acc[i], nx[i], lo, drafts[i], wl.temperature, ua[sl], us[sl])
                exact += bool(ok); flagged += not ok
                rep.max_rel_logit_err = max(rep.max_rel_logit_err, float(np.abs(glog - lo).max() / np.abs(lo).max()))
            om.commit(s, a, t, drafts[i])
            c_acc[i], c_nx[i] = a, t                       # teacher forcing on the sampled sequences
        if sampling is not None:
            # every token the batch sampled, against fp64 prefix sums of the GPU's own logits of the row it came from
            for i in ids:
                a, v = int(acc[i]), int(nx[i])
                r = int(row0[i]) + a
                l = dm.debug_logits(r, 1)[0].astype(np.float64) / wl.temperature
                w = np.exp(l - l.max())
                if a < ks[i]:
                    w[int(drafts[i][a])] = 0.0
                    assert v != int(drafts[i][a])
                cs = np.cumsum(w)
                u = float(us[r]) * cs[-1]
                lo_edge = cs[v - 1] if v > 0 else 0.0
                assert w[v] > 0 and lo_edge - 1e-4 * cs[-1] <= u <= cs[v] + 1e-4 * cs[-1], (i, v, u, lo_edge, cs[v])
                sampled_checked += 1
        # properties of the whole batch: every decision follows from the row argmaxes / is in range
        for i in ids:
            assert 0 <= acc[i] <= ks[i] and 0 <= nx[i] < shape.vocab
            if sampling is None:
                g = gg[row0[i]:row0[i + 1]]
                a = 0
                while a < ks[i] and drafts[i][a] == g[a]:
                    a += 1
                assert (int(acc[i]), int(nx[i])) == (a, int(g[a]))
        dm.kv_commit(ids, c_acc, c_nx)
        mirror.commit(ids, c_acc)
        check_bookkeeping(dm, mirror, ids, c_nx)           # the WHOLE batch, every round
        ctx = ctx + 1 + np.array(c_acc, dtype=np.int64)
        rep.steps += 1
    progress(name, rep, f"stochastic: exact={exact} flagged={flagged} sampled tokens checked={sampled_checked}; "
             f"accepted drafts on sampled sequences={accepted_sampled}")
    assert rep.max_rel_logit_err < 3e-2
    assert dm.debug_kv_saturated() == 0
    if wl.mode == "greedy":
        assert rep.decisions == ROUNDS * len(picks)
        assert accepted_sampled >= 2                       # accepted prefixes did occur
        assert rep.rows - rep.flagged_rows > 0
    else:
        assert exact >= 1 and flagged <= (exact + flagged) // 2, (exact, flagged)
        assert sampled_checked == ROUNDS * B
    dm.free()
    for s in seqs.values():
        s.close()
