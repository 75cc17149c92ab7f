"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The whole batch of a config runs one verify step on the GPU (full model, full batch, full context lengths; the
contexts are the keyed synthetic KV that das_kv_synth writes on the device).  The oracle then recomputes SAMPLED
sequences one by one from the same inputs (same bf16 weights widened to fp32, same synthetic KV, same drafts) and
their logits and decisions are compared under the usual protocol.  Sequences of a verify step are independent, so
a sampled sequence inside the full ragged batch must equal the oracle's stand-alone result.
"""
import numpy as np
import pytest

import das_inputs as di
import oracle
from parity_harness import StepReport, compare_greedy_step, compare_stochastic_step

pytestmark = pytest.mark.gpu


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


def _sample_ids(ctx, ks, limit_ctx):
    order = np.argsort(ctx, kind="stable")
    picks = [int(order[0]), int(order[len(order) // 2])]
    # the longest sequence whose oracle attention is still cheap, and the one with the largest budget
    ok = [int(i) for i in order if ctx[i] <= limit_ctx]
    picks.append(ok[-1])
    picks.append(int(max(ok, key=lambda i: (ks[i], ctx[i]))))
    return sorted(set(picks))


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_size_step_against_oracle_on_sampled_sequences(name, weights):
    import paper_2511_13841_amd as das
    wl = di.WORKLOADS[name]
    shape = di.MODELS[wl.model]
    blob, om = weights(wl.model)
    ctx = di.context_lengths(wl)
    ks = di.draft_budgets(wl, ctx)
    B = wl.batch
    kmax = int(ks.max())
    pages = int(sum(-(-(int(c) + kmax + 2) // 16) for c in ctx)) + 8
    T = int((ks + 1).sum())
    print(f"{name}: B={B} rows={T} kv_tokens={int(ctx.sum())} pages={pages}", flush=True)
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=-(-(int(ctx.max()) + kmax + 18) // 16) * 16, max_rows=max(T, 256),
                                     max_draft=max(kmax, 1), num_pages=pages), blob)
    rng = np.random.default_rng(wl.seed)
    pend = rng.integers(0, shape.vocab, size=B, dtype=np.int32)
    ids = list(range(B))
    for i in ids:
        dm.seq_create(i, int(ctx[i]), int(pend[i]))
        dm.kv_synth(i, wl.seed, i)
    drafts = [rng.integers(0, shape.vocab, size=int(k), dtype=np.int32) for k in ks]
    picks = _sample_ids(ctx, ks, limit_ctx=40000)
    seqs = {i: _oracle_seq(om, shape, wl.seed, i, int(ctx[i]), pend[i], kmax + 2) for i in picks}
    # make the first draft of every sampled sequence the oracle's own greedy token, so accepted prefixes occur
    for i in picks:
        if ks[i] > 0:
            drafts[i][0] = int(np.argmax(om.verify_logits(seqs[i], drafts[i][:0])[0]))
    row0 = np.concatenate([[0], np.cumsum(ks + 1)])
    sampling = None
    if wl.mode == "stochastic":
        keys = np.repeat(np.arange(B), ks + 1)
        pos = np.concatenate([np.arange(ctx[i], ctx[i] + ks[i] + 1) for i in ids])
        ua = di.uniforms(wl.seed, keys, pos, 0)
        us = di.uniforms(wl.seed, keys, pos, 1)
        ua = np.where(rng.random(ua.size) < 0.7, 0.0, ua).astype(np.float32)      # controlled mode: forced acceptances
        sampling = (wl.temperature, ua, us)
    print("verify step on the full batch", flush=True)
    acc, nx = dm.verify_step(ids, ctx, drafts, sampling)
    gg = dm.debug_row_argmax() if sampling is None else None
    if sampling is None:
        # that was the production path: row maxima gathered inside the LM-head GEMM, no logits in memory.  The same
        # step with the logits written out and scanned must take the same decisions, bit for bit.
        with pytest.raises(das.DasError):
            dm.debug_logits(0, 1)
        dm.kv_rollback(ids)
        dm.keep_logits(True)
        acc2, nx2 = dm.verify_step(ids, ctx, drafts, sampling)
        assert np.array_equal(gg, dm.debug_row_argmax()) and np.array_equal(acc, acc2) and np.array_equal(nx, nx2)
    rep = StepReport()
    exact = 0
    for i in picks:
        n = int(ks[i]) + 1
        glog = dm.debug_logits(int(row0[i]), n)
        print(f"  oracle for sequence {i}: ctx={int(ctx[i])} k={int(ks[i])}", flush=True)
        if sampling is None:
            a, t, lo = om.verify_greedy(seqs[i], drafts[i])
            compare_greedy_step(rep, glog, gg[row0[i]:row0[i] + n], acc[i], nx[i], lo, a, t, drafts[i])
        else:
            lo = om.verify_logits(seqs[i], drafts[i])
            sl = slice(int(row0[i]), int(row0[i]) + n)
            exact += bool(compare_stochastic_step(glog, acc[i], nx[i], lo, drafts[i], wl.temperature, ua[sl], us[sl]))
            rep.max_rel_logit_err = max(rep.max_rel_logit_err, float(np.abs(glog - lo).max() / np.abs(lo).max()))
    print(name, rep, "exact stochastic decisions:", exact)
    assert rep.max_rel_logit_err < 3e-2
    # properties of the whole batch: every decision follows from the row argmaxes / is in range
    for i in ids:
        assert 0 <= acc[i] <= ks[i] and 0 <= nx[i] < shape.vocab
        if sampling is None:
            g = gg[row0[i]:row0[i + 1]]
            a = 0
            while a < ks[i] and drafts[i][a] == g[a]:
                a += 1
            assert (int(acc[i]), int(nx[i])) == (a, int(g[a]))
    dm.kv_commit(ids, acc, nx)
    for i in picks:
        assert dm.debug_seq(i)["ctx_len"] == int(ctx[i]) + 1 + int(acc[i])
    dm.free()
    for s in seqs.values():
        s.close()
