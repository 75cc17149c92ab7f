"""Real prefill at full depth against the oracle (Fig. 3: a rollout starts from its prompt; Sec. 3: the verification
rounds then run on the KV the prefill wrote).

The 28-layer 1.5B-class model of config 2 takes three prompts of about 40, 300 and 1100 tokens in ONE das_prefill
call: several passes, several blocks of a prompt per pass, the longest prompt crosses the 1024-token boundary of the
split-KV chunks.  Compared with the oracle's own prefill of the same prompts: last-row logits, the K/V the passes
wrote in the first, a middle and the last layer, the first pending token; then three verification rounds on those
real contexts with teacher-forced commits and the page bookkeeping checked every round.
"""
import numpy as np
import pytest

import das_inputs as di
import oracle
from conftest import progress
from parity_harness import StepReport, compare_greedy_step, check_bookkeeping, top2_margin, LOGIT_RTOL, MARGIN

pytestmark = pytest.mark.gpu


def test_prefill_at_full_depth_across_chunks_then_verify_rounds():
    import paper_2511_13841_amd as das
    wl = di.WORKLOADS["c2"]
    shape = di.MODELS[wl.model]
    blob = di.weights_bf16(shape, seed=0)
    om = oracle.OracleModel(shape, di.bf16_to_f32(blob))
    lens = [41, 300, 1100]
    k, rounds = 4, 3
    num_pages = 256
    dm = das.DasModel(das.config_for(shape, max_seqs=4, max_ctx=2048, max_rows=320, max_draft=8, num_pages=num_pages), blob,
                      keep_logits=True)
    mirror = oracle.PageTableMirror(num_pages)
    prompts = di.prompts(lens, shape.vocab, 77)
    ids = [3, 8, 5]
    progress("prefill", lens)
    nxt = dm.prefill(ids, prompts)
    mirror.prefill(ids, lens)
    glog = dm.debug_logits()      # logits of the LAST pass: the row that ends the longest prompt (the others ended in earlier passes)
    assert glog.shape[0] == 1
    seqs, pend = [], []
    for i, p in enumerate(prompts):
        progress("oracle prefill of", len(p), "tokens")
        s = om.new_seq(len(p) + rounds * (k + 1) + 8)
        lo = om.prefill(s, p)
        if i == 2:
            err = float(np.abs(glog[0] - lo).max())
            progress(f"  last-row logit error {err / np.abs(lo).max():.3e} of max|logit|")
            assert err <= LOGIT_RTOL * float(np.abs(lo).max()), (i, err)
        s.pending = int(np.argmax(lo))
        if top2_margin(lo[None, :])[0] > MARGIN:
            assert int(nxt[i]) == s.pending
        for layer in (0, shape.n_layers // 2 - 1, shape.n_layers - 1):
            kg, vg = dm.kv_export(ids[i], layer, 0, len(p))
            ko, vo = s.kv(layer, 0)[: len(p)], s.kv(layer, 1)[: len(p)]
            assert np.abs(di.bf16_to_f32(kg) - ko).max() <= 3e-2 * np.abs(ko).max(), (i, layer)
            assert np.abs(di.bf16_to_f32(vg) - vo).max() <= 3e-2 * np.abs(vo).max(), (i, layer)
        seqs.append(s)
        pend.append(s.pending)
    assert dm.debug_kv_saturated() == 0
    # teacher forcing of the first pending token: same length, the oracle's token
    dm.seq_rewind(ids, lens, pend)
    check_bookkeeping(dm, mirror, ids, pend)
    # the oracle's own greedy continuation feeds the synthetic drafter; then its sequences are put back
    future = []
    for s, n in zip(seqs, lens):
        p0, toks0 = s.pending, list(s.tokens)
        future.append([p0] + om.ar_greedy(s, rounds * (k + 1) + 2))
        s.len, s.pending, s.tokens = n, p0, toks0
    rng = np.random.default_rng(5)
    emitted = [1] * 3
    rep = StepReport()
    for rnd in range(rounds):
        ctx = [s.len for s in seqs]
        drafts = [di.make_drafts(future[i][emitted[i]:emitted[i] + k], k, wl.accept_p, shape.vocab, rng) for i in range(3)]
        progress("verify round", rnd, ctx)
        acc, nx = dm.verify_step(ids, ctx, drafts)
        mirror.verify(ids, [k] * 3)
        glog, gg = dm.debug_logits(), dm.debug_row_argmax()
        o_acc, o_nx = [], []
        for i, s in enumerate(seqs):
            a, t, lo = om.verify_greedy(s, drafts[i])
            sl = slice((k + 1) * i, (k + 1) * (i + 1))
            compare_greedy_step(rep, glog[sl], gg[sl], acc[i], nx[i], lo, a, t, drafts[i])
            om.commit(s, a, t, drafts[i])
            emitted[i] += a + 1
            o_acc.append(a); o_nx.append(t)
        dm.kv_commit(ids, o_acc, o_nx)
        mirror.commit(ids, o_acc)
        check_bookkeeping(dm, mirror, ids, o_nx)
        rep.steps += 1
    progress(rep)
    assert rep.decisions == 3 * rounds and sum(emitted) > 3 * (rounds + 1)      # some drafts were accepted
    dm.seq_free(ids)
    mirror.release(ids)
    assert dm.debug_free_pages() == num_pages
    dm.free()
    for s in seqs:
        s.close()
    om.close()


def test_prefill_pass_takes_several_blocks_of_one_prompt():
    """A prompt longer than the 256-query-row limit of one attention work item enters a pass as several blocks:
    the result must not depend on how the prompt was cut (one pass of 300 rows against passes of 64 rows), bit for bit."""
    import paper_2511_13841_amd as das
    shape = di.MODELS["tiny"]
    blob = di.weights_bf16(shape, seed=0)
    prompts = di.prompts([300, 17, 130], shape.vocab, 3)
    res = []
    for max_rows in (512, 64):
        dm = das.DasModel(das.config_for(shape, max_seqs=4, max_ctx=512, max_rows=max_rows, max_draft=4, num_pages=64), blob, keep_logits=True)
        nxt = dm.prefill([0, 1, 2], prompts)
        kv = [dm.kv_export(i, layer, 0, len(p)) for i, p in enumerate(prompts) for layer in range(shape.n_layers)]
        acc, nx = dm.verify_step([0, 1, 2], [len(p) for p in prompts], [[1, 2], [3], []])
        res.append((nxt, kv, acc, nx, dm.debug_logits()))
        dm.free()
    a, b = res
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])
    for (k1, v1), (k2, v2) in zip(a[1], b[1]):
        assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert np.array_equal(a[4], b[4])
