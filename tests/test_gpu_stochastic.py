"""Stochastic verification (rejection sampling with seeded uniforms) on the GPU against the oracle."""
import numpy as np
import pytest

import das_inputs as di
import oracle
from oracle import softmax_weights

pytestmark = pytest.mark.gpu


def _check_sampled_token(w, u, v, eps):
    """v must satisfy u*Z in [prefix(v-1) - eps*Z, prefix(v) + eps*Z] under the oracle's weights."""
    cs = np.cumsum(w)
    Z = cs[-1]
    lo = cs[v - 1] if v > 0 else 0.0
    assert w[v] > 0.0, "sampled a zero-weight token"
    assert lo - eps * Z <= u * Z <= cs[v] + eps * Z, (v, u * Z, lo, cs[v], eps * Z)


@pytest.mark.parametrize("mode,tau", [("faithful", 1.0), ("controlled", 1.0), ("controlled", 0.6)])
def test_rejection_sampling_decisions_match_oracle(mode, tau):
    import paper_2511_13841_amd as das
    shape = di.MODELS["tiny"]
    blob = di.weights_bf16(shape, seed=0, sigma=0.06)          # sharper logits than config 1: p_max ~ 0.05
    om = oracle.OracleModel(shape, di.bf16_to_f32(blob))
    dm = das.DasModel(das.config_for(shape, max_seqs=8, max_ctx=1024, max_rows=256, max_draft=8, num_pages=256), blob, keep_logits=True)
    lens = [20, 33, 47, 64, 16]
    ids = list(range(5))
    prompts = di.prompts(lens, shape.vocab, 55)
    us0 = di.uniforms(9, ids, [l - 1 for l in lens], 1)
    nxt = dm.prefill(ids, prompts, sampling=(tau, None, us0))
    seqs = []
    for i, p in enumerate(prompts):
        s = om.new_seq(400)
        lo = om.prefill(s, p)
        w, _ = softmax_weights(lo, tau)
        _check_sampled_token(w, float(us0[i]), int(nxt[i]), 0.02)
        s.pending = int(nxt[i])
        seqs.append(s)
    rng = np.random.default_rng(7)
    flagged = exact = 0
    for rnd in range(10):
        ks = [int(k) for k in rng.integers(0, 7, size=5)]
        drafts, ua, us = [], [], []
        for i, s in enumerate(seqs):
            # likely drafts: the target's own argmax chain with noise
            d = rng.integers(0, shape.vocab, size=ks[i], dtype=np.int32)
            for j in range(ks[i]):
                if rng.random() < 0.7:
                    d[j] = int(np.argmax(om.verify_logits(s, d[:j])[j]))
            drafts.append(d)
            pos = np.arange(s.len, s.len + ks[i] + 1)
            a_u = di.uniforms(9, [ids[i]] * len(pos), pos, 0)
            if mode == "controlled":
                a_u = np.where(rng.random(len(pos)) < 0.7, 0.0, a_u).astype(np.float32)   # u = 0 forces acceptance
            ua.append(a_u)
            us.append(di.uniforms(9, [ids[i]] * len(pos), pos, 1))
        print("round", rnd, ks, flush=True)
        acc, nx = dm.verify_step(ids, [s.len for s in seqs], drafts, sampling=(tau, np.concatenate(ua), np.concatenate(us)))
        glog = dm.debug_logits()
        r0, o_acc, o_nx = 0, [], []
        for i, s in enumerate(seqs):
            n = ks[i] + 1
            a, t, lo = om.verify_stochastic(s, drafts[i], tau, ua[i], us[i])
            err = np.abs(glog[r0:r0 + n] - lo).max()
            assert err <= 3e-2 * np.abs(lo).max()
            delta = float(err) / tau
            # a decision is flagged when a uniform lies within e^{+-0.1} of the accept probability on the way
            flag = False
            for j in range(min(a + 1, ks[i])):
                w, Z = softmax_weights(lo[j], tau)
                pd = w[drafts[i][j]] / Z
                if pd * np.exp(-0.1) <= ua[i][j] <= pd * np.exp(0.1):
                    flag = True
            if flag:
                flagged += 1
            else:
                exact += 1
                assert int(acc[i]) == a, (rnd, i, int(acc[i]), a)
                w, _ = softmax_weights(lo[a], tau)
                if a < ks[i]:
                    w = w.copy(); w[drafts[i][a]] = 0.0
                    assert int(nx[i]) != int(drafts[i][a])
                _check_sampled_token(w, float(us[i][a]), int(nx[i]), np.exp(2 * delta) - 1 + 1e-6)
            om.commit(s, a, t, drafts[i])
            o_acc.append(a); o_nx.append(t)
            r0 += n
        dm.kv_commit(ids, o_acc, o_nx)
    print("exact", exact, "flagged", flagged)
    assert exact > 30
    if mode == "controlled":
        assert sum(s.len for s in seqs) - sum(lens) > 60      # forced acceptances really advance the sequences
    dm.free()


def test_first_emitted_token_distribution_chi_square_on_gpu():
    """Vocabulary 32, 64 copies of one state, fresh uniforms every call: the first emitted token of the
    speculative round follows softmax(logits/T) of the target (the rule is distribution-preserving)."""
    from scipy.stats import chi2
    import paper_2511_13841_amd as das
    shape = di.ModelShape("v32", 1, 64, 2, 1, 64, 64, 32, rope_theta=1.0e4)
    blob = di.weights_bf16(shape, seed=3, sigma=0.3)
    om = oracle.OracleModel(shape, di.bf16_to_f32(blob))
    B, tau = 64, 0.8
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=64, max_rows=B * 3, max_draft=2, num_pages=B * 2), blob)
    prompt = di.prompts([9], shape.vocab, 2)[0]
    ids = list(range(B))
    dm.prefill(ids, [prompt] * B)
    dm.seq_rewind(ids, [9] * B, [5] * B)            # same pending token everywhere
    s = om.new_seq(32)
    om.prefill(s, prompt)
    s.pending = 5
    lo = om.verify_logits(s, [])[0]
    w, Z = softmax_weights(lo, tau)
    p = w / Z
    d1 = int(np.argmax(p))
    rng = np.random.default_rng(1234)
    hist = np.zeros(shape.vocab)
    n_acc = 0
    rounds = 150
    for r in range(rounds):
        ua, us = rng.random(3 * B).astype(np.float32), rng.random(3 * B).astype(np.float32)
        acc, nx = dm.verify_step(ids, [9] * B, [[d1, 7]] * B, sampling=(tau, ua, us))
        dm.kv_rollback(ids)
        for i in range(B):
            hist[d1 if acc[i] >= 1 else nx[i]] += 1
            n_acc += int(acc[i] >= 1)
    n = rounds * B
    stat = float(((hist - n * p) ** 2 / (n * p)).sum())
    print("chi2", stat, "accept rate", n_acc / n, "p(d1)", p[d1])
    assert chi2.sf(stat, shape.vocab - 1) > 1e-3, stat
    assert abs(n_acc / n - p[d1]) < 4 * np.sqrt(p[d1] * (1 - p[d1]) / n) + 0.01
    dm.free()


@pytest.mark.parametrize("V", [30, 1000, 270001, 300004])
def test_inverse_cdf_walk_against_fp64_prefix_sums_of_the_gpu_logits(V):
    """The sampler alone: its token against fp64 prefix sums over the weights of the logits the GPU itself wrote, so the
    window is the fp32 summation error and not the GEMM's.  Vocabularies off the 16-byte load path (not a multiple of 4),
    below one block of 256 columns, and above 262144 (several blocks per recorded total); uniforms from 0 to just
    below 1; both the residual draw after a rejection (the rejected token must never come back) and the draw after
    the last accepted draft."""
    import paper_2511_13841_amd as das
    shape = di.ModelShape(f"v{V}", 1, 64, 2, 1, 64, 64, V, rope_theta=1.0e4)
    blob = di.weights_bf16(shape, seed=3, sigma=0.3)
    B, tau = 48, 0.8
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=64, max_rows=B * 2, max_draft=1, num_pages=B * 2), blob,
                      keep_logits=True)
    prompt = di.prompts([9], shape.vocab, 2)[0]
    ids = list(range(B))
    dm.prefill(ids, [prompt] * B)
    dm.seq_rewind(ids, [9] * B, [5] * B)
    dm.verify_step(ids, [9] * B, [[] for _ in ids])
    d1 = int(np.argmax(dm.debug_logits()[0]))                      # a draft with visible weight
    dm.kv_rollback(ids)
    u_spread = np.linspace(0.0, 1.0, B, endpoint=False, dtype=np.float64)
    u_spread[-1] = 1.0 - 2.0 ** -24
    for accept in (False, True):
        ua = np.full(2 * B, 0.0 if accept else 1.0 - 2.0 ** -24, np.float32)
        us = np.repeat(u_spread, 2).astype(np.float32)
        print("V", V, "accept", accept, flush=True)
        acc, nx = dm.verify_step(ids, [9] * B, [[d1]] * B, sampling=(tau, ua, us))
        glog = dm.debug_logits()
        dm.kv_rollback(ids)
        for i in range(B):
            assert int(acc[i]) == int(accept)
            row = 2 * i + int(acc[i])
            l = glog[row].astype(np.float64)
            w = np.exp((l - l.max()) / tau)
            if not accept:
                w[d1] = 0.0
                assert int(nx[i]) != d1
            _check_sampled_token(w, float(us[row]), int(nx[i]), 1e-4)
    dm.free()


@pytest.mark.parametrize("B", [80, 70, 3, 12, 20, 30, 41, 60])      # 640 and 560 rows: LM-head tiles of 7 and of 6 row blocks; 24 .. 480 rows: the few-row tiles
def test_sampling_pass_without_logits_equals_the_pass_that_writes_them(B):
    """A sampling pass never writes its logits: the LM-head GEMM leaves per-block softmax statistics and
    the draft tokens' logits, and the drawing kernel computes the one block it needs again.  The same step in inspection
    mode (logits written, statistics taken from them) must take the same decisions bit for bit; and those decisions are
    right by fp64 arithmetic on the written logits (accept tests outside a 1e-5 band, tokens inside a 1e-4 window)."""
    import paper_2511_13841_amd as das
    V = 20011                                                       # not a multiple of 32: a ragged last block
    shape = di.ModelShape("v20k", 1, 256, 4, 2, 64, 512, V, rope_theta=1.0e4)
    blob = di.weights_bf16(shape, seed=5, sigma=0.25)
    k, tau = 7, 0.7
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=128, max_rows=B * (k + 1), max_draft=k, num_pages=B * 4), blob)
    rng = np.random.default_rng(3)
    lens = rng.integers(5, 40, size=B)
    ids = list(range(B))
    dm.prefill(ids, di.prompts(lens, V, 9))
    # likely drafts: the greedy chain of a plain pass for the first draft, random after it
    acc, g1 = dm.verify_step(ids, lens, [[] for _ in ids])
    dm.kv_rollback(ids)
    drafts = [np.concatenate([[g1[i]], rng.integers(0, V, size=k - 1)]).astype(np.int32) for i in ids]
    T = B * (k + 1)
    for rnd in range(3):
        ua = rng.random(T).astype(np.float32)
        ua = np.where(rng.random(T) < 0.5, 0.0, ua).astype(np.float32)          # half of the tests forced to accept
        us = rng.random(T).astype(np.float32)
        us[:8] = [0.0, 1.0 - 2.0 ** -24, 0.5, 0.25, 0.75, 0.999, 0.001, 0.9]
        acc1, nx1 = dm.verify_step(ids, lens, drafts, sampling=(tau, ua, us))
        with pytest.raises(das.DasError):
            dm.debug_logits(0, 1)                                    # nothing was written
        dm.kv_rollback(ids)
        dm.keep_logits(True)
        acc2, nx2 = dm.verify_step(ids, lens, drafts, sampling=(tau, ua, us))
        glog = dm.debug_logits()
        dm.kv_rollback(ids)
        dm.keep_logits(False)
        assert np.array_equal(acc1, acc2) and np.array_equal(nx1, nx2)
        n_rej = 0
        for i in ids:
            r0 = i * (k + 1)
            a = 0
            for j in range(k):
                l = glog[r0 + j].astype(np.float64) / tau
                p = np.exp(l - l.max()); p /= p.sum()
                pd = p[drafts[i][j]]
                if abs(ua[r0 + j] - pd) < 1e-5 * max(pd, 1e-30) + 1e-12:
                    a = int(acc1[i]); break                          # on the edge: either decision is right
                if not ua[r0 + j] < pd:
                    break
                a += 1
            assert int(acc1[i]) == a, (rnd, i, int(acc1[i]), a)
            l = glog[r0 + a].astype(np.float64) / tau
            w = np.exp(l - l.max())
            if a < k:
                w[drafts[i][a]] = 0.0
                assert int(nx1[i]) != int(drafts[i][a])
                n_rej += 1
            _check_sampled_token(w, float(us[r0 + a]), int(nx1[i]), 1e-4)
        assert n_rej > min(10, B // 4)
    dm.free()


def test_sampled_prefill_of_a_large_vocabulary_without_logits():
    """The first token after a prompt, drawn at a temperature: the pass that leaves only block statistics and the pass that
    writes its logits draw the same tokens, and the tokens are right by fp64 prefix sums of the written logits."""
    import paper_2511_13841_amd as das
    V = 20011
    shape = di.ModelShape("v20k", 1, 256, 4, 2, 64, 512, V, rope_theta=1.0e4)
    blob = di.weights_bf16(shape, seed=5, sigma=0.25)
    B, tau = 9, 0.8
    # (one pass takes all prompts, so that the written logits of the last pass are those of all of them, in order)
    dm = das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=128, max_rows=1024, max_draft=4, num_pages=B * 8), blob)
    rng = np.random.default_rng(11)
    lens = rng.integers(3, 90, size=B)
    ids = list(range(B))
    prompts = di.prompts(lens, V, 13)
    us = rng.random(B).astype(np.float32)
    us[:3] = [0.0, 1.0 - 2.0 ** -24, 0.5]
    nx1 = dm.prefill(ids, prompts, sampling=(tau, None, us))
    with pytest.raises(das.DasError):
        dm.debug_logits(0, 1)                                        # nothing was written
    dm.seq_free(ids)
    dm.keep_logits(True)
    nx2 = dm.prefill(ids, prompts, sampling=(tau, None, us))
    glog = dm.debug_logits()
    assert np.array_equal(nx1, nx2)
    for i in ids:
        l = glog[i].astype(np.float64) / tau
        _check_sampled_token(np.exp(l - l.max()), float(us[i]), int(nx1[i]), 1e-4)
    dm.free()
