"""Whole rollouts on the GPU: speculative decoding must emit the tokens of plain decoding (the losslessness
the paper claims in its abstract and Sec. 5.1) while the batch collapses, in fewer forward passes."""
import pytest

pytestmark = pytest.mark.gpu


def test_speculative_rollout_equals_plain_rollout_tiny():
    from paper_2511_13841_amd.rollout_makespan import run
    r = run(model="tiny", batch=12, max_len=48, accept_p=0.7, k_medium=2, k_long=4, ctx_lo=16, ctx_hi=64, seed=77)
    assert r["sequences_differing_from_plain_decoding"] == 0
    assert r["speculative"]["forwards"] < r["plain"]["forwards"]
    assert r["speculative"]["accepted_drafts"] > 0
    assert r["plain"]["tokens_processed"] == r["target_len"]["sum"]


def test_speculative_rollout_equals_plain_rollout_wide_model_few_layers():
    from paper_2511_13841_amd.rollout_makespan import run
    r = run(model="1.5b", batch=6, max_len=24, accept_p=0.8, k_medium=3, k_long=6, ctx_lo=200, ctx_hi=2300, seed=78, n_layers=2)
    assert r["sequences_differing_from_plain_decoding"] == 0
    assert r["speculative"]["forwards"] < r["plain"]["forwards"]


def test_rollout_with_solver_budgets_is_lossless_too():
    from paper_2511_13841_amd.rollout_makespan import run
    r = run(model="tiny", batch=12, max_len=48, accept_p=0.7, k_long=6, ctx_lo=16, ctx_hi=64, seed=79, policy="solver",
            c_base=1.0, c_tok=0.02, alpha=0.6, cap=0.9)
    assert r["sequences_differing_from_plain_decoding"] == 0
    assert r["speculative"]["forwards"] < r["plain"]["forwards"]
    assert r["budgets"]["sequences_without_speculation"] > 0        # short requests skip speculation (Sec. 4.2.1)


def test_rollout_with_the_suffix_tree_drafter_over_the_previous_epoch():
    from paper_2511_13841_amd.rollout_makespan import run
    r = run(model="tiny", batch=12, max_len=48, k_medium=3, k_long=6, ctx_lo=16, ctx_hi=64, seed=81, drafter="tree")
    assert r["sequences_differing_from_plain_decoding"] == 0
    # same policy in both epochs: once the match is unique the tree proposes the true continuation
    assert r["speculative"]["accepted_drafts"] > 0.5 * (r["speculative"]["tokens_processed"] - r["speculative"]["forwards"])
    assert r["speculative"]["forwards"] < 0.7 * r["plain"]["forwards"]


def test_rollouts_follow_the_oracles_greedy_decoding():
    """The tokens of a whole collapsing-batch rollout against the ORACLE (not only against the GPU's own plain pass):
    every sequence is replayed by the oracle from the same synthetic context, one token per forward; wherever the
    oracle's top-1/top-2 margin exceeds 0.1 the GPU's token must be the oracle's greedy token.  The oracle is kept on
    the GPU's trajectory (teacher forcing), so one near-tie cannot desynchronise the comparison."""
    import numpy as np
    import das_inputs as di
    import oracle
    from paper_2511_13841_amd.rollout_makespan import run
    r = run(model="tiny", batch=24, max_len=64, accept_p=0.7, k_medium=2, k_long=4, ctx_lo=16, ctx_hi=64, seed=83, keep_rollouts=True)
    assert r["sequences_differing_from_plain_decoding"] == 0
    ro = r["rollouts"]
    shape = di.MODELS["tiny"]
    om = oracle.OracleModel(shape, di.bf16_to_f32(di.weights_bf16(shape, seed=0)))
    clear = flagged = 0
    for i, (c, p0) in enumerate(zip(ro["ctx0"], ro["pend0"])):
        c = int(c)
        toks = ro["speculative"][i]
        assert toks[0] == p0 and np.array_equal(toks, ro["plain"][i])
        s = om.new_seq(c + len(toks) + 2)
        for layer in range(shape.n_layers):
            for which in (0, 1):
                s.kv(layer, which)[:c] = di.bf16_to_f32(di.kv_synth(ro["kv_seed"], i, layer, which, 0, c, shape.n_kv_heads, shape.head_dim))
        s.len, s.pending = c, int(p0)
        for t in toks[1:]:
            lo = om.forward(s, s.len, [s.pending])[0]
            top = np.partition(lo, -2)[-2:]
            if top[1] - top[0] > 0.1:
                assert int(np.argmax(lo)) == int(t), (i, s.len)
                clear += 1
            else:
                flagged += 1
            om.commit(s, 0, int(t), [])
        s.close()
    print(f"rollout tokens checked against the oracle: {clear} clear, {flagged} under the margin")
    # (random-init logits are nearly flat: about two thirds of the rows fall under the margin and are only counted)
    assert clear >= 60
