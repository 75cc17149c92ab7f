"""Properties that hold at any size, checked on the GPU path alone or against the integer mirror:
losslessness of the GPU's own speculative rounds, rollback, multi-pass prefill, error behaviour."""
import numpy as np
import pytest

import das_inputs as di

pytestmark = pytest.mark.gpu

NARROW_7B = di.ModelShape("narrow7b", 2, 256, 28, 4, 128, 512, 4096, rope_theta=1.0e6)


def _model(shape, B, max_ctx, pages, max_rows=512, max_draft=16):
    import paper_2511_13841_amd as das
    blob = di.weights_bf16(shape, seed=0)
    return das, das.DasModel(das.config_for(shape, max_seqs=B, max_ctx=max_ctx, max_rows=max_rows, max_draft=max_draft,
                                            num_pages=pages), blob, keep_logits=True)


@pytest.mark.parametrize("shape,ctxs", [(di.MODELS["tiny"], [17, 40, 64, 33]), (NARROW_7B, [100, 1020, 2040, 5000]),
                                        (di.MODELS["tiny"], [1000, 1020, 2040, 90])],
                         ids=["tiny", "7b-heads", "tiny-chunk-boundaries"])
def test_gpu_speculative_rounds_equal_gpu_plain_decoding(shape, ctxs):
    """The emitted stream of speculative rounds (ragged budgets, a changing batch) is bit-identical to
    one-token-at-a-time decoding on the same engine: every row's result is independent of the batch
    it is verified in (fixed reduction orders in the GEMMs, position-aligned split-KV chunks)."""
    B, N = len(ctxs), 120
    # with 7 query heads per KV head, budgets above 17 need the attention kernel's second shape (up to 16 row blocks)
    budgets = [0, 1, 2, 4, 8, 16] + ([24, 32] if shape is NARROW_7B else [])
    das, dm = _model(shape, B, max(ctxs) + 256, sum(-(-(c + 256) // 16) for c in ctxs) + 4, max_draft=max(budgets))
    ids = list(range(B))
    rng = np.random.default_rng(3)
    pend0 = rng.integers(0, shape.vocab, size=B, dtype=np.int32)
    for i in ids:
        dm.seq_create(i, ctxs[i], int(pend0[i]))
        dm.kv_synth(i, 11, i)
    ctx0 = np.array(ctxs, np.int32)
    fut = np.empty((B, N + 1), np.int32)
    fut[:, 0] = pend0
    for t in range(N):
        acc, nxt = dm.verify_step(ids, ctx0 + t, [[] for _ in ids])
        dm.kv_commit(ids, acc, nxt)
        fut[:, t + 1] = nxt
    dm.seq_rewind(ids, ctx0, pend0)
    emitted = np.ones(B, np.int64)
    ctx = ctx0.copy()
    rounds = 0
    total_acc = 0
    while rounds < 12:
        # a changing sub-batch with ragged budgets
        active = [i for i in ids if rng.random() < 0.8] or [0]
        ks = [int(rng.choice(budgets)) for _ in active]
        drafts = []
        for i, k in zip(active, ks):
            d = fut[i, emitted[i]:emitted[i] + k].copy()
            bad = rng.random(k) >= 0.8
            d[bad] = rng.integers(0, shape.vocab, size=int(bad.sum()))
            drafts.append(d)
        print("round", rounds, active, ks, flush=True)
        acc, nxt = dm.verify_step(active, ctx[active], drafts)
        dm.kv_commit(active, acc, nxt)
        for j, i in enumerate(active):
            a = int(acc[j])
            want = fut[i, emitted[i]:emitted[i] + a + 1]
            got = list(drafts[j][:a]) + [int(nxt[j])]
            assert list(want) == got, (rounds, i, a, list(want), got)
            emitted[i] += a + 1
            ctx[i] += a + 1
            total_acc += a
        rounds += 1
    assert total_acc > 0
    dm.free()


# a long FFN: the down projection sums K in slices and, in passes of up to 512 rows, its slice-summing kernel also applies
# the next RMSNorm
LONG_FFN = di.ModelShape("longffn", 2, 256, 4, 2, 64, 8448, 2048, rope_theta=1.0e4)


# a model dimension of 1024: QKV, O and down all sum K in two slices -- over workgroups in passes of up to 512 rows (the QKV
# partials are then added by the rotation kernel), folded in registers above
WIDE_D = di.ModelShape("wided", 2, 1024, 8, 2, 128, 1024, 2048, rope_theta=1.0e4)


@pytest.mark.parametrize("shape", [di.MODELS["tiny"], NARROW_7B, LONG_FFN, WIDE_D], ids=["tiny", "7b-heads", "long-ffn", "wide-d"])
def test_logit_rows_do_not_depend_on_the_size_of_the_pass(shape):
    """The logits of a sequence's rows are the same bits whether it is verified alone (16 rows), in a batch of 13
    (208 rows), of 40 (640 rows) or of 70 (1120 rows): every launch-shape threshold of the row-wise kernels and of the
    GEMMs (64, 256, 512, 1024 rows) lies between those sizes, and none of them may change a reduction order."""
    B, k = 70, 15
    rng = np.random.default_rng(11)
    ctxs = rng.integers(20, 400, size=B)
    ctxs[:3] = [1030, 2050, 100]                                   # the sequences compared; two cross a chunk boundary
    das, dm = _model(shape, B, int(ctxs.max()) + 64, int(sum(-(-(int(c) + 32) // 16) for c in ctxs)) + 4,
                     max_rows=B * (k + 1), max_draft=k)
    ids = list(range(B))
    pend = rng.integers(0, shape.vocab, size=B, dtype=np.int32)
    for i in ids:
        dm.seq_create(i, int(ctxs[i]), int(pend[i]))
        dm.kv_synth(i, 5, i)
    drafts = [rng.integers(0, shape.vocab, size=k, dtype=np.int32) for _ in ids]
    ref = {}
    for nb in (B, 40, 13, 1):
        sub = ids[:nb] if nb > 3 else ids[:3][:nb]
        print("pass of", nb, "sequences", flush=True)
        passes = [sub] if nb > 1 else [[0], [1], [2]]               # alone: one pass per compared sequence
        for p in passes:
            dm.verify_step(p, ctxs[p], [drafts[i] for i in p])
            for j, i in enumerate(p):
                if i < 3:
                    got = dm.debug_logits(j * (k + 1), k + 1)
                    if i in ref:
                        assert np.array_equal(got, ref[i]), (nb, i, float(np.abs(got - ref[i]).max()))
                    else:
                        ref[i] = got
            dm.kv_rollback(p)
    dm.free()


@pytest.mark.parametrize("shape,ctx", [(di.MODELS["tiny"], 1000), (NARROW_7B, 2030)], ids=["tiny", "7b-heads"])
def test_rows_of_a_one_chunk_sequence_equal_the_same_rows_merged(shape, ctx):
    """A sequence whose keys fit one attention chunk is finished by the attention kernel; with more draft rows it spills
    into a second chunk and goes through the merge.  The rows both passes share must carry the same logit bits."""
    k_short, k_long = 8, 30
    das, dm = _model(shape, 1, ctx + 64, (ctx + 64) // 16 + 4, max_rows=k_long + 1, max_draft=k_long)
    rng = np.random.default_rng(5)
    dm.seq_create(0, ctx, 7)
    dm.kv_synth(0, 3, 0)
    drafts = rng.integers(0, shape.vocab, size=k_long, dtype=np.int32)
    dm.verify_step([0], [ctx], [drafts[:k_short]])                 # ctx + 9 keys: one chunk
    short = dm.debug_logits(0, k_short + 1)
    dm.kv_rollback([0])
    dm.verify_step([0], [ctx], [drafts])                           # ctx + 31 keys: past the chunk boundary
    long = dm.debug_logits(0, k_short + 1)
    dm.kv_rollback([0])
    assert np.array_equal(short, long), float(np.abs(short - long).max())
    dm.free()


def test_rollback_reverify_and_fresh_prefill_equivalence():
    shape = di.MODELS["tiny"]
    das, dm = _model(shape, 4, 512, 64)
    prompts = di.prompts([50, 31], shape.vocab, 4)
    nxt = dm.prefill([1, 2], prompts)
    free0 = dm.debug_free_pages()
    drafts = [np.array([5, 6, 7, 8, 9, 10, 11, 12], np.int32), np.array([1], np.int32)]
    a1, n1 = dm.verify_step([1, 2], [50, 31], drafts)
    l1 = dm.debug_logits()
    assert dm.debug_seq(1)["state"] == 1
    dm.kv_rollback([1, 2])
    assert dm.debug_free_pages() == free0 and dm.debug_seq(1)["ctx_len"] == 50 and dm.debug_seq(1)["pending"] == nxt[0]
    a2, n2 = dm.verify_step([1, 2], [50, 31], drafts)
    np.testing.assert_array_equal(dm.debug_logits(), l1)            # bit-identical after a rollback
    assert list(a1) == list(a2) and list(n1) == list(n2)
    dm.kv_commit([1, 2], [3, 0], [77, 78])                          # a caller-chosen decision (teacher forcing)
    st = dm.debug_seq(1)
    assert st["ctx_len"] == 54 and st["pending"] == 77 and len(st["pages"]) == 4
    # state after commit == a fresh sequence prefilled with the same tokens
    toks = np.concatenate([prompts[0], [nxt[0]], drafts[0][:3]]).astype(np.int32)
    dm.prefill([9], [toks])
    fresh_row = dm.debug_logits()[0]
    dm.verify_step([1], [54], [[]])
    dm.kv_rollback([1])
    # the committed sequence scores its pending token 77 next; compare against fresh + same pending
    dm.seq_rewind([9], [54], [77])
    dm.verify_step([9], [54], [[]])
    a = dm.debug_logits()[0]
    dm.kv_rollback([9])
    dm.verify_step([1], [54], [[]])
    b = dm.debug_logits()[0]
    np.testing.assert_allclose(a, b, atol=2e-2 * np.abs(b).max())
    # last prompt row of the fresh prefill == row 3 of the original verify pass (same tokens, same positions)
    np.testing.assert_allclose(fresh_row, l1[3], atol=2e-2 * np.abs(fresh_row).max())
    dm.free()


def test_multi_pass_prefill_equals_single_pass():
    shape = di.MODELS["tiny"]
    prompts = di.prompts([300, 45, 129, 7], shape.vocab, 8)
    das, big = _model(shape, 4, 512, 64, max_rows=512)
    das, small = _model(shape, 4, 512, 64, max_rows=48)
    n_big = big.prefill([1, 2, 3, 4], prompts)
    n_small = small.prefill([1, 2, 3, 4], prompts)
    assert list(n_big) == list(n_small)
    for sid, p in zip([1, 2, 3, 4], prompts):
        for layer in range(shape.n_layers):
            kb, vb = big.kv_export(sid, layer, 0, len(p))
            ks, vs = small.kv_export(sid, layer, 0, len(p))
            np.testing.assert_array_equal(kb, ks)
            np.testing.assert_array_equal(vb, vs)
    big.free(); small.free()


def test_error_paths_leave_state_untouched():
    shape = di.MODELS["tiny"]
    das, dm = _model(shape, 2, 128, 6, max_rows=64, max_draft=8)       # 6 pages = 96 tokens
    E = das.DasError
    prompts = di.prompts([40, 30], shape.vocab, 1)
    dm.prefill([1, 2], prompts)                                        # 3 + 2 pages
    before = (dm.debug_seq(1), dm.debug_seq(2), dm.debug_free_pages())

    def code(fn, *a, **k):
        try:
            fn(*a, **k)
        except E as e:
            return e.code
        return 0
    acc0, nxt0 = dm.verify_step([], [], [])                                        # an empty batch is a no-op
    assert len(acc0) == 0 and len(nxt0) == 0 and code(dm.kv_commit, [], [], []) == 0 and code(dm.kv_rollback, []) == 0
    assert code(dm.prefill, [3], [prompts[0]]) == das.DAS_ERR_NOMEM               # no slot
    assert code(dm.verify_step, [1, 2], [40, 31], [[1], [2]]) == das.DAS_ERR_STATE  # ctx mismatch
    assert code(dm.verify_step, [1, 1], [40, 40], [[1], [2]]) == das.DAS_ERR_INVALID
    assert code(dm.verify_step, [1, 7], [40, 30], [[1], [2]]) == das.DAS_ERR_INVALID
    assert code(dm.verify_step, [1], [40], [[shape.vocab]]) == das.DAS_ERR_INVALID
    assert code(dm.verify_step, [1], [40], [list(range(9))]) == das.DAS_ERR_INVALID  # k > max_draft
    assert code(dm.verify_step, [1, 2], [40, 30], [[1] * 8, [2] * 8]) == das.DAS_ERR_NOMEM  # needs 2 pages, 1 free
    assert code(dm.kv_commit, [1], [0], [5]) == das.DAS_ERR_STATE                  # nothing pending
    assert code(dm.kv_rollback, [1]) == das.DAS_ERR_STATE
    assert (dm.debug_seq(1), dm.debug_seq(2), dm.debug_free_pages()) == before
    dm.verify_step([1], [40], [[1, 2, 3]])
    assert code(dm.verify_step, [1], [40], [[1]]) == das.DAS_ERR_STATE             # second verify without commit
    assert code(dm.kv_commit, [1], [4], [5]) == das.DAS_ERR_INVALID                # accept_len > k
    assert code(dm.kv_commit, [1], [-1], [5]) == das.DAS_ERR_INVALID
    assert code(dm.kv_commit, [1], [1], [shape.vocab]) == das.DAS_ERR_INVALID
    assert dm.debug_seq(1)["state"] == 1
    dm.kv_commit([1], [3], [5])
    assert dm.debug_seq(1)["ctx_len"] == 44 and dm.debug_seq(1)["state"] == 0
    dm.seq_free([1, 2])
    assert dm.debug_free_pages() == 6
    dm.free()
