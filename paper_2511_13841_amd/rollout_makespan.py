"""Makespan of a whole rollout batch with and without speculation (Sec. 1, Fig. 1; Sec. 5.1).

    python -m paper_2511_13841_amd.rollout_makespan [--model 7b] [--batch 64] [--max-len 512] [--accept-p 0.7]

The quantity the paper reports is the time until the LAST sequence of a rollout batch has finished: lengths
are long-tailed, the effective batch collapses, and the few long sequences set the makespan.  This tool plays
that out on synthetic lengths:
  1. plain decoding (one token per sequence per forward) until every sequence has reached its target length;
     sequences leave the batch as they finish.  The emitted tokens are recorded;
  2. all sequences are rewound and decoded again with speculative verification: the drafter proposes the
     recorded continuation with every position independently replaced by a random token with probability
     1 - p (the stand-in for a suffix-tree match of acceptance p), with a length-aware budget per sequence:
     none for sequences in the short class, a medium chain for the middle class, a long chain for the long
     class (Sec. 4.2.2, length-class policy; classes by target length here, i.e. a perfect length predictor).
The second pass must emit exactly the tokens of the first (the method is lossless); the tool counts mismatches.
Target lengths are a seeded Pareto tail clipped at --max-len.  One JSON object is printed.
"""
import argparse
import json
import time

import numpy as np

import das_inputs as di
from . import binding as das
from .rollout import log


def target_lengths(n, max_len, seed):
    """Long-tailed generation lengths: min_len * Pareto(alpha = 1.2), clipped to max_len."""
    rng = np.random.default_rng(seed)
    lo = max(4, max_len // 16)
    ln = lo * (1.0 - rng.random(n)) ** (-1.0 / 1.2)
    return np.minimum(ln, max_len).astype(np.int64)


def class_budgets(lens, k_medium, k_long):
    """Length-class policy: shortest third 0, middle third k_medium, longest third k_long."""
    order = np.argsort(lens, kind="stable")
    rank = np.empty_like(order)
    rank[order] = np.arange(lens.size)
    third = (rank * 3) // lens.size
    return np.array([0, k_medium, k_long], np.int64)[third]


def decode_plain(dm, ids, ctx0, pend0, lens):
    """One token per sequence per forward until each has emitted lens[i] tokens (the pending token is the first)."""
    B = len(ids)
    traj = [np.empty(int(lens[i]) + 1, np.int32) for i in range(B)]
    for i in range(B):
        traj[i][0] = pend0[i]
    done = np.zeros(B, np.int64)           # tokens emitted after the pending one
    rounds, n_toks, active_hist = 0, 0, []
    t0 = time.perf_counter()
    while True:
        act = [i for i in range(B) if done[i] < lens[i]]
        if not act:
            break
        acc, nxt = dm.verify_step([ids[i] for i in act], [ctx0[i] + done[i] for i in act], [[] for _ in act])
        dm.kv_commit([ids[i] for i in act], acc, nxt)
        for j, i in enumerate(act):
            done[i] += 1
            traj[i][done[i]] = nxt[j]
        rounds += 1
        n_toks += len(act)
        active_hist.append(len(act))
    return traj, time.perf_counter() - t0, rounds, n_toks, active_hist


def decode_speculative(dm, ids, ctx0, lens, traj, budgets, p, vocab, seed, tree=None):
    B = len(ids)
    rng = np.random.default_rng(seed)
    # synthetic drafter's view of every sequence: its true continuation, each position kept with probability p
    prop = []
    for i in range(B):
        t = traj[i].copy()
        bad = rng.random(t.size) >= p
        t[bad] = rng.integers(0, vocab, size=int(bad.sum()), dtype=np.int32)
        prop.append(t)
    done = np.zeros(B, np.int64)
    out = [np.empty(int(lens[i]) + 1, np.int32) for i in range(B)]
    for i in range(B):
        out[i][0] = traj[i][0]
    rounds, n_toks, accepted = 0, 0, 0
    t0 = time.perf_counter()
    while True:
        act = [i for i in range(B) if done[i] < lens[i]]
        if not act:
            break
        drafts = []
        for i in act:
            k = int(min(budgets[i], lens[i] - done[i] - 1))        # never draft past the target length
            if tree is not None:                                   # suffix-tree drafter: longest match of what was emitted so far
                drafts.append(tree.propose(out[i][:done[i] + 1], max(k, 0))[1] if k > 0 else prop[i][:0])
            else:
                drafts.append(prop[i][done[i] + 1: done[i] + 1 + max(k, 0)])
        acc, nxt = dm.verify_step([ids[i] for i in act], [ctx0[i] + done[i] for i in act], drafts)
        dm.kv_commit([ids[i] for i in act], acc, nxt)
        for j, i in enumerate(act):
            a = int(acc[j])
            out[i][done[i] + 1: done[i] + 1 + a] = drafts[j][:a]
            out[i][done[i] + 1 + a] = nxt[j]
            done[i] += a + 1
            accepted += a
        rounds += 1
        n_toks += sum(len(d) + 1 for d in drafts)
    return out, time.perf_counter() - t0, rounds, n_toks, accepted


def solver_budgets(lens, c_base, c_tok, alpha, cap, k_max):
    """Per-sequence chain lengths from the budget model of Sec. 4.2.1 (das_budget_solve): target lengths as l_i, one
    accept efficiency and capacity factor for the whole batch, the forward-latency constants of Eq. 1."""
    from . import budget
    reqs = [(float(l), alpha, cap) for l in lens]
    n_fwd, p = budget.solve(reqs, c_base, c_tok)
    return budget.draft_lens(p, n_fwd, k_max).astype(np.int64), n_fwd


def run(model="7b", batch=64, max_len=512, accept_p=0.7, k_medium=4, k_long=8, ctx_lo=256, ctx_hi=1024, seed=4000,
        n_layers=None, policy="classes", c_base=8.0, c_tok=0.017, alpha=0.6, cap=0.9, drafter="synthetic", keep_rollouts=False):
    """keep_rollouts: also return, under "rollouts", what a checker needs to replay the batch elsewhere: the context
    lengths, the first pending tokens, the seed of the synthetic KV (sequence i has key i) and both token streams."""
    shape = di.MODELS[model]
    if n_layers is not None:
        shape = shape.replace(n_layers=n_layers)
    rng = np.random.default_rng(seed)
    ctx0 = rng.integers(ctx_lo, ctx_hi + 1, size=batch).astype(np.int64)
    lens = target_lengths(batch, max_len, seed + 1)
    predicted_n_fwd = None
    if policy == "solver":
        budgets, predicted_n_fwd = solver_budgets(lens, c_base, c_tok, alpha, cap, max(k_medium, k_long, 1))
    else:
        budgets = class_budgets(lens, k_medium, k_long)
    kmax = int(max(k_medium, k_long, 1))
    room = int(max_len) + kmax + 4
    pages = int(sum(-(-(int(c) + room) // 16) for c in ctx0)) + 16
    dm = das.DasModel(das.config_for(shape, max_seqs=batch, max_ctx=-(-(int(ctx0.max()) + room + 16) // 16) * 16,
                                     max_rows=max(batch * (kmax + 1), 256), max_draft=kmax, num_pages=pages), None, seed=0)
    ids = list(range(batch))
    pend0 = rng.integers(0, shape.vocab, size=batch, dtype=np.int32)
    for i in ids:
        dm.seq_create(i, int(ctx0[i]), int(pend0[i]))
        dm.kv_synth(i, seed, i)
    log(f"[makespan] {model}: batch {batch}, contexts {int(ctx0.min())}-{int(ctx0.max())}, target lengths "
        f"median {int(np.median(lens))} / max {int(lens.max())}")
    traj, t_plain, r_plain, n_plain, hist = decode_plain(dm, ids, ctx0, pend0, lens)
    log(f"[makespan] plain decoding: {t_plain:.3f}s, {r_plain} forwards, {n_plain} tokens")
    dm.seq_rewind(ids, ctx0, pend0)
    tree = None
    if drafter == "tree":
        # the previous epoch's rollouts of the same prompts, indexed in a suffix tree (Sec. 4.1.2); the policy has not
        # moved between the two epochs here, the limit of the recency effect the paper builds on
        from .drafter import Drafter
        tree = Drafter(max_epochs=1)
        t0 = time.perf_counter()
        for t in traj:
            tree.add(t)
        log(f"[makespan] suffix tree over {tree.size()['tokens']} tokens built in {(time.perf_counter() - t0) * 1e3:.1f} ms")
    out, t_spec, r_spec, n_spec, accepted = decode_speculative(dm, ids, ctx0, lens, traj, budgets, accept_p,
                                                               shape.vocab, seed + 2, tree)
    log(f"[makespan] speculative: {t_spec:.3f}s, {r_spec} forwards, {n_spec} tokens processed, {accepted} drafts accepted")
    mismatched = sum(int(not np.array_equal(out[i], traj[i])) for i in ids)
    dm.free()
    half = next((r for r, n in enumerate(hist) if n <= batch // 2), len(hist))
    extra = {"rollouts": {"ctx0": ctx0, "pend0": pend0, "kv_seed": seed, "plain": traj, "speculative": out}} if keep_rollouts else {}
    return {**extra, "model": model, "n_layers": shape.n_layers, "batch": batch, "drafter": drafter,
            "accept_p": accept_p if drafter == "synthetic" else None,
            "policy": policy, "budgets": {"short": 0, "medium": k_medium, "long": k_long} if policy == "classes" else
            {"k_max": kmax, "mean_k": float(np.mean(budgets)), "sequences_without_speculation": int((budgets == 0).sum()),
             "model_forward_passes": predicted_n_fwd},
            "target_len": {"median": int(np.median(lens)), "max": int(lens.max()), "sum": int(lens.sum())},
            "plain": {"makespan_s": t_plain, "forwards": r_plain, "tokens_processed": n_plain,
                      "forwards_until_half_the_batch_is_done": half},
            "speculative": {"makespan_s": t_spec, "forwards": r_spec, "tokens_processed": n_spec,
                            "accepted_drafts": accepted},
            "speedup": t_plain / t_spec, "forward_reduction": 1.0 - r_spec / r_plain,
            "sequences_differing_from_plain_decoding": mismatched}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="7b")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--max-len", type=int, default=512)
    ap.add_argument("--accept-p", type=float, default=0.7)
    ap.add_argument("--k-medium", type=int, default=4)
    ap.add_argument("--k-long", type=int, default=8)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--policy", choices=["classes", "solver"], default="classes",
                    help="classes: none/medium/long chains by target-length third; solver: chain lengths from das_budget_solve")
    ap.add_argument("--drafter", choices=["synthetic", "tree"], default="synthetic",
                    help="synthetic: the recorded continuation corrupted with probability 1-p; tree: das_drafter over the plain pass's rollouts")
    ap.add_argument("--c-base", type=float, default=8.0, help="ms per forward pass (Eq. 1), for --policy solver")
    ap.add_argument("--c-tok", type=float, default=0.017, help="ms per processed token (Eq. 1), for --policy solver")
    ap.add_argument("--alpha", type=float, default=0.6, help="accept efficiency of the drafter (Eq. 3), for --policy solver")
    ap.add_argument("--cap", type=float, default=0.9, help="drafter capacity factor k (Eq. 3), for --policy solver")
    a = ap.parse_args()
    print(json.dumps(run(a.model, a.batch, a.max_len, a.accept_p, a.k_medium, a.k_long, n_layers=a.layers, policy=a.policy,
                         c_base=a.c_base, c_tok=a.c_tok, alpha=a.alpha, cap=a.cap, drafter=a.drafter)))


if __name__ == "__main__":
    main()
