"""Fit the forward-latency model of Sec. 4.2.1, Eq. 1, on this GPU and sweep the uniform draft budget.

    python -m paper_2511_13841_amd.latency_model [--workload c3] [--ks 0,1,2,4,8,16,32] [--steps 5]

The paper models one forward pass as  t_fwd = c_base + c_tok * n_toks  (n_toks = tokens processed, accepted
and speculative alike) and argues from it that proposing too many tokens costs more than it saves
(Sec. 4.2.1; Sec. 5.3's budget study).  This tool measures verify steps (das_verify_step + das_kv_commit,
wall clock, host transfers included) on one workload's contexts with every sequence given the same chain
length k, fits (c_base, c_tok) by least squares, and turns the measured step times into emitted tokens per
second for a drafter of acceptance p with the closed form of a chain draft,
E[emitted per round] = (1 - q^(k+1)) / (1 - q),  q = p + (1-p)/V.
The drafts are random tokens (all rejected), so the contexts stay what they are from one k to the next.
One JSON object is printed.
"""
import argparse
import dataclasses
import json
import time

import numpy as np

import das_inputs as di
from .rollout import Rollout, log


def fit_line(x, y):
    """Least-squares (intercept, slope, r^2) of y = a + b x."""
    x = np.asarray(x, np.float64)
    y = np.asarray(y, np.float64)
    A = np.stack([np.ones_like(x), x], axis=1)
    (a, b), *_ = np.linalg.lstsq(A, y, rcond=None)
    res = y - (a + b * x)
    ss = ((y - y.mean()) ** 2).sum()
    return float(a), float(b), float(1.0 - (res ** 2).sum() / ss) if ss > 0 else 1.0


def expected_emitted(p, k, vocab):
    q = p + (1.0 - p) / vocab
    return (1.0 - q ** (k + 1)) / (1.0 - q)


def sweep(workload="c3", ks=(0, 1, 2, 4, 8, 16, 32), steps=5, warmup=1, layers=None, accept_p=None, batch=None):
    """Measure verify steps at uniform chain lengths `ks` on the workload's contexts, fit Eq. 1, and convert the measured
    times into emitted tokens/s for a drafter of acceptance p.  Returns the report (a JSON-able dict)."""
    ks = [int(k) for k in ks]
    wl = di.WORKLOADS[workload]
    p = wl.accept_p if accept_p is None else accept_p
    ro = Rollout(dataclasses.replace(wl, mode="greedy"), batch=batch, n_layers=layers, kmax=max(ks),
                 max_steps=(steps + warmup) * len(ks) + 2)
    ro.random_proposals()
    rows = []
    for k in ks:
        ro.wl = dataclasses.replace(ro.wl, budgets=f"k{k}")
        for _ in range(warmup):
            ro.step()
        t0 = time.perf_counter()
        for _ in range(steps):
            ro.step()
        ms = (time.perf_counter() - t0) / steps * 1e3
        n_toks = ro.B * (k + 1)
        e = expected_emitted(p, k, ro.shape.vocab)
        rows.append({"k": k, "n_toks": n_toks, "ms_per_step": ms, "expected_emitted_per_seq": e,
                     "emitted_tokens_per_s": ro.B * e / (ms * 1e-3)})
        log(f"[latency] k={k:2d} n_toks={n_toks:5d} {ms:8.3f} ms/step  -> {rows[-1]['emitted_tokens_per_s']:.0f} tok/s at p={p}")
    c_base, c_tok, r2 = fit_line([r["n_toks"] for r in rows], [r["ms_per_step"] for r in rows])
    pred = [c_base + c_tok * r["n_toks"] for r in rows]
    best = max(rows, key=lambda r: r["emitted_tokens_per_s"])
    out = {"workload": workload, "model": wl.model, "batch": ro.B, "kv_tokens": int(ro.ctx0.sum()),
           "n_layers": ro.shape.n_layers, "accept_p": p,
           "fit": {"c_base_ms": c_base, "c_tok_ms": c_tok, "r2": r2, "model": "t_fwd = c_base + c_tok * n_toks",
                   "mean_relative_error": float(sum(abs(q - r["ms_per_step"]) / r["ms_per_step"] for q, r in zip(pred, rows)) / len(rows))},
           "sweep": rows, "best_k": best["k"],
           "over_proposing_hurts": bool(rows[-1]["emitted_tokens_per_s"] < best["emitted_tokens_per_s"])}
    ro.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--ks", default="0,1,2,4,8,16,32")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--accept-p", type=float, default=None)
    a = ap.parse_args()
    print(json.dumps(sweep(a.workload, [int(x) for x in a.ks.split(",")], a.steps, a.warmup, a.layers, a.accept_p, a.batch)))


if __name__ == "__main__":
    main()
