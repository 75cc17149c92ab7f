#!/usr/bin/env python3
"""Throughput of the batched speculative-verification step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

A "step" is one whole round of the hot path over one batch of synthetic input:
das_verify_step (ragged (1+k_i)-row forward over the paged KV, acceptance) followed
by das_kv_commit of its own decisions.  Contexts, weights and drafts are seeded
and synthetic (das_inputs); nothing is read from disk.  One JSON line is printed.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import das_inputs as di                      # noqa: E402

HBM_PEAK_GBS = 8000.0                        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0               # MI355X dense bf16 MFMA, published
RIDGE_ROWS = 312                             # rows above which a weight GEMM is MFMA- rather than HBM-bound


def log(*a):
    print(*a, file=sys.stderr, flush=True)


import paper_2511_13841_amd as das                      # noqa: E402
from paper_2511_13841_amd.rollout import Rollout      # noqa: E402


def kernel_rooflines(shape, prof, T, kv_tokens, n_steps):
    """Per kernel class: ms per launch, algorithmic bytes / flops per launch, achieved rate, fraction of peak."""
    d, qd, kd, Fp, V = shape.d_model, shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim, \
        -(-shape.d_ffn // 64) * 64, shape.vocab
    gemms = {"gemm_qkv": ((qd + 2 * kd), d), "gemm_o": (d, qd), "gemm_gateup_silu": (2 * shape.d_ffn, d),
             "gemm_down": (d, shape.d_ffn), "gemm_lm_head": (V, d)}
    out = {}
    for name, (ms, n) in prof.items():
        if n == 0:
            continue
        per = ms / n
        e = {"ms_per_launch": per, "launches_per_step": n / n_steps, "ms_per_step": ms / n_steps}
        if name in gemms:
            N, K = gemms[name]
            flops, wbytes = 2.0 * T * N * K, 2.0 * N * K
            if T >= RIDGE_ROWS:
                e.update(bound="mfma", achieved=flops / per / 1e9, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s")
            else:
                e.update(bound="hbm", achieved=wbytes / per / 1e6, peak=HBM_PEAK_GBS, unit="GB/s")
        elif name == "attention":
            # KV of every visible position read once per layer + the new rows' K/V, q in, partials out not counted
            b = kv_tokens * 2.0 * kd * 2
            e.update(bound="hbm", achieved=b / per / 1e6, peak=HBM_PEAK_GBS, unit="GB/s")
        else:
            out[name] = e
            continue
        e["frac"] = e["achieved"] / e["peak"]
        out[name] = e
    return out


def _gemm_epilogue(kernel_name):
    """Sixth template argument of gemm_kernel<...> (the epilogue), or None for other kernels."""
    if not kernel_name.startswith("gemm_kernel<"):
        return None
    args = kernel_name[len("gemm_kernel<"):].rstrip(">").split(", ")
    return args[5] if len(args) > 5 else None


def stored_traffic(workload, kernel_class):
    """HBM-side bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, each
    scaled by the plain copy kernel), if one exists for this workload and kernel class; else None."""
    path = os.path.join(ROOT, "profiles", f"verify_step_{workload}_traffic.json")
    match = {"attention": lambda k: k.startswith("attn_partial_kernel"),
             "attention_merge": lambda k: k.startswith("attn_merge_kernel"),
             "gemm_gateup_silu": lambda k: _gemm_epilogue(k) == "2",
             "gemm_lm_head": lambda k: _gemm_epilogue(k) == "4"}.get(kernel_class)
    if not match or not os.path.exists(path):
        return None
    per = json.load(open(path))["per_launch"]
    hits = [v for k, v in per.items() if match(k)]
    return sum(v["fetch_bytes"] + v["write_bytes"] for v in hits) if hits else None


def cpu_baseline(ro, budget_s=20.0):
    """The oracle, as it stands, on a bounded sample of the same step: the first sequences of the batch
    (batch order is already random) with synthetic KV of the same generator, one verify round each."""
    import oracle
    shape = ro.shape
    t0 = time.time()
    om = oracle.OracleModel(shape, di.bf16_to_f32(ro.blob))
    log(f"[bench] oracle weights widened in {time.time() - t0:.1f}s")
    ks = di.draft_budgets(ro.wl, ro.ctx0)
    flops_per_row = 2.0 * shape.streamed_params
    rows, tokens, secs, used = 0, 0, 0.0, []
    order = np.argsort(ro.ctx0, kind="stable")           # shortest first: bounded memory and time
    est_rate = 15e9 * oracle.num_threads()               # only to size the sample before the first timing
    for i in order:
        k = int(ks[i])
        if secs + (1 + k) * flops_per_row / est_rate > budget_s and used:
            break
        c = int(ro.ctx0[i])
        s = om.new_seq(c + k + 1)
        for layer in range(shape.n_layers):
            s.kv(layer, 0)[:c] = di.bf16_to_f32(di.kv_synth(ro.seed, int(i), layer, 0, 0, c, shape.n_kv_heads, shape.head_dim))
            s.kv(layer, 1)[:c] = di.bf16_to_f32(di.kv_synth(ro.seed, int(i), layer, 1, 0, c, shape.n_kv_heads, shape.head_dim))
        s.len, s.pending = c, int(ro.pending0[i])
        drafts = ro.proposal[i, 1:1 + k]
        t1 = time.time()
        a, nxt, _ = om.verify_greedy(s, drafts)
        dt = time.time() - t1
        secs += dt
        rows += 1 + k
        tokens += a + 1
        used.append(int(i))
        est_rate = rows * flops_per_row / secs
        s.close()
        if secs > budget_s:
            break
    om.close()
    return {"value": tokens / secs, "unit": "emitted tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{len(used)} shortest sequences of the batch ({rows} rows, synthetic KV), one verify round each, "
                      f"{secs:.1f}s of CPU time"}


def measure(args, name, K, W, with_cpu_baseline):
    """K timed rounds of one workload (after W warm-up rounds) and the same K rounds again with per-launch events.
    Returns the fields of the bench line that belong to this workload."""
    import torch
    wl = di.WORKLOADS[name]
    ro = Rollout(wl, batch=args.batch, n_layers=args.layers, context=args.context, max_steps=W + 2 * K + 1)
    ro.faithful = args.faithful
    ro.rollback = args.rollback
    if args.drafts == "trajectory" and wl.mode == "greedy":
        ro.generate_trajectories()
    else:
        ro.random_proposals()

    for _ in range(W):
        ro.step()
    torch.cuda.synchronize()
    emitted = accepted = rows = kv_read = 0
    t0 = time.perf_counter()
    for _ in range(K):
        T, kv = ro.step_shape()
        ks, acc, _ = ro.step()
        emitted += int((acc + 1).sum()); accepted += int(acc.sum()); rows += T; kv_read += kv
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    roof, roof_attn, kernels, ms_prof = None, None, None, None
    if not args.no_profile:
        # the same K steps again, every launch bracketed by HIP events on the library's stream
        ro.dm.profile_enable(True)
        ro.dm.profile_reset()
        Tsum = kvsum = 0
        t1 = time.perf_counter()
        for _ in range(K):
            T, kv = ro.step_shape()
            Tsum += T; kvsum += kv
            ro.step()
        ms_prof = (time.perf_counter() - t1) / K * 1e3
        prof = ro.dm.profile_read()
        ro.dm.profile_enable(False)
        kernels = kernel_rooflines(ro.shape, prof, Tsum / K, kvsum / K, K)
        cand = {k: v for k, v in kernels.items() if "frac" in v}
        dom = max(cand, key=lambda k: cand[k]["ms_per_step"])
        total = sum(v["ms_per_step"] for v in kernels.values())

        def roof_of(k):
            e = cand[k]
            e["algorithmic"] = e["achieved"] * e["ms_per_launch"] * (1e9 if e["unit"] == "TFLOP/s" else 1e6)
            return {"kernel": k, "algorithmic_per_launch": e["algorithmic"], "bound": e["bound"], "achieved": e["achieved"],
                    "peak": e["peak"], "unit": e["unit"], "frac": e["frac"], "traffic": stored_traffic(wl.name, k),
                    "ms_per_launch": e["ms_per_launch"], "share_of_step": e["ms_per_step"] / total}
        roof = roof_of(dom)
        # the metric names the HBM roofline: the attention kernel's line is always reported, also when a GEMM class has
        # the larger share of the step (on c3 the two are within a few per cent of each other)
        roof_attn = roof if dom == "attention" or "attention" not in cand else roof_of("attention")

    if args.calibrate_copy:
        das.debug_copy(args.calibrate_copy << 20, 3)

    cpu = None
    if with_cpu_baseline and args.drafts == "trajectory" and wl.mode == "greedy":
        cpu = cpu_baseline(ro)

    # whole-step figures: algorithmic bytes of a step = every matrix once + the KV of every visible position once + the
    # new rows' KV written; its floor = (GEMMs at the matrix peak, or at the weight stream below the ridge) + KV stream
    shape = ro.shape
    ms = dt / K * 1e3
    w_bytes = 2.0 * shape.streamed_params
    kv_bytes = (kv_read / K + rows / K) * shape.kv_bytes_per_token
    gemm_floor = max(2.0 * (rows / K) * shape.streamed_params / (MFMA_BF16_PEAK_TFLOPS * 1e12), w_bytes / (HBM_PEAK_GBS * 1e9))
    floor_ms = (gemm_floor + kv_bytes / (HBM_PEAK_GBS * 1e9)) * 1e3
    out = {
        "value": emitted / dt, "ms_per_step": ms,
        "config": {"workload": f"{wl.name}: {wl.model} decoder, batch {ro.B}, lengths {wl.lengths}, budgets {wl.budgets}, "
                               f"drafter acceptance p={wl.accept_p}, context={args.context}"
                               + (f", layers={args.layers}" if args.layers else ""),
                   "rows_per_step": rows / K, "kv_tokens": int(ro.ctx0.sum())},
        "accepted_draft_tokens_per_s": accepted / dt,
        "mean_accept_len": accepted / (K * ro.B),
        "whole_step": {"algorithmic_bytes": w_bytes + kv_bytes, "hbm_frac": (w_bytes + kv_bytes) / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9),
                       "floor_ms": floor_ms, "floor_over_time": floor_ms / ms},
        "context_s": ro.context_s, "prefill_s": ro.context_s if args.context == "prefill" else None,
        "context_tokens_per_s": int(ro.ctx0.sum()) / ro.context_s if args.context == "prefill" else None,
        "roofline": roof, "roofline_attention": roof_attn, "cpu_baseline": cpu,
        "ms_per_step_with_events": ms_prof, "kernels": kernels,
    }
    ro.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads timed after the headline one and reported under `workloads` "
                         "(default: c4,c2,c5 when the headline is c3 with default settings; 'none' for none)")
    ap.add_argument("--context", default="prefill", choices=["synth", "prefill"],
                    help="how the contexts come to be: real das_prefill of random prompts (default), or synthetic KV written on the device")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--drafts", default="trajectory", choices=["trajectory", "random"],
                    help="random: uniform random drafts, no plain-decoding pass (same kernel shapes; for profiler runs)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also launch a plain copy kernel of this size 3 times (profiler byte-counter reference)")
    ap.add_argument("--faithful", action="store_true",
                    help="stochastic workload: honest accept uniforms everywhere (acceptance ~0 on random-init weights)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rollback", action="store_true", help="roll every step back instead of committing it (contexts stay fixed; also for development kernels whose outputs are not valid)")
    ap.add_argument("--no-profile", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (sequences shard by data parallelism without any "
                 "exchange; there is no multi-GPU path to time).  Use --gpus 1.")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs an MI355X; no HIP device is visible")
    K, W = args.steps, args.warmup
    plain = args.batch is None and args.layers is None and not args.rollback and \
        args.drafts == "trajectory" and not args.calibrate_copy and not args.faithful
    also = args.also if args.also is not None else ("c4,c2,c5" if args.workload == "c3" and plain else "none")
    also = [w for w in also.split(",") if w and w != "none" and w != args.workload]

    head = measure(args, args.workload, K, W, with_cpu_baseline=not args.no_cpu_baseline)
    out = {
        "metric": "accepted tokens/s per MI355X in batched spec-verify; % of HBM roofline",
        "value": head.pop("value"), "unit": "emitted tokens/s (accepted drafts + the target's own token per round)",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    out.update(head)
    # the other configurations under the same clock: fewer fields, same definitions
    others = {}
    for name in also:
        log(f"[bench] workload {name}")
        r = measure(args, name, K, W, with_cpu_baseline=False)
        kern = r.pop("kernels") or {}
        gemms = {k: v for k, v in kern.items() if k.startswith("gemm_") and "frac" in v}
        dom = max(gemms, key=lambda k: gemms[k]["ms_per_step"]) if gemms else None
        others[name] = {
            "ms_per_step": r["ms_per_step"], "emitted_tokens_per_s": r["value"], "accepted_draft_tokens_per_s": r["accepted_draft_tokens_per_s"],
            "steps": K, "warmup": W, "config": r["config"], "whole_step": r["whole_step"],
            "prefill_s": r.get("prefill_s"), "context_tokens_per_s": r.get("context_tokens_per_s"),
            "attention": r["roofline_attention"] and {k: r["roofline_attention"][k] for k in ("achieved", "peak", "unit", "frac", "ms_per_launch", "share_of_step")},
            "dominant_gemm": dom and {"kernel": dom, **{k: gemms[dom][k] for k in ("bound", "achieved", "peak", "unit", "frac", "ms_per_launch")}},
            "kernels_ms_per_step": {k: v["ms_per_step"] for k, v in kern.items()},
        }
    out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
