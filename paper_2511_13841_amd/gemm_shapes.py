"""Per-projection GEMM timing at a workload's row count: full launch against the same launch with its arithmetic off.

    python -m paper_2511_13841_amd.gemm_shapes --workload c4

For every projection of the workload's model (QKV, O, gate/up, down, LM head) at the number of rows a verification
pass of that workload has, prints the device time of one launch (weights rotating over several sets, so they are
cold as in a decoder pass), the time of the same launch with copies and barriers only, and what the full time is
of the two rooflines (weight bytes over 8 TB/s; flop over 2.5 PFLOP/s).  The copies-only column shows which shapes
are bound by their copy stream rather than by the matrix pipe (Sec. 4.2.1 calls the few-row part c_base: the cost of
moving the parameters).  With --vendor the same shapes are also timed through torch.matmul (the vendor's GEMM library,
bf16 in and out, no epilogue, weights rotating the same way): a reference point for what these shapes reach on this
chip, not part of the product path.
"""
import argparse
import json


def projections(shape, rows):
    """(name, epilogue id of das_debug_gemm_time, M, N, K, weight sets) per projection; gate/up counts both halves in N."""
    d, hq, hkv, hd, f, v = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab
    fp = -(-f // 64) * 64
    big = lambda n, k: max(2, min(16, int(600e6 // (2 * n * k))))      # enough sets to exceed the 256 MB memory-side cache
    return [("qkv", 3, rows, (hq + 2 * hkv) * hd, d, big((hq + 2 * hkv) * hd, d)), ("o", 1, rows, d, hq * hd, big(d, hq * hd)),
            ("gate_up", 2, rows, 2 * fp, d, big(2 * fp, d)), ("down", 1, rows, d, fp, big(d, fp)),
            ("lm_head", 4, rows, v, d, 3)]


def vendor_us(M, N, K, sets, iters):
    """torch.matmul on (M x K) x (N x K)^T in bf16: mean device time of one call, weights rotating over `sets` matrices."""
    import torch
    dev = torch.device("cuda")
    a = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
    ws = [torch.randn(N, K, device=dev, dtype=torch.bfloat16) * 0.02 for _ in range(sets)]
    for i in range(3):
        a @ ws[i % sets].t()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        a @ ws[i % sets].t()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def measure(workload, rows=None, iters=24, vendor=False):
    import das_inputs as di
    from . import binding
    wl = di.WORKLOADS[workload]
    shape = di.MODELS[wl.model]
    if rows is None:
        ctx = di.context_lengths(wl)
        rows = int((di.draft_budgets(wl, ctx) + 1).sum())
    out = []
    for name, epi, M, N, K, sets in projections(shape, rows):
        if epi == 4:
            M = min(M, wl.batch * (di.max_budget(wl) + 1))
        full = binding.debug_gemm_time(epi, M, N, K, iters=iters, weight_sets=sets)
        copies = binding.debug_gemm_time(epi, M, N, K, iters=iters, weight_sets=sets, copies_only=True)
        wbytes, flop = 2.0 * N * K, 2.0 * M * N * K
        out.append({"projection": name, "M": M, "N": N, "K": K, "us": full, "us_copies_only": copies,
                    "weight_TBps": wbytes / full / 1e6, "PFLOPps": flop / full / 1e9,
                    "frac_of_floor": max(wbytes / 8e12, flop / 2.5e15) * 1e6 / full})
        if vendor:
            out[-1]["us_vendor_library"] = vendor_us(M, N, K, sets, iters)
    return {"workload": workload, "model": wl.model, "rows": rows, "projections": out}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--rows", type=int, default=None, help="rows of the pass (default: the workload's own)")
    ap.add_argument("--iters", type=int, default=24)
    ap.add_argument("--vendor", action="store_true", help="also time torch.matmul (the vendor's GEMM library) on the same shapes")
    args = ap.parse_args()
    r = measure(args.workload, args.rows, args.iters, args.vendor)
    print(f"| projection | M | N | K | us | us, copies only | weights TB/s | PFLOP/s | of max(HBM, MFMA) floor |" + (" us, vendor library |" if args.vendor else ""))
    print("|---|---|---|---|---|---|---|---|---|" + ("---|" if args.vendor else ""))
    for p in r["projections"]:
        print(f"| {p['projection']} | {p['M']} | {p['N']} | {p['K']} | {p['us']:.1f} | {p['us_copies_only']:.1f} | {p['weight_TBps']:.2f} | "
              f"{p['PFLOPps']:.3f} | {p['frac_of_floor']:.2f} |" + (f" {p['us_vendor_library']:.1f} |" if args.vendor else ""))
    print(json.dumps(r))


if __name__ == "__main__":
    main()
