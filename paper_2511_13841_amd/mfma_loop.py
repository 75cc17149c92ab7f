"""What the matrix pipe delivers in a loop shaped like the GEMM kernels' inner loop, and at which shader clock.

    python -m paper_2511_13841_amd.mfma_loop

Runs das_debug_mfma_loop in its three modes (operands in registers; operands read from LDS; operands from LDS plus the
GEMM's HBM/L2 -> LDS copy traffic and barriers) and prints, per mode, the time one SIMD spends per
v_mfma_f32_32x32x16_bf16, the shader clock the loop ran at and the bf16 rate of the whole chip.  The projection GEMMs
of the verify step (Sec. 4.2.1: c_tok, the compute cost per processed token) cannot run faster than the last line.
"""
import argparse
import json

MODES = {0: "operands in registers (constant)", 1: "operands read from LDS (random bf16)", 2: "operands from LDS + the GEMM's tile copies and barriers"}


def measure(iters=4000):
    from . import binding
    rows = []
    for mode, what in MODES.items():
        ns, ghz, pf = binding.debug_mfma_loop(mode, iters)
        rows.append({"mode": mode, "loop": what, "ns_per_mfma": ns, "cycles_per_mfma": ns * ghz, "shader_GHz": ghz, "PFLOPps": pf,
                     "of_2p5_peak": pf / 2.5})
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--iters", type=int, default=4000)
    args = ap.parse_args()
    rows = measure(args.iters)
    print("| loop | ns per MFMA and SIMD | shader cycles per MFMA | shader clock GHz | chip PFLOP/s | of the 2.5 PFLOP/s peak |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['loop']} | {r['ns_per_mfma']:.2f} | {r['cycles_per_mfma']:.1f} | {r['shader_GHz']:.2f} | {r['PFLOPps']:.3f} | {r['of_2p5_peak']:.2f} |")
    print(json.dumps(rows))


if __name__ == "__main__":
    main()
