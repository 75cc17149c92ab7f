"""What the HBM/L2 -> LDS copy ring of the kernels delivers on this GPU, measured by itself.

    python -m paper_2511_13841_amd.copy_ring

Runs das_debug_copy_ring over ring depths, numbers of busy compute units, shares of copies that hit L2 and the
non-temporal hint, and prints one line per configuration: bytes into LDS per second for the chip and per compute
unit, and the part of it that comes from HBM.  The GEMM and attention kernels of the verify step are fed by exactly
this loop, so these are the ceilings their copy streams are read against.
"""
import argparse
import json

# (stages, copies of 1 KiB per wave and tile, of which shared)  ->  tile = 4 * copies KiB
SHAPES = [(4, 4, 0), (9, 4, 0), (4, 9, 0), (4, 4, 4), (9, 4, 4), (4, 9, 9), (4, 9, 6), (4, 9, 3), (5, 7, 5), (3, 7, 5)]


def measure(workgroup_counts=(32, 256), tiles=256):
    from . import binding
    rows = []
    for wgs in workgroup_counts:
        for stages, copies, shared in SHAPES:
            for nt in ((False, True) if shared < copies else (False,)):
                us, nbytes = binding.debug_copy_ring(wgs, stages, copies, shared, tiles=tiles, non_temporal=nt)
                rows.append({"workgroups": wgs, "stages": stages, "tile_KiB": 4 * copies, "shared_KiB": 4 * shared, "non_temporal": nt,
                             "us": us, "TBps_into_lds": nbytes / us / 1e6, "GBps_per_cu": nbytes / us / 1e3 / wgs,
                             "TBps_from_hbm": nbytes * (copies - shared) / copies / us / 1e6})
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workgroups", default="32,256")
    ap.add_argument("--tiles", type=int, default=256)
    args = ap.parse_args()
    rows = measure(tuple(int(x) for x in args.workgroups.split(",")), args.tiles)
    print("| busy CUs | stages | tile KiB | of it shared (L2 hits) | private stream | us | into LDS TB/s | per CU GB/s | from HBM TB/s |")
    print("|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        hint = "-" if r["shared_KiB"] == r["tile_KiB"] else ("non-temporal" if r["non_temporal"] else "plain")
        print(f"| {r['workgroups']} | {r['stages']} | {r['tile_KiB']} | {r['shared_KiB']} | {hint} | {r['us']:.1f} | {r['TBps_into_lds']:.2f} | "
              f"{r['GBps_per_cu']:.1f} | {r['TBps_from_hbm']:.2f} |")
    print(json.dumps(rows))


if __name__ == "__main__":
    main()
