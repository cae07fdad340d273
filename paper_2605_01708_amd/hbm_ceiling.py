"""What the memory system of this GPU gives a plain streaming kernel at best: a sweep of
splitzip_traffic_probe_shape over traffic mix (read only, write only, the codec's 4:3 and 3:4 mixes, a copy),
workgroups per CU (or one workgroup per step, handed out by the dispatcher), 4 KB runs in flight per workgroup, temporal / non-temporal accesses, round-robin or blocked
ownership of the runs, and the alignment of the written buffer against the read one.

    python -m paper_2605_01708_amd.hbm_ceiling [--gib 4] [--reps 3] [--quick]

Prints one line per setting and, last, one JSON line with the best setting of every mix ("GBps" counts bytes read
plus bytes written; "frac" is against the published 8 TB/s).  The codec's kernels are judged against these
figures: a kernel at the ceiling of its mix cannot be made faster by re-arranging its accesses.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

import paper_2605_01708_amd as sz

HBM_PEAK_GBPS = 8000.0

MIXES = {
    "read_only": [(1, 0), (2, 0), (4, 0), (8, 0)],
    "write_only": [(0, 1), (0, 2), (0, 4), (0, 8)],
    "compress_4_3": [(4, 3), (8, 6), (16, 12)],
    "decompress_3_4": [(3, 4), (6, 8), (12, 16)],
    "copy_1_1": [(1, 1), (2, 2), (4, 4)],
}


def time_shape(src, dst, rbytes, wbytes, r, w, wgs, flags, reps):
    """GB/s (read + written) of one setting, HIP events on the current stream around `reps` launches"""
    sz.traffic_probe_shape(src, rbytes, dst, wbytes, r, w, wgs, flags)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        sz.traffic_probe_shape(src, rbytes, dst, wbytes, r, w, wgs, flags)
    e1.record()
    torch.cuda.synchronize()
    moved = (rbytes if r else 0) + (wbytes if w else 0)
    return moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def sweep(gib: float = 4.0, reps: int = 3, quick: bool = False, out=sys.stdout):
    """Returns {mix: best setting}; prints every setting to `out` (None: silent)."""
    unit = int(gib * (1 << 30)) // (48 * 4096) * (48 * 4096)     # whole steps for every (reads, writes) pair
    src = torch.empty(unit + (2 << 20), dtype=torch.uint8, device="cuda")
    dst = torch.empty(unit + (2 << 20), dtype=torch.uint8, device="cuda")
    src.random_(0, 256)
    torch.cuda.synchronize()
    wgs_list = [0, 8] if quick else [0, 1, 2, 4, 8, 16]   # 0: one workgroup per step, in dispatch order
    best = {}
    for mix, shapes in MIXES.items():
        for r, w in ((shapes[:1] + shapes[-1:]) if quick else shapes):
            # bytes of each side so that both run the same number of steps
            rbytes = unit if r >= w else unit // w * r
            wbytes = unit if w >= r else unit // r * w
            for wgs in wgs_list:
                # a flag for a side the mix does not have, or for an ownership the setting does not have, is left out
                absent = (0 if r else 1) | (0 if w else 2) | (4 if wgs == 0 else 0)
                usable = sorted({f & ~absent for f in (3, 7)}) if quick else [f for f in range(8) if not f & absent]
                for flags in usable:
                    gbps = time_shape(src, dst, rbytes, wbytes, r, w, wgs, flags, reps)
                    rec = {"mix": mix, "reads": r, "writes": w, "wgs_per_cu": wgs, "nt_loads": bool(flags & 1),
                           "nt_stores": bool(flags & 2), "blocked": bool(flags & 4), "GBps": round(gbps, 1),
                           "frac": round(gbps / HBM_PEAK_GBPS, 4)}
                    if out:
                        print(json.dumps(rec), file=out, flush=True)
                    if mix not in best or gbps > best[mix]["GBps"]:
                        best[mix] = rec
    # the written buffer shifted against the read one, at the best compress-mix setting
    b = best["compress_4_3"]
    flags = (1 if b["nt_loads"] else 0) | (2 if b["nt_stores"] else 0) | (4 if b["blocked"] else 0)
    shifts = {}
    for shift in (0, 256, 512, 1024, 2048, 4096, 8192, 65536 + 4096, (1 << 20) + 4096 + 256):
        rbytes, wbytes = unit, unit // b["reads"] * b["writes"]
        gbps = time_shape(src, dst[shift:], rbytes, wbytes, b["reads"], b["writes"], b["wgs_per_cu"], flags, reps)
        shifts[str(shift)] = round(gbps, 1)
        if out:
            print(json.dumps({"mix": "compress_4_3", "dst_shift_bytes": shift, "GBps": round(gbps, 1)}), file=out, flush=True)
    best["compress_4_3_dst_shift_GBps"] = shifts
    return best


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--gib", type=float, default=4.0, help="bytes of the larger side of every mix")
    p.add_argument("--reps", type=int, default=3)
    p.add_argument("--quick", action="store_true", help="a handful of settings only")
    a = p.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    best = sweep(a.gib, a.reps, a.quick)
    print(json.dumps({"hbm_ceiling": best, "peak_GBps": HBM_PEAK_GBPS, "gib": a.gib, "reps": a.reps}))


if __name__ == "__main__":
    main()
