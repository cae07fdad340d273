#!/usr/bin/env python3
"""SplitZip codec benchmark on one MI355X.

One step = one pass of the whole hot path over the workload: every tensor is
compressed (one launch each), then every stream is decompressed (one launch
each).  Inputs, streams and outputs are resident in HBM; the tensors of a
pass are all distinct and together far larger than the 256 MB last-level
cache, so every launch streams from HBM.

Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

import kv_synth
import paper_2605_01708_amd as sz

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
TOKENS = {"config1": 32768, "config0": 4096}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=2)
    p.add_argument("--workload", default="config1", choices=["config1", "config0", "config4"])
    p.add_argument("--layers", type=int, default=32, help="layers of the KV cache (config1/4: 32)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--cpu-sample-tensors", type=int, default=8)
    return p.parse_args()


def build_workload(args):
    """tensors (device, raw words), codebooks per kind"""
    dev = "cuda"
    if args.workload == "config0":
        dtype = sz.BF16
        xs = [("K", kv_synth.kv_bf16(4096, 0, 0, "K", dev))]
        cbs = {"K": sz.calibrate(kv_synth.kv_bf16(4096, 1, 0, "K"), dtype)}
        return dtype, xs, cbs
    dtype = sz.BF16 if args.workload == "config1" else sz.FP8_E5M2
    gen = kv_synth.kv_bf16 if dtype == sz.BF16 else kv_synth.kv_e5m2
    xs = []
    for layer in range(args.layers):
        for kind in ("K", "V"):
            xs.append((kind, gen(32768, 0, layer, kind, dev)))
    # one codebook per tensor kind from a seed-1 sample of 1024 tokens spread over the layers
    cbs = {}
    per = max(1, 1024 // args.layers)
    for kind in ("K", "V"):
        sample = torch.cat([gen(per, 1, layer, kind) for layer in range(args.layers)])
        cbs[kind] = sz.calibrate(sample, dtype)
    return dtype, xs, cbs


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the codec has no cross-GPU step (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dtype, xs, cbs = build_workload(args)
    es = 2 if dtype == sz.BF16 else 1
    n = xs[0][1].numel()
    nt = len(xs)
    raw_bytes = n * es
    # stream capacity: the fixed part plus room for 3 % escapes
    cap = (sz.total_bytes(n, n * 3 // 100, dtype) + 255) // 256 * 256
    comps = [torch.empty(cap, dtype=torch.uint8, device="cuda") for _ in range(nt)]
    outs = [torch.empty_like(x) for _, x in xs]
    sizes = [sz.new_sizes() for _ in range(nt)]
    dsizes = sz.new_sizes()
    ws = sz.Workspace(n, dtype)
    torch.cuda.synchronize()

    def compress_all():
        for i, (kind, x) in enumerate(xs):
            sz.compress(x, cbs[kind], comps[i], ws, sizes[i])

    def decompress_all(totals):
        for i, (kind, x) in enumerate(xs):
            sz.decompress(comps[i], totals[i], n, cbs[kind], outs[i], dsizes)

    # verify the round trip bit for bit before timing (the paper's protocol, section 4.1)
    compress_all()
    torch.cuda.synchronize()
    rec = [sz.read_sizes(s) for s in sizes]
    assert all(r[2] == 0 for r in rec), f"compress status {rec}"
    totals = [r[0] for r in rec]
    escapes = sum(r[1] for r in rec)
    decompress_all(totals)
    torch.cuda.synchronize()
    assert sz.read_sizes(dsizes)[2] == 0, "decompress flagged a bad stream"
    for (kind, x), y in zip(xs, outs):
        assert torch.equal(x, y), "round trip is not bit exact"

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    for _ in range(args.warmup):
        compress_all()
        decompress_all(totals)
    torch.cuda.synchronize()
    t_c, t_d = [], []
    wall0 = time.perf_counter()
    for _ in range(args.steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        compress_all()
        e1.record()
        decompress_all(totals)
        e2.record()
        t_c.append((e0, e1))
        t_d.append((e1, e2))
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_c = [a.elapsed_time(b) for a, b in t_c]
    ms_d = [a.elapsed_time(b) for a, b in t_d]
    mean = lambda v: sum(v) / len(v)  # noqa: E731
    std = lambda v: (sum((x - mean(v)) ** 2 for x in v) / len(v)) ** 0.5  # noqa: E731
    total_raw = raw_bytes * nt
    comp_gbps = total_raw / (mean(ms_c) * 1e-3) / 1e9
    dec_gbps = total_raw / (mean(ms_d) * 1e-3) / 1e9
    ms_step = wall / args.steps * 1e3
    blob_bytes = sum(totals)
    # algorithmic traffic of one launch: read the words, write the stream (and the reverse)
    alg_bytes = raw_bytes + blob_bytes / nt
    c_launch_us = mean(ms_c) * 1e3 / nt
    d_launch_us = mean(ms_d) * 1e3 / nt
    c_ach = alg_bytes / (c_launch_us * 1e-6) / 1e9
    d_ach = alg_bytes / (d_launch_us * 1e-6) / 1e9

    # plain streaming kernel with the codec's traffic (reads 4, writes 3 parts) into the decode outputs
    wbytes = raw_bytes * 3 // 4 // 16 * 16
    for _ in range(2):
        for i, (kind, x) in enumerate(xs):
            sz.traffic_probe(x, raw_bytes, outs[i], wbytes)
    p0, p1 = ev(), ev()
    p0.record()
    for _ in range(3):
        for i, (kind, x) in enumerate(xs):
            sz.traffic_probe(x, raw_bytes, outs[i], wbytes)
    p1.record()
    torch.cuda.synchronize()
    probe_gbps = (raw_bytes + wbytes) * nt * 3 / (p0.elapsed_time(p1) * 1e-3) / 1e9

    result = {
        "metric": "SplitZip compress+decompress throughput, uncompressed GB/s, 1 MI355X",
        "value": round(2 * total_raw / (ms_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16" if dtype == sz.BF16 else "u8",
        "data": "synthetic",
        "config": {
            "workload": {"config1": "Llama-3-8B-shaped BF16 KV cache: 32 layers x {K,V} x [32768,8,128], 64 launches per direction",
                         "config0": "single BF16 K tensor [4096,8,128] (cache resident)",
                         "config4": "FP8 E5M2 KV cache: 32 layers x {K,V} x [32768,8,128]"}[args.workload],
            "tensors": nt, "elems_per_tensor": n, "uncompressed_bytes": total_raw,
        },
        "compress_GBps": round(comp_gbps, 1),
        "compress_GBps_std": round(std([total_raw / (m * 1e-3) / 1e9 for m in ms_c]), 1),
        "decompress_GBps": round(dec_gbps, 1),
        "decompress_GBps_std": round(std([total_raw / (m * 1e-3) / 1e9 for m in ms_d]), 1),
        "ratio": round(total_raw / blob_bytes, 4),
        "escape_rate": round(escapes / (n * nt), 6),
        "B_hide_GBps": round(min(comp_gbps, dec_gbps) / (total_raw / blob_bytes), 1),
        "paper_context": {"compress_GBps": 613.3, "decompress_GBps": 2181.8, "ratio": 1.324, "hardware": "NVIDIA H200, real Qwen3-32B BF16 KV"},
        "roofline": {
            "kernel": "compress_kernel<1024, Bf16>" if dtype == sz.BF16 else "compress_kernel<1024, E5m2>",
            "bound": "hbm", "achieved": round(c_ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(c_ach / HBM_PEAK_GBPS, 4), "traffic": None,
            "launch_us": round(c_launch_us, 2), "algorithmic_bytes_per_launch": int(alg_bytes),
        },
        "roofline_decompress": {
            "kernel": "decompress_kernel<DBf16>" if dtype == sz.BF16 else "decompress_kernel<DE5m2>",
            "bound": "hbm", "achieved": round(d_ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(d_ach / HBM_PEAK_GBPS, 4), "traffic": None,
            "launch_us": round(d_launch_us, 2), "algorithmic_bytes_per_launch": int(alg_bytes),
        },
        "copy_kernel_same_traffic_GBps": round(probe_gbps, 1),
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, dtype, xs, cbs, comps, totals, n, es)
    print(json.dumps(result))


def cpu_baseline(args, dtype, xs, cbs, comps, totals, n, es):
    """The oracle as it stands, one thread, on the first few tensors of the same workload;
    its streams are also compared with the GPU's (parity at full size)."""
    import numpy as np

    import oracle

    k = min(args.cpu_sample_tensors, len(xs))
    odt = oracle.BF16 if dtype == sz.BF16 else oracle.E5M2
    t_c = t_d = 0.0
    for i in range(k):
        kind, x = xs[i]
        xh = kv_synth.to_numpy_words(x)
        cb = oracle.codebook_from_dec(np.array(cbs[kind].dec, np.uint8), odt)
        t0 = time.perf_counter()
        blob, m = oracle.compress(xh, cb)
        t1 = time.perf_counter()
        y = oracle.decompress(blob, n, cb)
        t2 = time.perf_counter()
        t_c += t1 - t0
        t_d += t2 - t1
        assert np.array_equal(y, xh)
        assert np.array_equal(comps[i][: totals[i]].cpu().numpy(), blob), "GPU stream differs from the oracle's"
    raw = k * n * es
    return {
        "value": round(2 * raw / (t_c + t_d) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {k} of {len(xs)} tensors ({raw / 2**20:.0f} MiB), compress+decompress, streams compared with the GPU's",
        "compress_GBps": round(raw / t_c / 1e9, 4), "decompress_GBps": round(raw / t_d / 1e9, 4),
        "host_cores_available": os.cpu_count(),
    }


if __name__ == "__main__":
    main()
