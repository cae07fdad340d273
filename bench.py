#!/usr/bin/env python3
"""SplitZip codec benchmark on one MI355X.

One step = one pass of the whole hot path over the workload: every tensor of
the KV cache is compressed (one splitzip_compress_batch call), then every
stream is decompressed (one splitzip_decompress_batch call).  Inputs, streams
and outputs are resident in HBM; the tensors of a pass are all distinct and
together far larger than the 256 MB last-level cache, so the kernels stream
from HBM.  The round trip is verified bit for bit before anything is timed
(the paper's protocol, section 4.1).

The headline workload is config 1 (the 4 GiB BF16 cache).  The same line also
carries, under "other_workloads", configs 0, 2, 3 and 4 (config 3, the 4 MiB
streaming calls, timed three ways: single calls, batch calls per chunk
position, and a captured HIP graph of one chunk position replayed), the
single-tensor calls under "per_tensor_calls", the best plain streaming
kernels of this GPU under "copy_ceiling", and the CPU oracle under
"cpu_baseline".

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import torch

import kv_synth
import paper_2605_01708_amd as sz

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak

WORKLOADS = {
    "config1": "Llama-3-8B-shaped BF16 KV cache: 32 layers x {K,V} x [32768,8,128] (4 GiB), one codebook per kind",
    "config0": "single BF16 K tensor [4096,8,128] (8 MiB, cache resident)",
    "config2": "escape stress: 8 x BF16 [16384,8,128] with 0.5 % outliers and 0.1 % zeros/subnormals",
    "config3": "streaming prefill chunks, Llama-3-70B shape: BF16 [2048,8,128] K and V per layer (4 MiB calls)",
    "config4": "FP8 E5M2 KV cache: 32 layers x {K,V} x [32768,8,128] (2 GiB), one codebook per kind",
}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=10)
    p.add_argument("--warmup", type=int, default=2)
    p.add_argument("--workload", default="config1", choices=sorted(WORKLOADS))
    p.add_argument("--layers", type=int, default=0, help="layers of the KV cache (default: the workload's own)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-variants", action="store_true", help="skip the format variants of the ablations")
    p.add_argument("--no-others", action="store_true", help="skip the other workloads and the copy ceiling")
    p.add_argument("--cpu-sample-mib", type=int, default=1024, help="bytes of the workload the oracle is timed on")
    return p.parse_args()


def build_workload(w, layers=0):
    """[(kind, device tensor of raw words)], {kind: codebook}, dtype"""
    dev = "cuda"
    if w == "config0":
        return [("K", kv_synth.kv_bf16(4096, 0, 0, "K", dev))], {"K": sz.calibrate(kv_synth.kv_bf16(4096, 1, 0, "K"), sz.BF16)}, sz.BF16
    if w == "config2":
        xs = [("K", kv_synth.kv_bf16_outliers(16384, 0, layer, dev)) for layer in range(layers or 8)]
        return xs, {"K": sz.calibrate(kv_synth.kv_bf16(1024, 1, 0, "K"), sz.BF16)}, sz.BF16     # outlier-free calibration
    dtype = sz.FP8_E5M2 if w == "config4" else sz.BF16
    gen = kv_synth.kv_e5m2 if dtype == sz.FP8_E5M2 else kv_synth.kv_bf16
    layers = layers or (80 if w == "config3" else 32)
    tokens = 2048 if w == "config3" else 32768
    xs = [(kind, gen(tokens, 0, layer, kind, dev)) for layer in range(layers) for kind in ("K", "V")]
    # one codebook per tensor kind from a seed-1 sample of 1024 tokens spread over the layers
    per = max(1, 1024 // layers)
    cbs = {kind: sz.calibrate(torch.cat([gen(per, 1, layer, kind) for layer in range(layers)]), dtype) for kind in ("K", "V")}
    return xs, cbs, dtype


def measured_traffic(workload, kernel):
    """(HBM bytes per launch of `kernel`, the file they come from): from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE + WRITE_SIZE runs of this same script, scaled by a plain copy kernel), or (None, None)."""
    import glob
    import re

    here = os.path.dirname(os.path.abspath(__file__))
    for path in sorted(glob.glob(os.path.join(here, "profiles", "*hbm_counters*"))):
        for line in open(path):
            m = re.search(r'traffic_bytes_per_launch workload=(\S+) kernel="([^"]+)" bytes=(\d+)', line)
            if m and m.group(1) == workload and m.group(2) == kernel:
                return int(m.group(3)), "profiles/" + os.path.basename(path)
    return None, None


def ev():
    return torch.cuda.Event(enable_timing=True)


def mean(v):
    return sum(v) / len(v)


def std(v):
    m = mean(v)
    return (sum((x - m) ** 2 for x in v) / len(v)) ** 0.5


def fmt_of(dtype):
    return "Bf16" if dtype == sz.BF16 else "E5m2"


def compress_kernels(dtype):
    f = fmt_of(dtype)
    return f"compress_tile_kernel<{f}, {2 if dtype == sz.BF16 else 4}> + compress_finish_kernel<{f}>"


class Workload:
    """A workload resident on the device with everything a pass needs; verify() checks the round trip and that batch
    and single calls give the same streams."""

    def __init__(self, name, layers=0):
        self.name = name
        self.xs, cbs, self.dtype = build_workload(name, layers)
        self.es = 2 if self.dtype == sz.BF16 else 1
        self.n = self.xs[0][1].numel()
        self.nt = len(self.xs)
        self.raw_bytes = self.n * self.es
        self.total_raw = self.raw_bytes * self.nt
        # stream capacity: the fixed part plus room for 3 % escapes
        self.cap = (sz.total_bytes(self.n, self.n * 3 // 100, self.dtype) + 255) // 256 * 256
        self.comps = [torch.empty(self.cap, dtype=torch.uint8, device="cuda") for _ in range(self.nt)]
        self.outs = [torch.empty_like(x) for _, x in self.xs]
        self.books = [cbs[kind] for kind, _ in self.xs]
        self.rec = sz.new_sizes_array(self.nt)
        self.dsizes = sz.new_sizes()
        self.ws = sz.Workspace(self.n, self.dtype)
        self.cbatch = sz.CompressBatch([x for _, x in self.xs], self.books, self.comps)
        self.sizes1 = [sz.new_sizes() for _ in range(self.nt)]
        torch.cuda.synchronize()

    def verify(self):
        self.cbatch.launch(self.ws, self.rec)
        torch.cuda.synchronize()
        self.got = sz.read_sizes_array(self.rec)
        assert all(g[2] == 0 for g in self.got), f"compress status {self.got}"
        self.totals = [g[0] for g in self.got]
        self.escapes = sum(g[1] for g in self.got)
        self.blob_bytes = sum(self.totals)
        self.dbatch = sz.DecompressBatch(self.comps, self.totals, [self.n] * self.nt, self.books, self.outs)
        self.dbatch.launch(self.dsizes)
        torch.cuda.synchronize()
        assert sz.read_sizes(self.dsizes)[2] == 0, "decompress flagged a bad stream"
        for (kind, x), y in zip(self.xs, self.outs):
            assert torch.equal(x, y), "round trip is not bit exact"
        one = sz.new_sizes()
        probe_out = torch.empty(self.cap, dtype=torch.uint8, device="cuda")
        for i in (0, self.nt - 1):
            sz.compress(self.xs[i][1], self.books[i], probe_out, self.ws, one)
            torch.cuda.synchronize()
            assert sz.read_sizes(one) == self.got[i] and torch.equal(probe_out[: self.totals[i]], self.comps[i][: self.totals[i]]), \
                "batch and single call disagree"
        # algorithmic traffic of one pass: read the words, write the streams (and the reverse)
        self.alg_bytes = self.total_raw + self.blob_bytes
        self.ratio = self.total_raw / self.blob_bytes

    def time_steps(self, steps, warmup):
        """K steps of (compress batch, decompress batch); events on the launch stream.  -> ms lists, ms per step (host clock)"""
        for _ in range(warmup):
            self.cbatch.launch(self.ws, self.rec)
            self.dbatch.launch(self.dsizes)
        torch.cuda.synchronize()
        marks = []
        wall0 = time.perf_counter()
        for _ in range(steps):
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            self.cbatch.launch(self.ws, self.rec)
            e1.record()
            self.dbatch.launch(self.dsizes)
            e2.record()
            marks.append((e0, e1, e2))
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        return [a.elapsed_time(b) for a, b, _ in marks], [b.elapsed_time(c) for _, b, c in marks], wall / steps * 1e3

    def compress_each(self, stream=None, wss=None):
        for i, (kind, x) in enumerate(self.xs):
            sz.compress(x, self.books[i], self.comps[i], self.ws if wss is None else wss[i & 1], self.sizes1[i],
                        stream=None if stream is None else stream[i & 1])

    def decompress_each(self, stream=None):
        for i in range(self.nt):
            sz.decompress(self.comps[i], self.totals[i], self.n, self.books[i], self.outs[i], self.dsizes,
                          stream=None if stream is None else stream[i & 1])

    def time_single_calls(self, reps):
        """the same pass, one call per tensor on one stream; HIP events -> us per call, both ways"""
        self.compress_each()
        self.decompress_each()
        torch.cuda.synchronize()
        f0, f1, f2 = ev(), ev(), ev()
        f0.record()
        for _ in range(reps):
            self.compress_each()
        f1.record()
        for _ in range(reps):
            self.decompress_each()
        f2.record()
        torch.cuda.synchronize()
        return f0.elapsed_time(f1) * 1e3 / reps / self.nt, f1.elapsed_time(f2) * 1e3 / reps / self.nt

    def time_two_streams(self, reps):
        """the per-tensor calls alternating over two streams, each with its own workspace (host clock, whole pass)"""
        streams2 = [torch.cuda.Stream(), torch.cuda.Stream()]
        ws2 = [self.ws, sz.Workspace(self.n, self.dtype)]
        torch.cuda.synchronize()
        two = []
        for f in (lambda: self.compress_each(streams2, ws2), lambda: self.decompress_each(streams2)):
            f()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                f()
            torch.cuda.synchronize()
            two.append((time.perf_counter() - t0) * 1e6 / reps / self.nt)
        assert all(sz.read_sizes(self.sizes1[i]) == self.got[i] for i in range(self.nt)), "two-stream compress differs"
        return two

    def summary(self, ms_c, ms_d, c1_us, d1_us):
        """the figures every workload reports"""
        launches = (self.nt + 63) // 64      # a batch call takes 64 tensors per pair of launches
        alg1 = self.alg_bytes / self.nt
        f = fmt_of(self.dtype)
        return {
            "workload": f"{self.name}: {WORKLOADS[self.name]}", "dtype": "u16" if self.dtype == sz.BF16 else "u8",
            "tensors": self.nt, "elems_per_tensor": self.n, "uncompressed_bytes": self.total_raw,
            "ratio": round(self.ratio, 4), "escape_rate": round(self.escapes / (self.n * self.nt), 6),
            "batch_calls": {
                "compress_GBps": round(self.total_raw / (mean(ms_c) * 1e-3) / 1e9, 1),
                "decompress_GBps": round(self.total_raw / (mean(ms_d) * 1e-3) / 1e9, 1),
                "compress_us": round(mean(ms_c) * 1e3, 2), "decompress_us": round(mean(ms_d) * 1e3, 2),
                "compress_frac_of_peak": round(self.alg_bytes / (mean(ms_c) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "decompress_frac_of_peak": round(self.alg_bytes / (mean(ms_d) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "calls_per_pass": launches,
                "kernels": [compress_kernels(self.dtype), f"decompress_batch_kernel<D{f}>"],
            },
            "per_tensor_calls": {
                "compress_GBps": round(self.raw_bytes / c1_us * 1e-3, 1), "compress_us": round(c1_us, 2),
                "compress_frac_of_peak": round(alg1 / c1_us * 1e-3 / HBM_PEAK_GBPS, 4),
                "decompress_GBps": round(self.raw_bytes / d1_us * 1e-3, 1), "decompress_us": round(d1_us, 2),
                "decompress_frac_of_peak": round(alg1 / d1_us * 1e-3 / HBM_PEAK_GBPS, 4),
                "algorithmic_bytes_per_call": int(alg1),
                "kernels": [compress_kernels(self.dtype), f"decompress_kernel<D{f}>"],
                "how": "one call per tensor, back to back on one stream; HIP events around the pass",
            },
        }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the codec has no cross-GPU step and this build uses one device "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    W = Workload(args.workload, args.layers)
    W.verify()
    xs, dtype, n, nt, es, books, comps, outs, ws = W.xs, W.dtype, W.n, W.nt, W.es, W.books, W.comps, W.outs, W.ws
    raw_bytes, total_raw, totals, got, cap = W.raw_bytes, W.total_raw, W.totals, W.got, W.cap

    # ---- the timed region: K steps of (compress batch, decompress batch)
    ms_c, ms_d, ms_step = W.time_steps(args.steps, args.warmup)
    comp_gbps = total_raw / (mean(ms_c) * 1e-3) / 1e9
    dec_gbps = total_raw / (mean(ms_d) * 1e-3) / 1e9
    alg_bytes = W.alg_bytes
    c_ach = alg_bytes / (mean(ms_c) * 1e-3) / 1e9
    d_ach = alg_bytes / (mean(ms_d) * 1e-3) / 1e9
    launches = (nt + 63) // 64

    # ---- the same pass, one call per tensor
    reps = max(2, args.steps // 2)
    c1_us, d1_us = W.time_single_calls(reps)
    two = W.time_two_streams(reps)
    summ = W.summary(ms_c, ms_d, c1_us, d1_us)
    alg1 = alg_bytes / nt

    # ---- plain streaming kernel with the codec's traffic (same bytes read and written per tensor, no arithmetic)
    wbytes = (W.blob_bytes // nt) // 16 * 16
    wbytes = min(wbytes, outs[0].numel() * es)
    for i in range(nt):
        sz.traffic_probe(xs[i][1], raw_bytes, outs[i], wbytes)
    p0, p1 = ev(), ev()
    p0.record()
    for _ in range(3):
        for i in range(nt):
            sz.traffic_probe(xs[i][1], raw_bytes, outs[i], wbytes)
    p1.record()
    torch.cuda.synchronize()
    probe_gbps = (raw_bytes + wbytes) * nt * 3 / (p0.elapsed_time(p1) * 1e-3) / 1e9

    # ---- calibration per call ("dynamic codebook", the paper's pre-calibration ablation): device histogram of the
    # tensor itself, 2 KB to the host, ranking on the host, then the ordinary compress call
    one = sz.new_sizes()
    probe_out = torch.empty(cap, dtype=torch.uint8, device="cuda")
    kdyn = min(nt, 16)
    hist = torch.zeros(256, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(kdyn):
        hist.zero_()
        sz.histogram(xs[i][1], dtype, hist)
        cb_dyn = sz.codebook_from_hist(hist.cpu(), dtype)          # the copy waits for the histogram
        sz.compress(xs[i][1], cb_dyn, probe_out, ws, one)
    torch.cuda.synchronize()
    dyn_us = (time.perf_counter() - t0) * 1e6 / kdyn
    h0, h1, h2 = ev(), ev(), ev()
    h0.record()
    for i in range(kdyn):
        sz.histogram(xs[i][1], dtype, hist)
    h1.record()
    # the same with the codebook staying on the device: nothing waits for the host
    dcb = sz.DeviceCodebook(dtype)
    for i in range(kdyn):
        hist.zero_()
        sz.histogram(xs[i][1], dtype, hist)
        sz.codebook_device(hist, dtype, dcb)
        sz.compress_dcb(xs[i][1], dcb, probe_out, ws, one)
    h2.record()
    torch.cuda.synchronize()
    hist_us = h0.elapsed_time(h1) * 1e3 / kdyn
    dyn_dev_us = h1.elapsed_time(h2) * 1e3 / kdyn
    # the whole cache at once: every tensor's own codebook counted and ranked on the device (three launches per 64
    # tensors), then one batch call under those codebooks
    dcbs = sz.DeviceCodebooks(nt, dtype)
    cal = sz.CalibrateBatchDevice([x for _, x in xs], dcbs)
    cdyn = sz.CompressBatchDcb([x for _, x in xs], dcbs, comps)
    rec_dyn = sz.new_sizes_array(nt)
    cal.launch()
    cdyn.launch(ws, rec_dyn)
    torch.cuda.synchronize()
    got_dyn = sz.read_sizes_array(rec_dyn)
    assert all(g[2] == 0 for g in got_dyn)
    b0, b1, b2 = ev(), ev(), ev()
    b0.record()
    for _ in range(3):
        cal.launch()
    b1.record()
    for _ in range(3):
        cdyn.launch(ws, rec_dyn)
    b2.record()
    torch.cuda.synchronize()
    cal_us, cdyn_us = b0.elapsed_time(b1) * 1e3 / 3 / nt, b1.elapsed_time(b2) * 1e3 / 3 / nt
    W.cbatch.launch(ws, W.rec)          # the pre-calibrated streams again, for what follows
    torch.cuda.synchronize()

    fmt = fmt_of(dtype)
    ratio = W.ratio
    ck = compress_kernels(dtype)
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
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", "tensors": nt, "elems_per_tensor": n,
                   "uncompressed_bytes": total_raw, "calls_per_step": 2 * launches},
        "compress_GBps": round(comp_gbps, 1),
        "compress_GBps_std": round(std([total_raw / (m * 1e-3) / 1e9 for m in ms_c]), 1),
        "decompress_GBps": round(dec_gbps, 1),
        "decompress_GBps_std": round(std([total_raw / (m * 1e-3) / 1e9 for m in ms_d]), 1),
        "ratio": round(ratio, 4),
        "escape_rate": round(W.escapes / (n * nt), 6),
        "B_hide_GBps": round(min(comp_gbps, dec_gbps) / ratio, 1),
        "paper_context": {"compress_GBps": 613.3, "decompress_GBps": 2181.8, "ratio": 1.324,
                          "hardware": "NVIDIA H200, real Qwen3-32B BF16 KV (Table 2)"},
        "roofline": {
            "kernel": ck, "what": "one splitzip_compress_batch call over the whole workload: its two launches, timed together",
            "bound": "hbm", "achieved": round(c_ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(c_ach / HBM_PEAK_GBPS, 4), "traffic": None, "traffic_source": None,
            "launch_us": round(mean(ms_c) * 1e3 / launches, 2), "algorithmic_bytes_per_launch": int(alg_bytes / launches),
        },
        "roofline_decompress": {
            "kernel": f"decompress_batch_kernel<D{fmt}>",
            "bound": "hbm", "achieved": round(d_ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(d_ach / HBM_PEAK_GBPS, 4), "traffic": None, "traffic_source": None,
            "launch_us": round(mean(ms_d) * 1e3 / launches, 2), "algorithmic_bytes_per_launch": int(alg_bytes / launches),
        },
        "roofline_single_calls": {
            "what": "splitzip_compress / splitzip_decompress, one tensor per call, back to back on one stream",
            "compress": {"kernel": ck, "bound": "hbm", "achieved": round(alg1 / c1_us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(alg1 / c1_us * 1e-3 / HBM_PEAK_GBPS, 4), "launch_us": round(c1_us, 2), "algorithmic_bytes_per_launch": int(alg1)},
            "decompress": {"kernel": f"decompress_kernel<D{fmt}>", "bound": "hbm", "achieved": round(alg1 / d1_us * 1e-3, 1), "peak": HBM_PEAK_GBPS,
                           "unit": "GB/s", "frac": round(alg1 / d1_us * 1e-3 / HBM_PEAK_GBPS, 4), "launch_us": round(d1_us, 2),
                           "algorithmic_bytes_per_launch": int(alg1)},
        },
        "per_tensor_calls": dict(summ["per_tensor_calls"], two_streams={
            "compress_GBps": round(raw_bytes / two[0] * 1e-3, 1), "compress_us": round(two[0], 2),
            "compress_frac_of_peak": round(alg1 / two[0] * 1e-3 / HBM_PEAK_GBPS, 4),
            "decompress_GBps": round(raw_bytes / two[1] * 1e-3, 1), "decompress_us": round(two[1], 2),
            "decompress_frac_of_peak": round(alg1 / two[1] * 1e-3 / HBM_PEAK_GBPS, 4),
            "how": "the same calls alternating over two streams, a workspace each; host clock over the pass"}),
        "copy_kernel_same_traffic_GBps": round(probe_gbps, 1),
        "dynamic_codebook": {
            "compress_GBps": round(raw_bytes / dyn_us * 1e-3, 1), "us_per_tensor": round(dyn_us, 2),
            "on_device_compress_GBps": round(raw_bytes / dyn_dev_us * 1e-3, 1), "on_device_us_per_tensor": round(dyn_dev_us, 2),
            "histogram_us": round(hist_us, 2), "histogram_GBps": round(raw_bytes / hist_us * 1e-3, 1),
            "batch_on_device_compress_GBps": round(raw_bytes / (cal_us + cdyn_us) * 1e-3, 1),
            "batch_on_device_us_per_tensor": round(cal_us + cdyn_us, 2), "batch_calibrate_us_per_tensor": round(cal_us, 2),
            "batch_escape_rate": round(sum(g[1] for g in got_dyn) / (n * nt), 6),
            "how": "per tensor: device histogram, 2 KB copy + ranking on the host (synchronises), compress call; host clock. "
                   "on_device: histogram, ranking and compress with a codebook in device memory, no host round trip; HIP events. "
                   "batch_on_device: all tensors at once, each under a codebook counted from itself (calibrate batch: three "
                   "launches per 64 tensors; compress batch under the device codebooks); HIP events",
            "paper_context_GBps": 80.7,
        },
        "pipeline_model": pipeline_model(raw_bytes, comp_gbps, dec_gbps, ratio),
    }
    if not args.layers:     # the counter summaries were taken at the workload's own size
        for key in ("roofline", "roofline_decompress"):
            result[key]["traffic"], result[key]["traffic_source"] = measured_traffic(args.workload, result[key]["kernel"])
            t = result[key]["traffic"]
            if t is not None and abs(t / result[key]["algorithmic_bytes_per_launch"] - 1.0) > 0.05:
                result[key]["traffic_note"] = "the committed counter figure is more than 5 % off this run's algorithmic bytes: stale or wasteful"

    result["paged"] = paged_calls(dtype, xs[0][1], books[0], ws, c1_us, d1_us)
    if args.workload in ("config1", "config3", "config4"):
        result["per_layer_codebooks"] = per_layer_codebooks(args, dtype, xs, ws, cap, got, comp_gbps, dec_gbps)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(W, args.cpu_sample_mib)
    # the headline workload leaves the device before the others are built
    del W, xs, books, comps, outs, ws, cal, cdyn, dcbs, probe_out
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_variants:
        result["format_variants"] = format_variants()
    if not args.no_others:
        others = {}
        for name in ("config0", "config2", "config3", "config4"):
            if name == args.workload:
                continue
            others[name] = other_workload(name, args)
            gc.collect()
            torch.cuda.empty_cache()
        if args.workload != "config1":
            others["config1"] = other_workload("config1", args)
        result["other_workloads"] = others
        result["copy_ceiling"] = copy_ceiling()
    print(json.dumps(result))


def other_workload(name, args):
    """one of the workloads that is not the headline: the same measurements, fewer steps, and for config 3 the timing
    of the streaming calls; with the oracle timed on a sample of it where the plan of the CPU baseline asks for one"""
    W = Workload(name)
    W.verify()
    steps = max(3, args.steps // 2)
    ms_c, ms_d, _ = W.time_steps(steps, 1)
    c1_us, d1_us = W.time_single_calls(2 if W.nt >= 64 else 5)
    rec = W.summary(ms_c, ms_d, c1_us, d1_us)
    if name == "config3":
        rec["streaming"] = streaming_calls(W)
    if not args.no_cpu_baseline and name in ("config0", "config4"):
        rec["cpu_baseline"] = cpu_baseline(W, args.cpu_sample_mib)
    return rec


def streaming_calls(W, positions=64):
    """Config 3 at its stated extent: 80 layers x {K, V} x 64 chunk positions = 10 240 calls of 4 MiB.  The 160 tensors
    of one chunk position (640 MiB, more than the last-level cache holds) serve as the ring that the 64 positions
    cycle through.  Three ways: (a) eager single calls, every call between two events on the stream (per-call
    latency as the device sees it) and a subset between host clocks with a synchronise (as a caller sees it);
    (b) one batch call per chunk position (three pairs of launches for 160 tensors); (c) the batch calls of one chunk
    position captured in a HIP graph and replayed per position."""
    nt, n = W.nt, W.n
    calls = nt * positions
    out = {"calls": calls, "positions": positions, "tensors_per_position": nt, "bytes_per_call": W.raw_bytes}

    def pct(ts, q):
        ts = sorted(ts)
        return round(ts[min(len(ts) - 1, int(len(ts) * q))], 2)

    # (a) eager single calls
    for name, call in (("compress", lambda i: sz.compress(W.xs[i][1], W.books[i], W.comps[i], W.ws, W.sizes1[i])),
                       ("decompress", lambda i: sz.decompress(W.comps[i], W.totals[i], n, W.books[i], W.outs[i], W.dsizes))):
        for i in range(nt):
            call(i)
        torch.cuda.synchronize()
        evs = [ev() for _ in range(calls + 1)]
        t0 = time.perf_counter()
        evs[0].record()
        for p in range(positions):
            for i in range(nt):
                call(i)
                evs[p * nt + i + 1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        dev_us = [evs[k].elapsed_time(evs[k + 1]) * 1e3 for k in range(calls)]
        host_us = []
        for i in range(nt):                                    # one position, every call awaited
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            call(i)
            torch.cuda.synchronize()
            host_us.append((time.perf_counter() - t1) * 1e6)
        out[name] = {
            "aggregate_GBps": round(W.raw_bytes * calls / wall / 1e9, 1), "us_per_call_enqueued": round(wall * 1e6 / calls, 2),
            "device_p50_us": pct(dev_us, 0.5), "device_p99_us": pct(dev_us, 0.99),
            "host_p50_us": pct(host_us, 0.5), "host_p99_us": pct(host_us, 0.99), "host_calls": len(host_us),
            "how": "10 240 calls back to back on one stream, host clock over all of them; device_*: between the events recorded "
                   "behind consecutive calls; host_*: host clock around one call plus a stream synchronise",
        }
    # (b) one batch call per chunk position
    for _ in range(2):
        W.cbatch.launch(W.ws, W.rec)
        W.dbatch.launch(W.dsizes)
    e0, e1, e2 = ev(), ev(), ev()
    e0.record()
    for p in range(positions):
        W.cbatch.launch(W.ws, W.rec)
    e1.record()
    for p in range(positions):
        W.dbatch.launch(W.dsizes)
    e2.record()
    torch.cuda.synchronize()
    out["batch_per_position"] = {
        "compress_GBps": round(W.total_raw * positions / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1),
        "decompress_GBps": round(W.total_raw * positions / (e1.elapsed_time(e2) * 1e-3) / 1e9, 1),
        "compress_us_per_position": round(e0.elapsed_time(e1) * 1e3 / positions, 1),
        "decompress_us_per_position": round(e1.elapsed_time(e2) * 1e3 / positions, 1),
        "how": "splitzip_compress_batch / _decompress_batch over the 160 tensors of a position; HIP events over 64 positions",
    }
    # (c) a captured graph of one position, replayed (the library records no memset nodes; every replay is checked below)
    stream = torch.cuda.Stream()
    graphs = {}
    with torch.cuda.stream(stream):
        for name, launch in (("compress", lambda: W.cbatch.launch(W.ws, W.rec, stream)), ("decompress", lambda: W.dbatch.launch(W.dsizes, stream))):
            launch()
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                launch()
            graphs[name] = g
        stream.synchronize()
        res = {}
        for name, g in graphs.items():
            g.replay()
            stream.synchronize()
            t0 = time.perf_counter()
            for p in range(positions):
                g.replay()
            stream.synchronize()
            res[name] = (time.perf_counter() - t0) / positions
    torch.cuda.synchronize()
    assert sz.read_sizes_array(W.rec) == W.got and all(torch.equal(x, y) for (_, x), y in zip(W.xs, W.outs)), "graph replay differs"
    out["graph_replay_per_position"] = {
        "compress_GBps": round(W.total_raw / res["compress"] / 1e9, 1), "decompress_GBps": round(W.total_raw / res["decompress"] / 1e9, 1),
        "compress_us_per_position": round(res["compress"] * 1e6, 1), "decompress_us_per_position": round(res["decompress"] * 1e6, 1),
        "how": "the batch calls of one position captured in a HIP graph each and replayed 64 times; host clock; results "
               "compared with the eager calls' after the replays",
    }
    return out


def copy_ceiling():
    """the best plain streaming kernels of this GPU per traffic mix: a handful of settings of
    splitzip_traffic_probe_shape (python -m paper_2605_01708_amd.hbm_ceiling sweeps all of them)"""
    from paper_2605_01708_amd.hbm_ceiling import time_shape

    unit = (2 << 30) // (48 * 4096) * (48 * 4096)
    src = torch.empty(unit, dtype=torch.uint8, device="cuda")
    dst = torch.empty(unit, dtype=torch.uint8, device="cuda")
    src.random_(0, 256)
    torch.cuda.synchronize()
    out = {"how": "read + written GB/s of plain kernels moving 2 GiB on the larger side, the best of a few shapes per mix: "
                  "reads x writes 4 KB runs per workgroup and step; wgs_per_cu 0 = one workgroup per step, started by the "
                  "hardware in order; non-temporal accesses", "peak_GBps": HBM_PEAK_GBPS}
    mixes = (("read_only", ((8, 0),)), ("write_only", ((0, 1), (0, 8))), ("compress_4_3", ((4, 3), (16, 12))),
             ("decompress_3_4", ((3, 4), (12, 16))), ("copy_1_1", ((1, 1), (4, 4))))
    for mix, shapes in mixes:
        best = None
        for r, w in shapes:
            rb = unit if r >= w else unit // w * r
            wb = unit if w >= r else unit // r * w
            for wgs in (0, 1, 4):
                flags = (1 if r else 0) | (2 if w else 0)
                g = time_shape(src, dst, rb, wb, r, w, wgs, flags, 3)
                if best is None or g > best[0]:
                    best = (g, wgs, r, w)
        out[mix] = {"GBps": round(best[0], 1), "frac": round(best[0] / HBM_PEAK_GBPS, 4), "reads": best[2], "writes": best[3],
                    "wgs_per_cu": best[1]}
    return out


def per_layer_codebooks(args, dtype, xs, ws, cap, shared, shared_c_gbps, shared_d_gbps, reps=5):
    """The batch calls with one codebook per tensor instead of one per kind (the section "Ablation on Layer-Wise
    Coverage" names per-layer codebooks as the way to remove the low-coverage tail of a shared one): each tensor's
    codebook comes from a seed-1 sample of 1024 tokens of its own layer and kind, counted on the device."""
    gen = kv_synth.kv_e5m2 if dtype == sz.FP8_E5M2 else kv_synth.kv_bf16
    nt, n = len(xs), xs[0][1].numel()
    es = 2 if dtype == sz.BF16 else 1
    hist = torch.zeros(256, dtype=torch.int64, device="cuda")
    books = []
    for i, (kind, _) in enumerate(xs):
        hist.zero_()
        sz.histogram(gen(1024, 1, i // 2, kind, "cuda"), dtype, hist)
        books.append(sz.codebook_from_hist(hist.cpu(), dtype))
    comps = [torch.empty(cap, dtype=torch.uint8, device="cuda") for _ in range(nt)]
    outs = [torch.empty_like(x) for _, x in xs]
    rec, dsz = sz.new_sizes_array(nt), sz.new_sizes()
    cb = sz.CompressBatch([x for _, x in xs], books, comps)
    cb.launch(ws, rec)
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    assert all(g[2] == 0 for g in got)
    db = sz.DecompressBatch(comps, [g[0] for g in got], [n] * nt, books, outs)
    db.launch(dsz)
    torch.cuda.synchronize()
    assert sz.read_sizes(dsz)[2] == 0 and all(torch.equal(x, y) for (_, x), y in zip(xs, outs)), "round trip is not bit exact"
    e0, e1, e2 = ev(), ev(), ev()
    e0.record()
    for _ in range(reps):
        cb.launch(ws, rec)
    e1.record()
    for _ in range(reps):
        db.launch(dsz)
    e2.record()
    torch.cuda.synchronize()
    raw = n * es * nt
    return {
        "how": "one codebook per tensor (seed-1 sample of its own layer and kind), all in the same batch launches",
        "codebooks": len({tuple(b.dec) for b in books}),
        "escape_rate": round(sum(g[1] for g in got) / (n * nt), 6), "shared_escape_rate": round(sum(g[1] for g in shared) / (n * nt), 6),
        "worst_tensor_escape_rate": round(max(g[1] for g in got) / n, 6),
        "shared_worst_tensor_escape_rate": round(max(g[1] for g in shared) / n, 6),
        "ratio": round(raw / sum(g[0] for g in got), 4), "shared_ratio": round(raw / sum(g[0] for g in shared), 4),
        "compress_GBps": round(raw * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1), "shared_compress_GBps": round(shared_c_gbps, 1),
        "decompress_GBps": round(raw * reps / (e1.elapsed_time(e2) * 1e-3) / 1e9, 1), "shared_decompress_GBps": round(shared_d_gbps, 1),
    }


def paged_calls(dtype, x, cb, ws, c_contig_us, d_contig_us, block_tokens=16, reps=10):
    """splitzip_compress_paged / _decompress_paged on the workload's first tensor, held in a pool of shuffled pages
    of block_tokens tokens each (the layout of a paged KV cache); the stream must equal the contiguous call's."""
    n, es = x.numel(), x.element_size()
    be = block_tokens * 1024
    n_blocks = (n + be - 1) // be
    stride = be * es
    perm = torch.randperm(n_blocks, generator=torch.Generator().manual_seed(7)).to(torch.int32)
    pool = torch.empty(n_blocks * be, dtype=x.dtype, device="cuda")
    padded = torch.zeros(n_blocks * be, dtype=x.dtype, device="cuda")
    padded[:n] = x
    pool.view(n_blocks, be)[perm.long().cuda()] = padded.view(n_blocks, be)
    table = perm.cuda()
    src = sz.Paged(pool, table, be, stride, 0, n_blocks)
    cap = (sz.total_bytes(n, n * 3 // 100, dtype) + 255) // 256 * 256
    out_p = torch.empty(cap, dtype=torch.uint8, device="cuda")
    out_c = torch.empty(cap, dtype=torch.uint8, device="cuda")
    rec = sz.new_sizes()
    sz.compress_paged(src, n, cb, out_p, ws, rec)
    sz.compress(x, cb, out_c, ws, rec)
    torch.cuda.synchronize()
    total = sz.read_sizes(rec)[0]
    assert torch.equal(out_p[:total], out_c[:total]), "paged stream differs from the contiguous one"
    pool2 = torch.zeros_like(pool)
    dst = sz.Paged(pool2, table, be, stride, 0, n_blocks)
    sz.decompress_paged(out_p, total, n, cb, dst)
    torch.cuda.synchronize()
    assert torch.equal(pool2, pool), "paged round trip differs"
    e0, e1, e2 = ev(), ev(), ev()
    e0.record()
    for _ in range(reps):
        sz.compress_paged(src, n, cb, out_p, ws, rec)
    e1.record()
    for _ in range(reps):
        sz.decompress_paged(out_p, total, n, cb, dst)
    e2.record()
    torch.cuda.synchronize()
    c_us, d_us = e0.elapsed_time(e1) * 1e3 / reps, e1.elapsed_time(e2) * 1e3 / reps
    return {"how": f"one tensor in a pool of {n_blocks} shuffled pages of {block_tokens} tokens, one call each way",
            "compress_GBps": round(n * es / c_us * 1e-3, 1), "decompress_GBps": round(n * es / d_us * 1e-3, 1),
            "contiguous_compress_GBps": round(n * es / c_contig_us * 1e-3, 1),
            "contiguous_decompress_GBps": round(n * es / d_contig_us * 1e-3, 1)}


def format_variants(tokens=32768, reps=10):
    """The formats of the paper's ablations (top-k, escape-position metadata, chunk size, FP8) side by side, each
    through the same generic kernels (splitzip_variant_*), on one K tensor of [tokens, 8, 128] of each word type,
    codebooks calibrated on a separate 1024-token sample.  Round trip checked before timing; HIP events."""
    rows = []
    gens = {sz.BF16: kv_synth.kv_bf16, sz.FP8_E5M2: kv_synth.kv_e5m2, sz.FP8_E4M3: kv_synth.kv_e4m3}
    names = {sz.BF16: "bf16", sz.FP8_E5M2: "e5m2", sz.FP8_E4M3: "e4m3"}
    table = [(sz.BF16, 4, 16, sz.ESC_POS, 1024, "top-16, 16-bit chunk-relative positions (the main format)"),
             (sz.BF16, 4, 15, sz.ESC_SENTINEL, 1024, "top-15 + sentinel, no positions"),
             (sz.BF16, 3, 8, sz.ESC_POS, 1024, "top-8, 3-bit codes"),
             (sz.BF16, 4, 16, sz.ESC_POS, 256, "chunk 256, 8-bit positions"),
             (sz.BF16, 4, 16, sz.ESC_ABS32, 0, "32-bit absolute positions, no chunks"),
             (sz.FP8_E5M2, 4, 16, sz.ESC_POS, 1024, "E5M2 top-16"),
             (sz.FP8_E5M2, 3, 8, sz.ESC_POS, 1024, "E5M2 top-8"),
             (sz.FP8_E4M3, 3, 8, sz.ESC_POS, 1024, "E4M3 top-8")]
    data = {}
    for dt, bits, k, mode, chunk, what in table:
        if dt not in data:
            data[dt] = (gens[dt](tokens, 0, 0, "K", device="cuda"), gens[dt](1024, 1, 0, "K"))
        x, sample = data[dt]
        n, es = x.numel(), x.element_size()
        v = sz.variant(dt, bits, k, mode, chunk)
        cb = sz.variant_calibrate(sample, v)
        out = torch.empty(sz.variant_total_bytes(n, n // 5, v), dtype=torch.uint8, device="cuda")
        wsp = torch.empty(sz.variant_workspace_bytes(n, v), dtype=torch.uint8, device="cuda")
        rec, st = sz.new_sizes(), sz.new_sizes()
        y = torch.empty_like(x)
        sz.variant_compress(x, v, cb, out, wsp, rec)
        torch.cuda.synchronize()
        total, m, status = sz.read_sizes(rec)
        assert status == 0, (what, status)
        sz.variant_decompress(out, total, n, v, cb, y, st)
        torch.cuda.synchronize()
        assert sz.read_sizes(st)[2] == 0 and torch.equal(x, y), what
        for _ in range(3):                       # warm: the first format measured would otherwise pay the ramp of the clocks
            sz.variant_compress(x, v, cb, out, wsp, rec)
            sz.variant_decompress(out, total, n, v, cb, y, st)
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        for _ in range(reps):
            sz.variant_compress(x, v, cb, out, wsp, rec)
        e1.record()
        for _ in range(reps):
            sz.variant_decompress(out, total, n, v, cb, y, st)
        e2.record()
        torch.cuda.synchronize()
        c_us, d_us = e0.elapsed_time(e1) * 1e3 / reps, e1.elapsed_time(e2) * 1e3 / reps
        rows.append({"format": what, "words": names[dt], "code_bits": bits, "k": k,
                     "escape_rate": round(m / n, 5), "ratio": round(n * es / total, 4),
                     "compress_GBps": round(n * es / c_us * 1e-3, 1), "decompress_GBps": round(n * es / d_us * 1e-3, 1)})
    return {"how": "one [32768, 8, 128] K tensor per word type through the generic variant kernels (three or four launches per "
                   "compress, one or two per decompress); uncompressed GB/s; ratios count the whole stream",
            "paper_context": "Tables of the ablations (H200): top-8 440/711 GB/s ratio 1.241, top-15+sentinel 396/621 ratio 1.331, "
                             "main 613/2182 ratio 1.324; chunk 256 encodes at 351 GB/s; 32-bit absolute positions decode at 1422 GB/s",
            "rows": rows}


def pipeline_model(tensor_bytes, g_enc, g_dec, ratio):
    """The overlap model of the paper's appendix "The Potential of Hiding Codec Overhead with Pipeline Overlap"
    with this run's codec rates: per link, time of one tensor raw, additive (encode + transfer + decode) and
    pipelined (the slowest of the three stages), and B_hide = min(G_enc, G_dec) / ratio."""
    out = {"B_hide_GBps": round(min(g_enc, g_dec) / ratio, 1), "tensor_bytes": tensor_bytes, "links": {}}
    for name, gbps in (("nic_400Gb", 50.0), ("roce_4x200Gb_effective", 87.5), ("xgmi_link", 153.6)):
        t_raw = tensor_bytes / gbps * 1e-3
        t_enc, t_dec, t_x = tensor_bytes / g_enc * 1e-3, tensor_bytes / g_dec * 1e-3, tensor_bytes / ratio / gbps * 1e-3
        out["links"][name] = {"GBps": gbps, "raw_us": round(t_raw, 1), "additive_us": round(t_enc + t_x + t_dec, 1),
                              "pipelined_us": round(max(t_enc, t_x, t_dec), 1),
                              "speedup_pipelined": round(t_raw / max(t_enc, t_x, t_dec), 3)}
    return out


def cpu_baseline(W, sample_mib):
    """The oracle as it stands, one thread pinned to one core, on the first tensors of the workload (the whole of it
    if it is smaller than the sample); its streams are also compared with the GPU's (parity at full size)."""
    import numpy as np

    import oracle

    k = max(1, min(W.nt, (sample_mib << 20) // W.raw_bytes))
    odt = oracle.BF16 if W.dtype == sz.BF16 else oracle.E5M2
    before = os.sched_getaffinity(0)
    core = min(before)
    os.sched_setaffinity(0, {core})
    try:
        t_c = t_d = 0.0
        for i in range(k):
            xh = kv_synth.to_numpy_words(W.xs[i][1])
            cb = oracle.codebook_from_dec(np.array(W.books[i].dec, np.uint8), odt)
            t0 = time.perf_counter()
            blob, m = oracle.compress(xh, cb)
            t1 = time.perf_counter()
            y = oracle.decompress(blob, W.n, cb)
            t2 = time.perf_counter()
            t_c += t1 - t0
            t_d += t2 - t1
            assert np.array_equal(y, xh)
            assert np.array_equal(W.comps[i][: W.totals[i]].cpu().numpy(), blob), "GPU stream differs from the oracle's"
    finally:
        os.sched_setaffinity(0, before)
    raw = k * W.raw_bytes
    return {
        "value": round(2 * raw / (t_c + t_d) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{W.name}: first {k} of {W.nt} tensors ({raw / 2**20:.0f} MiB), compress+decompress, pinned to core {core}, "
                  "streams compared with the GPU's",
        "compress_GBps": round(raw / t_c / 1e9, 4), "decompress_GBps": round(raw / t_d / 1e9, 4),
        "host_cores_available": len(before), "host_cores_online": os.cpu_count(),
    }


if __name__ == "__main__":
    main()
