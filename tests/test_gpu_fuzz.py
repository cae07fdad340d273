"""Seeded random cases through every entry point of the library against the oracles: sizes anywhere between
nothing and a few hundred chunks, exponent laws from "one value" to "uniform over all", codebooks from perfect to
useless.  Bit-exact streams and round trips, as everywhere."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import variants as ov
import paper_2605_01708_amd as sz

pytestmark = pytest.mark.gpu

EXPS = {sz.BF16: 256, sz.FP8_E5M2: 32, sz.FP8_E4M3: 16}
# more seeds on request: SPLITZIP_FUZZ_ROUNDS=10 runs each test on ten consecutive seeds
ROUNDS = max(1, int(os.environ.get("SPLITZIP_FUZZ_ROUNDS", "1")))
ODT = {sz.BF16: oracle.BF16, sz.FP8_E5M2: oracle.E5M2}


def random_words(dt, n, rng):
    """exponents from one of several laws, random sign and mantissa"""
    ne = EXPS[dt]
    law = rng.integers(0, 5)
    if law == 0:      # tight cluster
        e = np.clip(np.rint(rng.normal(ne * 0.45, 1.2, n)), 0, ne - 1)
    elif law == 1:    # wide cluster: many escapes
        e = np.clip(np.rint(rng.normal(ne * 0.5, ne * 0.08 + 2, n)), 0, ne - 1)
    elif law == 2:    # uniform over everything
        e = rng.integers(0, ne, n)
    elif law == 3:    # a single value, with bursts of something else
        e = np.full(n, ne // 3)
        for _ in range(rng.integers(0, 4)):
            if n:
                a = rng.integers(0, n)
                e[a:a + rng.integers(1, 3000)] = rng.integers(0, ne)
    else:             # two values alternating in runs
        e = np.where((np.arange(n) // max(1, rng.integers(1, 700))) % 2 == 0, ne // 2, ne - 1)
    e = e.astype(np.uint32)
    if dt == sz.BF16:
        return ((rng.integers(0, 2, n).astype(np.uint32) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint32)).astype(np.uint16)
    if dt == sz.FP8_E5M2:
        return ((rng.integers(0, 2, n).astype(np.uint32) << 7) | (e << 2) | rng.integers(0, 4, n).astype(np.uint32)).astype(np.uint8)
    return ((rng.integers(0, 2, n).astype(np.uint32) << 7) | (e << 3) | rng.integers(0, 8, n).astype(np.uint32)).astype(np.uint8)


def random_size(rng):
    pick = rng.integers(0, 6)
    if pick == 0:
        return int(rng.integers(0, 20))
    if pick == 1:
        return int(rng.integers(1, 40)) * 1024 + int(rng.integers(-2, 3))
    return int(rng.integers(0, 300_000))


def dev(x):
    return torch.from_numpy(x.view(np.int16).copy() if x.dtype == np.uint16 else x.copy()).cuda()


@pytest.mark.parametrize("round_", range(ROUNDS))
def test_single_and_batch_calls_on_random_cases(round_):
    assert torch.cuda.is_available()
    rng = np.random.default_rng(20260501 + 1000 * round_)
    for dt in (sz.BF16, sz.FP8_E5M2):
        ws = sz.Workspace(400_000, dt)
        for case in range(12):
            k = int(rng.integers(1, 7))
            xs = [random_words(dt, random_size(rng), rng) for _ in range(k)]
            # a codebook per tensor: calibrated on one of the tensors, or on unrelated data
            cbs_or = [oracle.calibrate(xs[int(rng.integers(0, k))] if rng.integers(0, 2) else random_words(dt, 5000, rng), ODT[dt])
                      for _ in xs]
            cbs = [sz.codebook_from_dec(c.dec.tolist(), dt) for c in cbs_or]
            cb_or, cb = cbs_or[0], cbs[0]
            print(f"case fuzz dtype={dt} #{case}: sizes={[x.size for x in xs]}", flush=True)
            refs = [oracle.compress(x, c) for x, c in zip(xs, cbs_or)]
            xd = [dev(x) for x in xs]
            outs = [torch.full((sz.compress_bound(x.size, dt) + 512,), 0xA5, dtype=torch.uint8, device="cuda") for x in xs]
            rec = sz.new_sizes_array(k)
            sz.compress_batch(xd, cbs, outs, ws, rec, capacities=[o.numel() - 512 for o in outs])
            torch.cuda.synchronize()
            got = sz.read_sizes_array(rec)
            for i, (ref, m) in enumerate(refs):
                assert got[i] == (ref.size, m, 0), (i, got[i], ref.size, m)
                assert np.array_equal(outs[i][:ref.size].cpu().numpy(), ref), f"batch stream {i} differs"
                assert (outs[i][ref.size:ref.size + 512].cpu().numpy() == 0xA5).all()
            ys = [torch.empty(max(x.size, 1), dtype=t.dtype, device="cuda") for x, t in zip(xs, xd)]
            st = sz.new_sizes()
            sz.decompress_batch(outs, [r[0].size for r in refs], [x.size for x in xs], cbs, ys, st)
            torch.cuda.synchronize()
            assert sz.read_sizes(st)[2] == 0
            for x, y, t in zip(xs, ys, xd):
                assert torch.equal(y[:x.size], t), "batch round trip differs"
            # the first tensor through the single calls as well
            one = torch.full((sz.compress_bound(xs[0].size, dt) + 512,), 0xA5, dtype=torch.uint8, device="cuda")
            s1 = sz.new_sizes()
            sz.compress(xd[0], cb, one, ws, s1, capacity=one.numel() - 512)
            torch.cuda.synchronize()
            assert sz.read_sizes(s1) == got[0] and torch.equal(one[:got[0][0]], outs[0][:got[0][0]])
            y = torch.empty(max(xs[0].size, 1), dtype=xd[0].dtype, device="cuda")
            sz.decompress(one, got[0][0], xs[0].size, cb, y)
            torch.cuda.synchronize()
            assert torch.equal(y[:xs[0].size], xd[0])


@pytest.mark.parametrize("round_", range(ROUNDS))
def test_variant_calls_on_random_cases(round_):
    rng = np.random.default_rng(20260502 + 1000 * round_)
    combos = [(sz.BF16, 4, 16, sz.ESC_POS, 1024), (sz.BF16, 4, 15, sz.ESC_SENTINEL, 256), (sz.BF16, 3, 8, sz.ESC_ABS32, 0),
              (sz.FP8_E5M2, 3, 7, sz.ESC_SENTINEL, 1024), (sz.FP8_E5M2, 4, 16, sz.ESC_POS, 256),
              (sz.FP8_E4M3, 3, 8, sz.ESC_POS, 1024), (sz.FP8_E4M3, 3, 5, sz.ESC_ABS32, 0), (sz.BF16, 4, 3, sz.ESC_POS, 256)]
    for dt, bits, k, mode, chunk in combos:
        v, o = sz.variant(dt, bits, k, mode, chunk), ov.variant(dt, bits, k, mode, chunk)
        for case in range(5):
            x = random_words(dt, random_size(rng), rng)
            dec, _ = ov.calibrate(x if rng.integers(0, 2) else random_words(dt, 3000, rng), o.dtype, o.k)
            print(f"case fuzz variant {v} #{case}: n={x.size}", flush=True)
            cb = sz.variant_codebook_from_dec(dec[:k], v)
            ref, m = ov.compress(x, o, dec)
            out = torch.full((sz.variant_compress_bound(x.size, v) + 512,), 0xA5, dtype=torch.uint8, device="cuda")
            wsp = torch.empty(max(sz.variant_workspace_bytes(x.size, v), 16), dtype=torch.uint8, device="cuda")
            rec = sz.new_sizes()
            sz.variant_compress(dev(x), v, cb, out, wsp, rec, capacity=out.numel() - 512)
            torch.cuda.synchronize()
            assert sz.read_sizes(rec) == (ref.size, m, 0)
            assert np.array_equal(out[:ref.size].cpu().numpy(), ref), "variant stream differs"
            assert (out[ref.size:ref.size + 512].cpu().numpy() == 0xA5).all()
            xd = dev(x)
            y = torch.empty(max(x.size, 1), dtype=xd.dtype, device="cuda")
            st = sz.new_sizes()
            sz.variant_decompress(out, ref.size, x.size, v, cb, y, st)
            torch.cuda.synchronize()
            assert sz.read_sizes(st) == (ref.size, m, 0) and torch.equal(y[:x.size], xd)


@pytest.mark.parametrize("round_", range(ROUNDS))
def test_device_calibrated_batches_on_random_cases(round_):
    rng = np.random.default_rng(20260503 + 1000 * round_)
    for dt in (sz.BF16, sz.FP8_E5M2):
        ws = sz.Workspace(400_000, dt)
        for case in range(6):
            k = int(rng.integers(1, 9))
            xs = [random_words(dt, random_size(rng), rng) for _ in range(k)]
            print(f"case fuzz device calibration dtype={dt} #{case}: sizes={[x.size for x in xs]}", flush=True)
            xd = [dev(x) for x in xs]
            dcbs = sz.DeviceCodebooks(k, dt)
            sz.CalibrateBatchDevice(xd, dcbs).launch()
            outs = [torch.full((sz.compress_bound(x.size, dt) + 512,), 0xA5, dtype=torch.uint8, device="cuda") for x in xs]
            rec = sz.new_sizes_array(k)
            sz.CompressBatchDcb(xd, dcbs, outs, capacities=[o.numel() - 512 for o in outs]).launch(ws, rec)
            torch.cuda.synchronize()
            got = sz.read_sizes_array(rec)
            totals = []
            for i, x in enumerate(xs):
                cb_or = oracle.calibrate(x, ODT[dt])
                assert dcbs.to_host(i).dec == cb_or.dec.tolist(), f"item {i}: codebook"
                ref, m = oracle.compress(x, cb_or)
                totals.append(ref.size)
                assert got[i] == (ref.size, m, 0), (i, got[i], ref.size, m)
                assert np.array_equal(outs[i][:ref.size].cpu().numpy(), ref), f"stream {i} differs"
                assert (outs[i][ref.size:ref.size + 512].cpu().numpy() == 0xA5).all()
            ys = [torch.empty(max(x.size, 1), dtype=t.dtype, device="cuda") for x, t in zip(xs, xd)]
            st = sz.new_sizes()
            sz.DecompressBatchDcb(outs, totals, [x.size for x in xs], dcbs, ys).launch(st)
            torch.cuda.synchronize()
            assert sz.read_sizes(st)[2] == 0
            for x, y, t in zip(xs, ys, xd):
                assert torch.equal(y[:x.size], t), "round trip differs"
