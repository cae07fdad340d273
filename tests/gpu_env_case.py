"""Helper for GPU tests that need the library's environment knobs, which are read once per process.
Run as `python tests/gpu_env_case.py <case>` with the knobs set; prints CASE-OK on success.
Compares against the CPU oracle like the parity tests do."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import kv_synth  # noqa: E402
import oracle  # noqa: E402
import paper_2605_01708_amd as sz  # noqa: E402

DT = {sz.BF16: oracle.BF16, sz.FP8_E5M2: oracle.E5M2}


def words(dtype, tokens, seed):
    gen = kv_synth.kv_bf16 if dtype == sz.BF16 else kv_synth.kv_e5m2
    return kv_synth.to_numpy_words(gen(tokens, seed))


def dev(x):
    return torch.from_numpy(x.view(np.int16).copy() if x.dtype == np.uint16 else x.copy()).cuda()


def several_launches():
    """SPLITZIP_COMPRESS_MAX_WGS=4: a tensor of 5 Mi elements takes five segment launches and the
    finishing launch; the stream must still be the oracle's.  The batch call routes it the same way."""
    for dtype in (sz.BF16, sz.FP8_E5M2):
        x = words(dtype, 5 * 1024 + 3, 4)[:-517].copy()
        x[:: 997] = 0
        cb_or = oracle.calibrate(words(dtype, 256, 1), DT[dtype])
        cb = sz.codebook_from_dec(cb_or.dec.tolist(), dtype)
        ref, m = oracle.compress(x, cb_or)
        out = torch.full((sz.compress_bound(x.size, dtype) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        ws = sz.Workspace(x.size, dtype)
        sizes = sz.new_sizes()
        xd = dev(x)
        for rep in range(2):
            sz.compress(xd, cb, out, ws, sizes)
            torch.cuda.synchronize()
            assert sz.read_sizes(sizes) == (ref.size, m, 0), (sz.read_sizes(sizes), ref.size, m)
            assert np.array_equal(out[: ref.size].cpu().numpy(), ref), "stream differs"
            assert (out[ref.size:].cpu().numpy() == 0xA5).all()
        # batch: the large item falls back to the single call, the small ones go through the batch kernel
        small = [x[:70000].copy(), x[100:100 + 1025].copy()]
        xs = [dev(small[0]), xd, dev(small[1])]
        outs = [torch.empty(sz.compress_bound(t.numel(), dtype), dtype=torch.uint8, device="cuda") for t in xs]
        rec = sz.new_sizes_array(3)
        sz.compress_batch(xs, [cb] * 3, outs, ws, rec)
        torch.cuda.synchronize()
        got = sz.read_sizes_array(rec)
        for k, src in enumerate((small[0], x, small[1])):
            r, mm = oracle.compress(src, cb_or)
            assert got[k] == (r.size, mm, 0), (k, got[k], r.size, mm)
            assert np.array_equal(outs[k][: r.size].cpu().numpy(), r), f"batch item {k} differs"
        y = torch.empty_like(xd)
        st = sz.new_sizes()
        sz.decompress(out, ref.size, x.size, cb, y, st)
        torch.cuda.synchronize()
        assert sz.read_sizes(st)[2] == 0 and torch.equal(y, xd)


def exchange_timeout():
    """SPLITZIP_TEST_AWAIT_EXTRA_WGS=1 with a tiny SPLITZIP_SPIN_TICKS: every workgroup waits for a word that
    never comes, gives up, and the call reports SPLITZIP_STATUS_INTERNAL; every kernel still ends normally."""
    dtype = sz.BF16
    x = words(dtype, 64, 4)
    cb = sz.calibrate(torch.from_numpy(words(dtype, 64, 1).view(np.int16).copy()), dtype)
    out = torch.empty(sz.compress_bound(x.size, dtype), dtype=torch.uint8, device="cuda")
    ws = sz.Workspace(x.size, dtype)
    sizes = sz.new_sizes()
    sz.compress(dev(x), cb, out, ws, sizes)
    torch.cuda.synchronize()
    status = sz.read_sizes(sizes)[2]
    assert status & sz.STATUS_INTERNAL, status


if __name__ == "__main__":
    assert torch.cuda.is_available()
    {"several_launches": several_launches, "exchange_timeout": exchange_timeout}[sys.argv[1]]()
    print("CASE-OK", sys.argv[1], flush=True)
