"""splitzip_compress_noalloc (the entry point for callers that cannot allocate) against splitzip_compress:
same stream bytes and sizes record, on two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

import kv_synth
import paper_2605_01708_amd as sz

pytestmark = pytest.mark.gpu


def _both_ways(x, cb, dtype):
    n = x.numel()
    bound = sz.compress_bound(n, dtype)
    ref = torch.full((bound + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    out = torch.full((bound + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    s_ref, s_out = sz.new_sizes(), sz.new_sizes()
    ws = sz.Workspace(n, dtype)
    sz.compress(x, cb, ref, ws, s_ref, capacity=bound)
    # through the C ABI, no binding helper in between
    L = sz.lib()
    rc = L.splitzip_compress_noalloc(x.data_ptr(), n, dtype, C.byref(cb.c), out.data_ptr(), bound, s_out.data_ptr(),
                                     C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, rc
    torch.cuda.synchronize()
    got, want = sz.read_sizes(s_out), sz.read_sizes(s_ref)
    assert got == want and got[2] == 0, (got, want)
    assert torch.equal(out, ref), "stream of the no-alloc call differs"      # the bytes behind the stream too: untouched
    y = torch.empty_like(x)
    d = sz.new_sizes()
    sz.decompress(out, got[0], n, cb, y, d)
    torch.cuda.synchronize()
    assert sz.read_sizes(d)[2] == 0 and torch.equal(y, x)
    return got


@pytest.mark.parametrize("dtype,gen", [(sz.BF16, kv_synth.kv_bf16), (sz.FP8_E5M2, kv_synth.kv_e5m2)])
def test_no_alloc_matches_compress_twice(dtype, gen):
    cb = sz.calibrate(gen(256, 1), dtype)
    big = gen(3000, 0).cuda().reshape(-1)[:-333].contiguous()          # 3 Mi elements, ragged last chunk
    small = gen(41, 5).cuda().reshape(-1)[:-1000].contiguous()         # 41 chunks, ragged
    a = _both_ways(big, cb, dtype)
    b = _both_ways(small, cb, dtype)
    assert a[1] > 0 and b[0] < a[0]
    # a third call, larger again: the array carries whatever the smaller call left
    _both_ways(big, cb, dtype)


def test_no_alloc_rejects_what_it_cannot_take():
    L = sz.lib()
    most = sz.noalloc_max_elems()
    assert most >= 1 << 20
    cb = sz.calibrate(kv_synth.kv_bf16(64, 1), sz.BF16)
    x = torch.zeros(16, dtype=torch.int16, device="cuda")
    out = torch.empty(4096, dtype=torch.uint8, device="cuda")
    s = sz.new_sizes()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # too many elements: turned away before anything is read
    assert L.splitzip_compress_noalloc(x.data_ptr(), most + 1, sz.BF16, C.byref(cb.c), out.data_ptr(), 4096, s.data_ptr(), st) == -2
    assert L.splitzip_compress_noalloc(None, 16, sz.BF16, C.byref(cb.c), out.data_ptr(), 4096, s.data_ptr(), st) == -1
    assert L.splitzip_compress_noalloc(x.data_ptr(), 16, sz.BF16, C.byref(cb.c), out.data_ptr(), 8, s.data_ptr(), st) == -3
    torch.cuda.synchronize()
