"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-side logic (calibration, size functions,
argument validation) agrees with the oracle.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

import kv_synth
import oracle
import paper_2605_01708_amd as sz

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "splitzip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(splitzip_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"splitzip_calibrate", "splitzip_compress", "splitzip_decompress", "splitzip_workspace_init",
            "splitzip_fixed_bytes", "splitzip_total_bytes", "splitzip_compress_bound",
            "splitzip_workspace_bytes", "splitzip_codebook_from_dec", "splitzip_strerror",
            "splitzip_version", "splitzip_traffic_probe", "splitzip_traffic_probe_shape", "splitzip_compress_batch",
            "splitzip_decompress_batch", "splitzip_histogram", "splitzip_codebook_from_hist",
            "splitzip_codebook_device", "splitzip_compress_dcb", "splitzip_decompress_dcb"} <= set(names)
    L = C.CDLL(sz.lib_path())
    for n in names:
        assert hasattr(L, n), n
    assert sz.lib().splitzip_version() == 1
    assert sz.lib().splitzip_strerror(-3) == b"buffer too small"


@pytest.mark.parametrize("dtype,gen", [(sz.BF16, kv_synth.kv_bf16), (sz.FP8_E5M2, kv_synth.kv_e5m2)])
def test_host_calibrate_matches_oracle(dtype, gen):
    for seed, tokens in [(1, 64), (2, 7), (3, 1)]:
        s = gen(tokens, seed)
        cb, hist = sz.calibrate(s, dtype, return_hist=True)
        ref = oracle.calibrate(kv_synth.to_numpy_words(s), dtype)
        assert cb.dec == ref.dec.tolist()
        assert cb.enc == ref.enc.tolist()
        assert cb.member == ref.member.tolist()
        assert hist == ref.hist.tolist()
        assert cb.dtype == dtype


def test_codebook_from_hist_ranks_like_calibrate():
    """the tables built from a histogram are those of calibrate on the sample that has it (same reading of ties)"""
    for dtype, gen in ((sz.BF16, kv_synth.kv_bf16), (sz.FP8_E5M2, kv_synth.kv_e5m2)):
        s = gen(9, 4)
        cb, hist = sz.calibrate(s, dtype, return_hist=True)
        cb2 = sz.codebook_from_hist(hist, dtype)
        assert (cb2.dec, cb2.enc, cb2.member, cb2.dtype) == (cb.dec, cb.enc, cb.member, cb.dtype)
    h = [0] * 256
    h[130] = h[120] = h[3] = 50
    h[125] = 70
    assert sz.codebook_from_hist(h, sz.BF16).dec == [125, 3, 120, 130, 0, 1, 2, 4, 5, 6, 7, 8, 9, 10, 11, 12]
    assert sz.lib().splitzip_codebook_from_hist(None, sz.BF16, None) == -1
    assert sz.lib().splitzip_histogram(None, 16, sz.BF16, None, None) == -1


def test_host_calibrate_ties_and_empty():
    # ties to the smaller exponent, unseen values fill in ascending order (same reading as the oracle)
    es = np.array([130] * 50 + [120] * 50 + [125] * 70 + [3] * 50, np.uint16)
    cb = sz.calibrate(torch.from_numpy((es << 7).astype(np.int16)), sz.BF16)
    assert cb.dec == [125, 3, 120, 130, 0, 1, 2, 4, 5, 6, 7, 8, 9, 10, 11, 12]
    cb = sz.calibrate(torch.zeros(0, dtype=torch.int16), sz.BF16)
    assert cb.dec == list(range(16))
    cb = sz.calibrate(torch.tensor([31 << 2] * 9 + [30 << 2] * 9 + [2 << 2] * 10, dtype=torch.uint8), sz.FP8_E5M2)
    assert cb.dec == [2, 30, 31, 0, 1, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13]


def test_codebook_from_dec_validation():
    cb = sz.codebook_from_dec(range(100, 116), sz.BF16)
    assert cb.dec == list(range(100, 116)) and sum(cb.member) == 16 and cb.enc[107] == 7
    with pytest.raises(sz.SplitZipError):
        sz.codebook_from_dec([1] * 16, sz.BF16)            # duplicates
    with pytest.raises(sz.SplitZipError):
        sz.codebook_from_dec(range(20, 36), sz.FP8_E5M2)   # 5-bit exponents only
    with pytest.raises(sz.SplitZipError):
        sz.codebook_from_dec(range(16), 7)                 # dtype


def test_size_functions_match_oracle():
    for dtype in (sz.BF16, sz.FP8_E5M2):
        for n in [0, 1, 2, 15, 16, 17, 1023, 1024, 1025, 8191, 8192, 8193, 4194304, 33554432]:
            assert sz.fixed_bytes(n, dtype) == oracle.total_bytes(n, 0, dtype)
            assert sz.compress_bound(n, dtype) == oracle.total_bytes(n, n, dtype)
            for m in {0, 1, 7, 8, min(n, 12345)}:
                if m <= n:
                    assert sz.total_bytes(n, m, dtype) == oracle.total_bytes(n, m, dtype)
            assert sz.workspace_bytes(n, dtype) >= n + 64
    assert sz.fixed_bytes(1 << 32, sz.BF16) == 0 and sz.fixed_bytes(8, 5) == 0


def test_argument_validation_without_gpu():
    """Every rejected call returns before any GPU work is enqueued."""
    L = sz.lib()
    cb = sz.codebook_from_dec(range(100, 116), sz.BF16)
    buf = (C.c_uint8 * 4096)()
    base = (C.addressof(buf) + 15) & ~15
    n = 64
    good = dict(d_in=base, n=n, dtype=sz.BF16, cb=C.byref(cb.c), d_out=base + 1024, cap=1 << 20,
                ws=base + 2048, wsb=1 << 24, sizes=base + 3072, stream=None)

    def comp(**kw):
        a = dict(good, **kw)
        return L.splitzip_compress(a["d_in"], a["n"], a["dtype"], a["cb"], a["d_out"], a["cap"], a["ws"],
                                   a["wsb"], a["sizes"], a["stream"])

    assert comp(d_in=None) == -1
    assert comp(d_out=None) == -1
    assert comp(ws=None) == -1
    assert comp(sizes=None) == -1
    assert comp(d_in=base + 2) == -1           # misaligned
    assert comp(d_out=base + 1024 + 8) == -1
    assert comp(dtype=9) == -1
    assert comp(n=1 << 32) == -2
    assert comp(cap=sz.fixed_bytes(n, sz.BF16) - 1) == -3
    assert comp(wsb=16) == -3
    bad = sz.codebook_from_dec(range(100, 116), sz.BF16)
    bad.c.enc[100] = 3                         # enc/dec no longer inverse
    assert comp(cb=C.byref(bad.c)) == -1
    e5 = sz.codebook_from_dec(range(16), sz.FP8_E5M2)
    assert comp(cb=C.byref(e5.c)) == -1        # codebook built for another dtype

    def decomp(**kw):
        a = dict(d_comp=base, cb=C.byref(cb.c), bytes=1 << 20, n=n, dtype=sz.BF16, d_out=base + 1024,
                 sizes=None, stream=None)
        a.update(kw)
        return L.splitzip_decompress(a["d_comp"], a["bytes"], a["n"], a["dtype"], a["cb"], a["d_out"],
                                     a["sizes"], a["stream"])

    assert decomp(d_comp=None) == -1
    assert decomp(d_out=None) == -1
    assert decomp(d_comp=base + 4) == -1
    assert decomp(bytes=sz.fixed_bytes(n, sz.BF16) - 1) == -3
    assert decomp(n=1 << 32) == -2
    assert decomp(dtype=2) == -1
    # batch calls: every item is checked before anything is enqueued
    from paper_2605_01708_amd.binding import _CDItem, _CItem
    items = (_CItem * 2)(_CItem(base, n, base + 1024, 1 << 20, C.pointer(cb.c)),
                         _CItem(base, n, base + 1024, 1 << 20, C.pointer(cb.c)))
    bcomp = lambda its, k, ws=base + 2048, wsb=1 << 24, sizes=base + 3072: L.splitzip_compress_batch(  # noqa: E731
        its, k, sz.BF16, ws, wsb, sizes, None)
    assert bcomp(None, 2) == -1
    assert bcomp(items, 2, ws=None) == -1
    assert bcomp(items, 2, sizes=None) == -1
    assert bcomp(items, 2, wsb=16) == -3
    items[1].out_capacity = sz.fixed_bytes(n, sz.BF16) - 1
    assert bcomp(items, 2) == -3
    items[1].out_capacity = 1 << 20
    items[1].d_in = base + 2
    assert bcomp(items, 2) == -1
    items[1].d_in = base
    items[1].n_elems = 1 << 32
    assert bcomp(items, 2) == -2
    items[1].n_elems = n
    items[1].cb = C.pointer(e5.c)
    assert bcomp(items, 2) == -1
    assert bcomp(items, 0) == 0                                   # an empty list is fine and launches nothing
    ditems = (_CDItem * 2)(_CDItem(base, 1 << 20, n, base + 1024, C.pointer(cb.c)),
                           _CDItem(base, sz.fixed_bytes(n, sz.BF16) - 1, n, base + 1024, C.pointer(cb.c)))
    assert L.splitzip_decompress_batch(ditems, 2, sz.BF16, None, None) == -3
    ditems[1].comp_bytes = 1 << 20
    ditems[1].d_comp = None
    assert L.splitzip_decompress_batch(ditems, 2, sz.BF16, None, None) == -1
    assert L.splitzip_decompress_batch(None, 2, sz.BF16, None, None) == -1
    assert L.splitzip_decompress_batch(ditems, 0, sz.BF16, None, None) == 0
    # device-codebook calls: the codebook pointer is all the host can check
    assert L.splitzip_compress_dcb(base, n, sz.BF16, None, base + 1024, 1 << 20, base + 2048, 1 << 20, base + 3072, None) == -1
    assert L.splitzip_compress_dcb(base, n, sz.BF16, base + 512 + 2, base + 1024, 1 << 20, base + 2048, 1 << 20, base + 3072, None) == -1
    assert L.splitzip_compress_dcb(base, n, sz.BF16, base + 512, base + 1024, 16, base + 2048, 1 << 24, base + 3072, None) == -3
    assert L.splitzip_decompress_dcb(base, 1 << 20, n, sz.BF16, None, base + 1024, None, None) == -1
    assert L.splitzip_decompress_dcb(base, 16, n, sz.BF16, base + 512, base + 1024, None, None) == -3
    assert L.splitzip_codebook_device(None, sz.BF16, base, None) == -1
    assert L.splitzip_codebook_device(base, 7, base + 512, None) == -1
    assert L.splitzip_workspace_init(None, 1024, None) == -1
    assert L.splitzip_traffic_probe(None, 16, base, 16, None) == -1


def test_device_calibrated_batch_calls_reject_bad_arguments_without_gpu():
    from paper_2605_01708_amd.binding import _CItem, _CDItem, _CCodebook
    L = sz.lib()
    buf = (C.c_uint8 * 8192)()
    base = (C.addressof(buf) + 15) & ~15
    null_cb = C.POINTER(_CCodebook)()
    items = (_CItem * 1)(_CItem(base, 64, base + 1024, 1 << 20, null_cb))
    hists, dcbs, ws, sizes = base + 2048, base + 4096, base + 5120, base + 6144
    f = L.splitzip_calibrate_batch_device
    assert f(items, 1, sz.BF16, None, dcbs, None) == -1
    assert f(items, 1, sz.BF16, hists, None, None) == -1
    assert f(items, 1, sz.BF16, hists + 4, dcbs, None) == -1       # counts 8-byte aligned
    assert f(items, 1, sz.BF16, hists, dcbs + 2, None) == -1       # codebooks 4-byte aligned
    assert f(items, 1, 9, hists, dcbs, None) == -1
    assert f(None, 0, sz.BF16, None, None, None) == 0              # nothing to do
    bad = (_CItem * 1)(_CItem(base + 2, 64, None, 0, null_cb))
    assert f(bad, 1, sz.BF16, hists, dcbs, None) == -1             # misaligned sample
    g = L.splitzip_compress_batch_dcb
    assert g(items, 1, sz.BF16, None, ws, 1 << 20, sizes, None) == -1          # no codebooks
    assert g(items, 1, sz.BF16, dcbs + 2, ws, 1 << 20, sizes, None) == -1
    assert g(items, 1, sz.BF16, dcbs, ws, 16, sizes, None) == -3               # workspace too small
    small = (_CItem * 1)(_CItem(base, 64, base + 1024, 8, null_cb))
    assert g(small, 1, sz.BF16, dcbs, ws, 1 << 20, sizes, None) == -3          # output below the fixed part
    d = (_CDItem * 1)(_CDItem(base, 1 << 20, 64, base + 1024, null_cb))
    h = L.splitzip_decompress_batch_dcb
    assert h(d, 1, sz.BF16, None, None, None) == -1
    assert h(d, 1, sz.BF16, dcbs + 1, None, None) == -1
    short = (_CDItem * 1)(_CDItem(base, 8, 64, base + 1024, null_cb))
    assert h(short, 1, sz.BF16, dcbs, None, None) == -3
    o = L.splitzip_decompress_batch_own
    assert o(d, 1, 9, None, None) == -1 and o(short, 1, sz.BF16, None, None) == -3 and o(None, 0, sz.BF16, None, None) == 0
    assert L.splitzip_decompress_own(None, 1 << 20, 64, sz.BF16, base + 1024, None, None) == -1
    assert L.splitzip_decompress_own(base, 8, 64, sz.BF16, base + 1024, None, None) == -3
    assert L.splitzip_decompress_own(base + 4, 1 << 20, 64, sz.BF16, base + 1024, None, None) == -1
    # and the host-codebook batch calls still insist on a valid codebook per item
    assert L.splitzip_compress_batch(items, 1, sz.BF16, ws, 1 << 20, sizes, None) == -1
