"""The format variants of the ablations: host logic of the library against the variant oracle (CPU), and
the variant kernels, called through the C ABI, against the same oracle byte for byte (GPU)."""
import ctypes as C

import numpy as np
import pytest
import torch

import kv_synth
import oracle
from oracle import variants as ov
import paper_2605_01708_amd as sz

POISON = 0xA5
GEN = {sz.BF16: kv_synth.kv_bf16, sz.FP8_E5M2: kv_synth.kv_e5m2, sz.FP8_E4M3: kv_synth.kv_e4m3}


def variants():
    """(library variant, oracle variant) pairs: the formats the paper ablates, per dtype"""
    out = []
    for dt in (sz.BF16, sz.FP8_E5M2):
        for cb, k, mode, chunk in ((4, 16, sz.ESC_POS, 1024), (4, 15, sz.ESC_SENTINEL, 1024), (3, 8, sz.ESC_POS, 1024),
                                   (4, 16, sz.ESC_POS, 256), (4, 16, sz.ESC_ABS32, 0), (3, 7, sz.ESC_SENTINEL, 256)):
            out.append((sz.variant(dt, cb, k, mode, chunk), ov.variant(dt, cb, k, mode, chunk)))
    for cb, k, mode, chunk in ((3, 8, sz.ESC_POS, 1024), (3, 7, sz.ESC_SENTINEL, 1024), (3, 8, sz.ESC_ABS32, 0),
                               (3, 8, sz.ESC_POS, 256)):
        out.append((sz.variant(sz.FP8_E4M3, cb, k, mode, chunk), ov.variant(ov.E4M3, cb, k, mode, chunk)))
    # escape values in the exponent's own width (the top-8 columns of the paper's FP8 table), in every escape mode
    for dt, odt, vb in ((sz.FP8_E5M2, ov.E5M2, 5), (sz.FP8_E4M3, ov.E4M3, 4)):
        for cb, k, mode, chunk in ((3, 8, sz.ESC_POS, 1024), (3, 7, sz.ESC_SENTINEL, 256), (3, 8, sz.ESC_ABS32, 0)):
            out.append((sz.variant(dt, cb, k, mode, chunk, vb), ov.variant(odt, cb, k, mode, chunk, vb)))
    out.append((sz.variant(sz.FP8_E5M2, 4, 16, sz.ESC_POS, 1024, 5), ov.variant(ov.E5M2, 4, 16, ov.ESC_POS, 1024, 5)))
    return out


def vid(pair):
    v = pair[0]
    return f"dt{v.dtype}-b{v.code_bits}-k{v.k}-m{v.escape_mode}-c{v.chunk_elems}" + (f"-v{v.value_bits}" if v.value_bits else "")


def words(dt, tokens, seed, layer=0, kind="K", device="cpu"):
    return kv_synth.to_numpy_words(GEN[dt](tokens, seed, layer, kind, device))


# ---- CPU: host logic ------------------------------------------------------------------------

@pytest.mark.parametrize("pair", variants(), ids=vid)
def test_sizes_and_calibration_match_the_oracle(pair):
    v, o = pair
    assert sz.variant_supported(v) and ov.valid(o)
    for n, m in ((0, 0), (1, 1), (255, 0), (256, 3), (1024, 1024), (1025, 7), (5000, 12), (1 << 25, 54321)):
        assert sz.variant_total_bytes(n, m, v) == ov.total_bytes(n, m, o)
        assert sz.variant_compress_bound(n, v) == ov.total_bytes(n, n, o)
    assert sz.variant_total_bytes(1 << 32, 0, v) == 0
    for seed, tokens in ((1, 64), (2, 3)):
        s = GEN[v.dtype](tokens, seed)
        cb, hist = sz.variant_calibrate(s, v, return_hist=True)
        dec, h = ov.calibrate(kv_synth.to_numpy_words(s), o.dtype, o.k)
        assert cb.dec == dec.tolist() and hist == h.tolist()
        assert sum(cb.member) == v.k and all(cb.member[e] for e in dec[:v.k])
        assert [cb.enc[e] for e in dec[:v.k]] == list(range(v.k))
        cb2 = sz.variant_codebook_from_dec(dec[:v.k], v)
        assert (cb2.dec, cb2.enc, cb2.member) == (cb.dec, cb.enc, cb.member)


def test_unsupported_variants_and_bad_arguments_are_refused():
    bad = [sz.variant(sz.BF16, 4, 16, sz.ESC_SENTINEL, 1024), sz.variant(sz.BF16, 3, 9, sz.ESC_POS, 1024),
           sz.variant(sz.BF16, 5, 16, sz.ESC_POS, 1024), sz.variant(sz.BF16, 4, 16, sz.ESC_POS, 512),
           sz.variant(3, 4, 16, sz.ESC_POS, 1024), sz.variant(sz.BF16, 4, 16, 3, 1024),
           sz.variant(sz.FP8_E4M3, 4, 17, sz.ESC_POS, 1024), sz.variant(sz.BF16, 4, 0, sz.ESC_POS, 1024)]
    for v in bad:
        assert not sz.variant_supported(v)
        assert sz.variant_total_bytes(100, 0, v) == 0 and sz.variant_workspace_bytes(100, v) == 0
    L = sz.lib()
    v = sz.variant(sz.BF16, 3, 8, sz.ESC_POS, 1024)
    cb = sz.variant_calibrate(kv_synth.kv_bf16(8, 1), v)
    cb16 = sz.calibrate(kv_synth.kv_bf16(8, 1), sz.BF16)          # 16 members: not this variant's codebook
    buf = 1 << 12                                                  # an aligned non-null "pointer"; never dereferenced
    args = lambda **k: [k.get("d_in", buf), k.get("n", 100), C.byref(k.get("v", v)), C.byref(k.get("cb", cb).c),
                        k.get("d_out", buf), k.get("cap", 1 << 20), k.get("ws", buf), k.get("wsb", 1 << 20),
                        k.get("sizes", buf), None]
    assert L.splitzip_variant_compress(*args(v=bad[0])) == -1
    assert L.splitzip_variant_compress(*args(cb=cb16)) == -1
    assert L.splitzip_variant_compress(*args(d_in=buf + 2)) == -1
    assert L.splitzip_variant_compress(*args(d_out=None)) == -1
    assert L.splitzip_variant_compress(*args(sizes=None)) == -1
    assert L.splitzip_variant_compress(*args(n=1 << 32)) == -2
    assert L.splitzip_variant_compress(*args(cap=100)) == -3
    assert L.splitzip_variant_compress(*args(wsb=16)) == -3
    dargs = lambda **k: [k.get("comp", buf), k.get("bytes", 1 << 20), k.get("n", 100), C.byref(k.get("v", v)),
                         C.byref(k.get("cb", cb).c), k.get("out", buf), None, None]
    assert L.splitzip_variant_decompress(*dargs(v=bad[1])) == -1
    assert L.splitzip_variant_decompress(*dargs(cb=cb16)) == -1
    assert L.splitzip_variant_decompress(*dargs(out=buf + 4)) == -1
    assert L.splitzip_variant_decompress(*dargs(n=1 << 32)) == -2
    assert L.splitzip_variant_decompress(*dargs(bytes=64)) == -3
    # the main calls do not take E4M3
    assert sz.fixed_bytes(100, sz.FP8_E4M3) == 0


# ---- GPU: parity with the oracle -------------------------------------------------------------

def dev(x):
    return torch.from_numpy(x.view(np.int16).copy() if x.dtype == np.uint16 else x.copy()).cuda()


class Run:
    def __init__(self, nmax, v):
        self.v = v
        self.out = torch.empty(sz.variant_compress_bound(nmax, v) + 4160, dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(max(sz.variant_workspace_bytes(nmax, v), 16), dtype=torch.uint8, device="cuda")
        self.sizes = sz.new_sizes()

    def compress(self, x_dev, cb, capacity=None):
        self.out.fill_(POISON)
        self.ws.fill_(0x3C)              # the workspace needs no initialisation
        self.sizes.fill_(-1)
        sz.variant_compress(x_dev, self.v, cb, self.out, self.ws, self.sizes,
                            capacity=self.out.numel() - 4160 if capacity is None else capacity)
        torch.cuda.synchronize()
        return sz.read_sizes(self.sizes)

    def decompress(self, comp, nbytes, n, cb):
        es = 2 if self.v.dtype == sz.BF16 else 1
        y = torch.full((n + 64,), 0x5A5A if es == 2 else 0x5A, dtype=torch.int16 if es == 2 else torch.uint8, device="cuda")
        st = sz.new_sizes()
        sz.variant_decompress(comp, nbytes, n, self.v, cb, y, st)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        yh = yh.view(np.uint16) if es == 2 else yh
        assert (yh[n:] == (0x5A5A if es == 2 else 0x5A)).all(), "decompress wrote past n_elems"
        return yh[:n], sz.read_sizes(st)


def check(run, o, x, dec, label):
    print(f"case {label}: n={x.size} {run.v}", flush=True)
    cb = sz.variant_codebook_from_dec(dec[:run.v.k], run.v)
    ref, m_ref = ov.compress(x, o, dec)
    total, m, status = run.compress(dev(x), cb)
    assert (total, m, status) == (ref.size, m_ref, 0), (total, m, status, ref.size, m_ref)
    got = run.out[:total].cpu().numpy()
    if not np.array_equal(got, ref):
        badb = np.flatnonzero(got != ref)
        raise AssertionError(f"{label}: stream differs at {badb.size} bytes, first {badb[:8]} got {got[badb[:8]]} "
                             f"want {ref[badb[:8]]}")
    assert (run.out[total:total + 4096].cpu().numpy() == POISON).all(), "compress wrote past total_bytes"
    y, (t2, m2, st2) = run.decompress(run.out, total, x.size, cb)
    assert (t2, m2, st2) == (total, m, 0) and np.array_equal(y, x), f"{label}: GPU round trip differs"
    y2, (_, _, st3) = run.decompress(torch.from_numpy(ref.copy()).cuda(), ref.size, x.size, cb)   # the oracle's stream
    assert st3 == 0 and np.array_equal(y2, x)
    assert np.array_equal(ov.decompress(got, x.size, o, dec), x)
    return total, m


@pytest.mark.gpu
@pytest.mark.parametrize("pair", variants(), ids=vid)
def test_variant_streams_match_the_oracle(pair):
    v, o = pair
    assert torch.cuda.is_available()
    dt = v.dtype
    dec, _ = ov.calibrate(words(dt, 1024, 1), o.dtype, o.k)
    run = Run(4096 * 1024, v)
    # the small benchmark tensor, ragged sizes around every boundary, nothing at all
    check(run, o, words(dt, 4096, 0, device="cuda"), dec, "config0")
    base = words(dt, 40, 3)
    for n in (0, 1, 7, 8, 9, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 4097, 40 * 1024 - 5):
        check(run, o, base[:n].copy(), dec, f"ragged {n}")
    # every bit pattern, under the calibrated codebook and one of exponents that never occur in KV data
    allw = np.arange(65536 if dt == sz.BF16 else 256, dtype=np.uint32).astype(base.dtype)
    pats = np.tile(allw, 1 if dt == sz.BF16 else 40)
    top = np.zeros(16, np.uint8)
    nexp = {sz.BF16: 256, sz.FP8_E5M2: 32, sz.FP8_E4M3: 16}[dt]
    top[:v.k] = np.arange(nexp - v.k, nexp)
    check(run, o, pats, dec, "all patterns")
    check(run, o, pats, top, "all patterns, odd codebook")
    # nearly everything escapes: the escape sections dominate the stream
    check(run, o, base, top, "nearly all escape")


@pytest.mark.gpu
def test_variant_overflow_and_bad_streams():
    v, o = sz.variant(sz.BF16, 4, 16, sz.ESC_POS, 256), ov.variant(ov.BF16, 4, 16, ov.ESC_POS, 256)
    x = words(sz.BF16, 64, 2)
    dec, _ = ov.calibrate(words(sz.BF16, 1, 1)[:16].copy(), ov.BF16, 16)        # a poor codebook: many escapes
    cb = sz.variant_codebook_from_dec(dec, v)
    ref, m = ov.compress(x, o, dec)
    assert m > 100
    run = Run(x.size, v)
    fixed = sz.variant_total_bytes(x.size, 0, v)
    total, m2, status = run.compress(dev(x), cb, capacity=fixed + 64)
    assert (total, m2, status) == (ref.size, m, sz.STATUS_OVERFLOW)
    assert np.array_equal(run.out[:fixed].cpu().numpy()[64:], ref[64:fixed])     # the fixed part is complete
    assert (run.out[fixed + 64:fixed + 4096].cpu().numpy() == POISON).all()      # nothing past the capacity
    # damaged streams are flagged, not followed
    good = torch.from_numpy(ref.copy()).cuda()
    for off, val in ((0, 0x54), (4, 1), (13, 15), (24, (m + 1) & 0xFF), (64 + 4, 0xFF)):
        bad = good.clone()
        bad[off] = val
        _, (_, _, st) = run.decompress(bad, ref.size, x.size, cb)
        assert st & sz.STATUS_BAD_STREAM, (off, st)
    _, (_, _, st) = run.decompress(good, ref.size, x.size, cb)
    assert st == 0
    # positions inside a chunk must ascend: two records of one chunk change places (the oracle's decoder rejects it)
    n_chunks = (x.size + 255) // 256
    tab = ref[64:64 + 4 * (n_chunks + 1)].view(np.uint32)
    ch = int(np.argmax(np.diff(tab) >= 2))
    assert tab[ch + 1] - tab[ch] >= 2
    off_pos = sz.variant_total_bytes(x.size, 0, v)              # 8-bit positions start behind the fixed part
    swapped = ref.copy()
    j = off_pos + int(tab[ch])
    swapped[j], swapped[j + 1] = swapped[j + 1], swapped[j]
    with pytest.raises(ValueError):
        ov.decompress(swapped, x.size, o, dec)
    _, (_, _, st) = run.decompress(torch.from_numpy(swapped).cuda(), ref.size, x.size, cb)
    assert st & sz.STATUS_BAD_STREAM
    # the same for absolute positions
    va, oa = sz.variant(sz.BF16, 4, 16, sz.ESC_ABS32, 0), ov.variant(ov.BF16, 4, 16, ov.ESC_ABS32, 0)
    cba = sz.variant_codebook_from_dec(dec, va)
    refa, ma = ov.compress(x, oa, dec)
    posa = sz.variant_total_bytes(x.size, 0, va)
    swapped = refa.copy()
    p32 = swapped[posa:posa + 4 * ma].view(np.uint32)
    p32[5], p32[6] = p32[6], p32[5]
    with pytest.raises(ValueError):
        ov.decompress(swapped, x.size, oa, dec)
    runa = Run(x.size, va)
    _, (_, _, st) = runa.decompress(torch.from_numpy(swapped).cuda(), refa.size, x.size, cba)
    assert st & sz.STATUS_BAD_STREAM
    _, (_, _, st) = runa.decompress(torch.from_numpy(refa.copy()).cuda(), refa.size, x.size, cba)
    assert st == 0


@pytest.mark.gpu
def test_variant_full_size_tensor():
    """one K tensor of the benchmark's shape [32768, 8, 128] through two of the variants"""
    x = words(sz.BF16, 32768, 0, 3, "K", device="cuda")
    for v, o in ((sz.variant(sz.BF16, 3, 8, sz.ESC_POS, 1024), ov.variant(ov.BF16, 3, 8, ov.ESC_POS, 1024)),
                 (sz.variant(sz.BF16, 4, 15, sz.ESC_SENTINEL, 1024), ov.variant(ov.BF16, 4, 15, ov.ESC_SENTINEL, 1024))):
        dec, _ = ov.calibrate(words(sz.BF16, 1024, 1), ov.BF16, o.k)
        total, m = check(Run(x.size, v), o, x, dec, "full size")
        print(f"{v}: eps={m / x.size:.4f} ratio={2 * x.size / total:.4f}", flush=True)
