"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
byte for byte -- the compressed stream and the decompressed tensor -- on the
same seeded inputs.  All integer / bit work, so the bar is exact equality."""
import numpy as np
import pytest
import torch

import kv_synth
import oracle
import paper_2605_01708_amd as sz

pytestmark = pytest.mark.gpu

POISON = 0xA5
DT = {sz.BF16: oracle.BF16, sz.FP8_E5M2: oracle.E5M2}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU (run them on the MI355X box)"
    print("device:", torch.cuda.get_device_name(0), flush=True)


def words_tensor(x_np):
    """numpy raw words -> device tensor of the same bytes"""
    if x_np.dtype == np.uint16:
        return torch.from_numpy(x_np.view(np.int16).copy()).cuda()
    return torch.from_numpy(x_np.copy()).cuda()


def gpu_codebook(cb_or):
    return sz.codebook_from_dec(cb_or.dec.tolist(), cb_or.dtype)


class Gpu:
    """buffers for a run of calls of up to nmax elements"""

    def __init__(self, nmax, dtype):
        self.dtype = dtype
        self.ws = sz.Workspace(nmax, dtype)
        self.cap = sz.compress_bound(nmax, dtype) + 64
        self.out = torch.empty(self.cap, dtype=torch.uint8, device="cuda")
        self.sizes = sz.new_sizes()

    def compress(self, x_dev, cb, capacity=None):
        self.out.fill_(POISON)
        self.sizes.fill_(-1)
        sz.compress(x_dev, cb, self.out, self.ws, self.sizes, capacity=capacity)
        torch.cuda.synchronize()
        return sz.read_sizes(self.sizes)

    def decompress(self, comp_dev, comp_bytes, n, cb):
        es = 2 if self.dtype == sz.BF16 else 1
        y = torch.full((n + 64,), 0x5A if es == 1 else 0x5A5A, dtype=torch.int16 if es == 2 else torch.uint8,
                       device="cuda")
        st = sz.new_sizes()
        sz.decompress(comp_dev, comp_bytes, n, cb, y, st)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        yh = yh.view(np.uint16) if es == 2 else yh
        guard = 0x5A5A if es == 2 else 0x5A
        assert (yh[n:] == guard).all(), "decompress wrote past n_elems"
        return yh[:n], sz.read_sizes(st)


def check_parity(g, x_np, cb_or, label=""):
    print(f"case {label}: n={x_np.size} dtype={g.dtype}", flush=True)
    cb = gpu_codebook(cb_or)
    x_dev = words_tensor(x_np)
    ref_blob, ref_m = oracle.compress(x_np, cb_or)
    total, m, status = g.compress(x_dev, cb)
    assert status == 0
    assert m == ref_m
    assert total == ref_blob.size
    got = g.out[:total].cpu().numpy()
    if not np.array_equal(got, ref_blob):
        bad = np.flatnonzero(got != ref_blob)
        raise AssertionError(f"{label}: stream differs at {bad.size} bytes, first {bad[:8]} "
                             f"got {got[bad[:8]]} want {ref_blob[bad[:8]]}")
    tail = g.out[total:total + 4096].cpu().numpy()
    assert (tail == POISON).all(), "compress wrote past total_bytes"
    # GPU decoder on the GPU stream and on the oracle's stream
    y, (t2, m2, st2) = g.decompress(g.out, total, x_np.size, cb)
    assert st2 == 0 and t2 == total and m2 == m
    assert np.array_equal(y, x_np), f"{label}: GPU round trip differs"
    ref_dev = torch.from_numpy(ref_blob.copy()).cuda()
    y2, (_, _, st3) = g.decompress(ref_dev, ref_blob.size, x_np.size, cb)
    assert st3 == 0 and np.array_equal(y2, x_np)
    # oracle decoder on the GPU stream
    assert np.array_equal(oracle.decompress(got, x_np.size, cb_or), x_np)
    return total, m


def synth(dtype, tokens, seed, layer=0, kind="K"):
    gen = kv_synth.kv_bf16 if dtype == sz.BF16 else kv_synth.kv_e5m2
    return kv_synth.to_numpy_words(gen(tokens, seed, layer, kind))


def calibrated(dtype, seed=1, tokens=1024, layer=0, kind="K"):
    return oracle.calibrate(synth(dtype, tokens, seed, layer, kind), DT[dtype])


DTYPES = [sz.BF16, sz.FP8_E5M2]


@pytest.mark.parametrize("dtype", DTYPES)
def test_config0_single_k_tensor(dtype):
    """[4096, 8, 128] tensor, codebook from a separate seed-1 tensor of the same law"""
    x = synth(dtype, 4096, 0)
    cb = calibrated(dtype, seed=1, tokens=4096)
    g = Gpu(x.size, dtype)
    total, m = check_parity(g, x, cb, "config0")
    es = 2 if dtype == sz.BF16 else 1
    print(f"config0 dtype={dtype}: eps={m / x.size:.5f} ratio={es * x.size / total:.4f}", flush=True)
    assert m / x.size < 0.01


@pytest.mark.parametrize("dtype", DTYPES)
def test_ragged_and_tiny_sizes(dtype):
    """empty, single element, pack / lane / chunk / tile boundaries, several tiles plus a ragged tail"""
    cb = calibrated(dtype)
    base = synth(dtype, 64, 5).copy()                     # 65536 elements
    rng = np.random.default_rng(2)
    esc = rng.random(base.size) < 0.01                     # sprinkle zeros / max exponents
    base[esc] = 0
    base[::4099] = 0x7F80 if dtype == sz.BF16 else 0x7C
    g = Gpu(base.size, dtype)
    sizes = [0, 1, 2, 3, 15, 16, 17, 31, 32, 33, 1023, 1024, 1025, 2047, 2048, 2049, 8191, 8192, 8193,
             16384, 3 * 8192 + 5, 5 * 8192 - 1, 40000, 65535, 65536]
    for n in sizes:
        check_parity(g, base[:n].copy(), cb, f"n={n}")


def test_all_bf16_bit_patterns():
    rng = np.random.default_rng(7)
    x = rng.permutation(65536).astype(np.uint16)
    g = Gpu(x.size, sz.BF16)
    books = [oracle.codebook_from_dec(np.arange(119, 135, dtype=np.uint8), oracle.BF16),
             oracle.codebook_from_dec(np.arange(200, 216, dtype=np.uint8), oracle.BF16),
             oracle.codebook_from_dec(np.array([0, 255] + list(range(120, 134)), np.uint8), oracle.BF16)]
    for i, cb in enumerate(books):
        check_parity(g, x, cb, f"patterns/cb{i}")


def test_all_e5m2_bit_patterns():
    """every byte value, many times over in random order, under a calibrated-like, an adversarial and an extreme codebook"""
    rng = np.random.default_rng(8)
    x = rng.permutation(np.tile(np.arange(256, dtype=np.uint8), 41))[:-3].copy()
    g = Gpu(x.size, sz.FP8_E5M2)
    books = [oracle.codebook_from_dec(np.arange(7, 23, dtype=np.uint8), oracle.E5M2),
             oracle.codebook_from_dec(np.array([0, 31, 1, 30, 2, 29, 3, 28, 4, 27, 5, 26, 6, 25, 24, 23], np.uint8), oracle.E5M2),
             oracle.codebook_from_dec(np.arange(16, 32, dtype=np.uint8), oracle.E5M2)]
    for i, cb in enumerate(books):
        check_parity(g, x, cb, f"e5m2 patterns/cb{i}")


@pytest.mark.parametrize("dtype", DTYPES)
def test_all_escape_and_no_escape(dtype):
    """codebook that covers nothing (M = N, every chunk full) next to one that covers everything"""
    x = synth(dtype, 41, 3)[: 5 * 8192 + 777].copy()
    g = Gpu(x.size, dtype)
    if dtype == sz.BF16:
        none = oracle.codebook_from_dec(np.arange(230, 246, dtype=np.uint8), oracle.BF16)
    else:
        none = oracle.codebook_from_dec(np.array([0, 31, 1, 30, 2, 29, 3, 28, 4, 27, 5, 26, 6, 25, 24, 23], np.uint8),
                                        oracle.E5M2)
        x = x[(((x >> 2) & 0x1F) >= 7) & (((x >> 2) & 0x1F) <= 22)][: 3 * 8192 + 77].copy()
    total, m = check_parity(g, x, none, "all-escape")
    assert m == x.size
    cb = calibrated(dtype)
    e = ((x >> 7) & 0xFF) if dtype == sz.BF16 else ((x >> 2) & 0x1F)
    covered = x[np.isin(e, cb.dec)].copy()
    total, m = check_parity(g, covered, cb, "no-escape")
    assert m == 0
    # mixed: an all-escape chunk right next to clean ones
    y = covered[: 4 * 8192].copy()
    y[1024:2048] = 0
    y[8191] = 0
    y[8192] = 0
    check_parity(g, y, cb, "burst")


def test_escape_stress_outliers():
    """config-2 law at reduced size: 0.5 % outliers x 2^U{6..14}, 0.1 % zeros / subnormals"""
    x = kv_synth.to_numpy_words(kv_synth.kv_bf16_outliers(512, 0))
    cb = calibrated(sz.BF16)
    g = Gpu(x.size, sz.BF16)
    total, m = check_parity(g, x, cb, "outliers")
    print(f"outliers eps={m / x.size:.5f}", flush=True)
    assert m / x.size > 0.003


@pytest.mark.parametrize("dtype", DTYPES)
def test_deterministic_and_workspace_reuse(dtype):
    """same input twice -> identical stream; one workspace serves calls of different sizes in a row"""
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    x = synth(dtype, 300, 11)
    g = Gpu(x.size, dtype)
    xd = words_tensor(x)
    t1 = g.compress(xd, cb)
    a = g.out[: t1[0]].clone()
    for n in (x.size, 12345, x.size, 1, x.size):
        t = g.compress(xd[:n], cb)
        assert t[2] == 0
        if n == x.size:
            assert t == t1 and torch.equal(g.out[: t[0]], a)
        else:
            ref, _ = oracle.compress(x[:n], cb_or)
            assert np.array_equal(g.out[: t[0]].cpu().numpy(), ref)


def test_overflow_reports_needed_size():
    """escapes that do not fit: status OVERFLOW, total_bytes = size needed, nothing written past capacity"""
    x = synth(sz.BF16, 64, 3)
    none = oracle.codebook_from_dec(np.arange(230, 246, dtype=np.uint8), oracle.BF16)
    cb = gpu_codebook(none)
    g = Gpu(x.size, sz.BF16)
    xd = words_tensor(x)
    fixed = sz.fixed_bytes(x.size, sz.BF16)
    need = sz.total_bytes(x.size, x.size, sz.BF16)
    for cap in (fixed, fixed + 1000, need - 1):
        total, m, status = g.compress(xd, cb, capacity=cap)
        assert status == sz.STATUS_OVERFLOW and total == need and m == x.size
        assert (g.out[cap:cap + 4096].cpu().numpy() == POISON).all()
        # the fixed part is still the oracle's
        ref, _ = oracle.compress(x, none)
        assert np.array_equal(g.out[64:fixed].cpu().numpy(), ref[64:fixed])
    total, m, status = g.compress(xd, cb, capacity=need)
    assert status == 0 and total == need


def test_bad_stream_is_flagged_not_followed():
    x = synth(sz.BF16, 16, 3).copy()
    x[5] = 0
    x[9000] = 0x7F80
    cb_or = calibrated(sz.BF16)
    cb = gpu_codebook(cb_or)
    blob, m = oracle.compress(x, cb_or)
    g = Gpu(x.size, sz.BF16)
    n = x.size

    def run(mut):
        b = blob.copy()
        mut(b)
        y, (_, _, st) = g.decompress(torch.from_numpy(b).cuda(), b.size, n, cb)
        return y, st

    def set_(i, v):
        def f(b):
            b[i] = v
        return f

    y, st = run(lambda b: None)
    assert st == 0 and np.array_equal(y, x)
    for mut in (set_(0, 0x58), set_(6, 1), set_(16, int(blob[16]) ^ 1), set_(40, int(blob[40]) ^ 1)):
        y, st = run(mut)                     # header disagrees: flagged
        assert st & sz.STATUS_BAD_STREAM
    off_pos = blob.size - m - (2 * m + 255) // 256 * 256
    y, st = run(set_(off_pos + 1, 0xFF))     # position outside the chunk: skipped and flagged
    assert st & sz.STATUS_BAD_STREAM
    c = (n + 1023) // 1024
    y, st = run(set_(64 + 4 * c + 3, 0x7F))  # M in the offset table far beyond the stream
    assert st & sz.STATUS_BAD_STREAM

    # positions inside a chunk must ascend (the oracle's decoder rejects such a stream; the GPU's flags it): a chunk
    # with two escapes, a chunk with a few (corrected in registers) and one with many (corrected in the LDS tile)
    x2 = synth(sz.BF16, 16, 3).copy()
    x2[[7, 300]] = 0                          # chunk 0: two escapes
    x2[3 * 1024: 3 * 1024 + 200: 2] = 0       # chunk 3: a hundred of them
    blob2, m2 = oracle.compress(x2, cb_or)
    off_pos2 = blob2.size - m2 - (2 * m2 + 255) // 256 * 256
    tab2 = blob2[64:64 + 4 * (c + 1)].view(np.uint32)

    def swap(j):                               # records j and j + 1 change places (positions only)
        def f(b):
            p = b[off_pos2:off_pos2 + 2 * m2].view(np.uint16)
            p[j], p[j + 1] = p[j + 1], p[j]
        return f

    def dup(j):                                # record j + 1 repeats the position of record j
        def f(b):
            p = b[off_pos2:off_pos2 + 2 * m2].view(np.uint16)
            p[j + 1] = p[j]
        return f

    def run2(mut):
        b = blob2.copy()
        mut(b)
        with pytest.raises(ValueError):
            oracle.decompress(b, n, cb_or)
        y, (_, _, st) = g.decompress(torch.from_numpy(b).cuda(), b.size, n, cb)
        return st

    assert tab2[1] - tab2[0] >= 2 and tab2[4] - tab2[3] >= 100
    for mut in (swap(int(tab2[0])), dup(int(tab2[0])), swap(int(tab2[3]) + 10), dup(int(tab2[3]) + 70), swap(int(tab2[3]) + 63)):
        assert run2(mut) & sz.STATUS_BAD_STREAM


@pytest.mark.parametrize("dtype", DTYPES)
def test_batch_calls_match_the_oracle_item_by_item(dtype):
    """one batch launch over tensors of mixed sizes (empty, ragged, all-escape, several ranges), nearly every one
    with a codebook of its own: every stream is the oracle's, every tensor comes back"""
    es = 2 if dtype == sz.BF16 else 1
    cbs_or = [calibrated(dtype, kind="K"), calibrated(dtype, kind="V")]
    if dtype == sz.BF16:
        cbs_or.append(oracle.codebook_from_dec(np.arange(230, 246, dtype=np.uint8), oracle.BF16))
    else:
        cbs_or.append(oracle.codebook_from_dec(np.array([0, 31, 1, 30, 2, 29, 3, 28, 4, 27, 5, 26, 6, 25, 24, 23], np.uint8), oracle.E5M2))
    sizes = [300 * 1024, 0, 1, 8191, 123457, 64 * 1024, 1025, 700 * 1024 + 5, 2048, 40000, 17, 256 * 1024]
    xs_np, books = [], []
    for k, n in enumerate(sizes):
        x = synth(dtype, (n + 1023) // 1024 + 1, 20 + k, layer=k % 3, kind="KV"[k % 2])[:n].copy()
        if k % 4 == 3 and n:
            x[:: max(1, n // 50)] = 0
        xs_np.append(x)
        books.append(cbs_or[2] if k in (5, 10) else cbs_or[k % 2] if k < 4 else calibrated(dtype, seed=3 + k, tokens=256, layer=k, kind="KV"[k % 2]))
    gbooks = [gpu_codebook(c) for c in books]
    xs = [words_tensor(x) for x in xs_np]
    outs = [torch.full((sz.compress_bound(x.size, dtype) + 512,), POISON, dtype=torch.uint8, device="cuda") for x in xs_np]
    ws = sz.Workspace(max(sizes), dtype)
    rec = sz.new_sizes_array(len(xs))
    rec.fill_(-1)
    batch = sz.CompressBatch(xs, gbooks, outs)
    for rep in range(2):                                   # the second launch re-uses the workspace
        batch.launch(ws, rec)
        torch.cuda.synchronize()
        got = sz.read_sizes_array(rec)
        for k, x in enumerate(xs_np):
            ref, m = oracle.compress(x, books[k])
            total, gm, status = got[k]
            assert (total, gm, status) == (ref.size, m, 0), f"item {k}: {got[k]} vs {(ref.size, m)}"
            blob = outs[k][:total].cpu().numpy()
            assert np.array_equal(blob, ref), f"item {k} (n={x.size}): stream differs from the oracle's"
            assert (outs[k][total:total + 256].cpu().numpy() == POISON).all()
    # and back, in one launch
    ys = [torch.full((x.size + 64,), 0x5A5A if es == 2 else 0x5A, dtype=torch.int16 if es == 2 else torch.uint8, device="cuda")
          for x in xs_np]
    st = sz.new_sizes()
    sz.decompress_batch(outs, [g[0] for g in got], [x.size for x in xs_np], gbooks, ys, st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0
    for k, x in enumerate(xs_np):
        y = ys[k].cpu().numpy()
        y = y.view(np.uint16) if es == 2 else y
        assert np.array_equal(y[: x.size], x), f"item {k}: batch round trip differs"
        assert (ys[k][x.size:].cpu().numpy() == (0x5A if es == 1 else 0x5A5A)).all()


@pytest.mark.parametrize("dtype", DTYPES)
def test_device_histogram_matches_the_oracle_calibration(dtype):
    """exponent counts of device samples, ragged sizes included, accumulated over several calls; the codebook
    built from them is the oracle's"""
    total = np.zeros(256, np.int64)
    hist = None
    parts = []
    for k, n in enumerate((0, 1, 7, 16, 1000, 8191, 300 * 1024 + 13, 1024 * 1024)):
        x = synth(dtype, (n + 1023) // 1024 + 1, 30 + k, layer=k % 4, kind="KV"[k % 2])[:n].copy()
        if n > 100:
            x[:: 97] = 0                                    # zeros and a few maximal exponents
            x[5:: 1013] = 0x7F80 if dtype == sz.BF16 else 0x7C
        parts.append(x)
        ref = oracle.calibrate(x, DT[dtype])
        one = sz.histogram(words_tensor(x) if n else torch.zeros(0, dtype=torch.int16 if dtype == sz.BF16 else torch.uint8, device="cuda"), dtype)
        torch.cuda.synchronize()
        assert one.cpu().tolist() == ref.hist.tolist(), f"n={n}"
        if n:
            hist = sz.histogram(words_tensor(x), dtype, hist)
        total += ref.hist.astype(np.int64)
    torch.cuda.synchronize()
    assert hist.cpu().tolist() == total.tolist()
    ref_all = oracle.calibrate(np.concatenate(parts), DT[dtype])
    cb = sz.codebook_from_hist(hist.cpu(), dtype)
    assert cb.dec == ref_all.dec.tolist() and cb.enc == ref_all.enc.tolist() and cb.member == ref_all.member.tolist()


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """compress + decompress (single and batch) captured once, replayed with new data between the replays and
    the library's own eager calls in between: every replay must give the oracle's streams.  The exchange
    words are tagged from a counter in the workspace, so a replay never mistakes an earlier launch's words
    for its own."""
    dtype = sz.BF16
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    n = 300 * 1024 + 77
    datas = [synth(dtype, 301, 40 + r)[:n].copy() for r in range(3)]
    for d in datas:
        d[:: 1231] = 0
    x = words_tensor(datas[0])
    x2 = words_tensor(datas[0][: 70000].copy())
    ws = sz.Workspace(n, dtype)
    outs = [torch.zeros(sz.compress_bound(n, dtype), dtype=torch.uint8, device="cuda") for _ in range(3)]
    y = torch.zeros_like(x)
    rec1, rec2, dst = sz.new_sizes(), sz.new_sizes_array(2), sz.new_sizes()
    batch = sz.CompressBatch([x, x2], [cb, cb], outs[1:])
    ref0, m0 = oracle.compress(datas[0], cb_or)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        sz.compress(x, cb, outs[0], ws, rec1)              # warm-up outside the capture
        torch.cuda.current_stream().synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            sz.compress(x, cb, outs[0], ws, rec1)
            batch.launch(ws, rec2)
            sz.decompress(outs[0], ref0.size + 4096, n, cb, y, dst)   # comp_bytes: a bound, the header holds the size
    torch.cuda.synchronize()
    for rep, d in enumerate(datas + datas[:1]):
        x.copy_(words_tensor(d))
        x2.copy_(words_tensor(d[: 70000].copy()))
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        ref, m = oracle.compress(d, cb_or)
        ref2, mm2 = oracle.compress(d[: 70000].copy(), cb_or)
        assert sz.read_sizes(rec1) == (ref.size, m, 0), f"replay {rep}"
        assert np.array_equal(outs[0][: ref.size].cpu().numpy(), ref), f"replay {rep}: single call stream"
        got = sz.read_sizes_array(rec2)
        assert got == [(ref.size, m, 0), (ref2.size, mm2, 0)], f"replay {rep}: {got}"
        assert np.array_equal(outs[1][: ref.size].cpu().numpy(), ref) and np.array_equal(outs[2][: ref2.size].cpu().numpy(), ref2)
        assert sz.read_sizes(dst)[2] == 0 and torch.equal(y, x), f"replay {rep}: round trip"
        # eager work of the library between the replays
        sz.compress(x2, cb, outs[2], ws, rec1)
        torch.cuda.synchronize()
        assert sz.read_sizes(rec1) == (ref2.size, mm2, 0)


@pytest.mark.parametrize("dtype", DTYPES)
def test_codebook_that_never_leaves_the_device(dtype):
    """device histogram -> device ranking -> compress / decompress with the device codebook: tables, stream and
    tensor are those of the oracle calibrated on the same sample (ties and unseen exponents included)"""
    n = 200 * 1024 + 321
    x = synth(dtype, 201, 50)[:n].copy()
    x[:: 777] = 0
    sample = x[: 40000].copy()
    sample[:5] = (0x7F80 if dtype == sz.BF16 else 0x7C)            # a rare exponent with a small count
    ref_cb = oracle.calibrate(sample, DT[dtype])
    hist = sz.histogram(words_tensor(sample), dtype)
    dcb = sz.codebook_device(hist, dtype)
    torch.cuda.synchronize()
    host = dcb.to_host()
    assert (host.dec, host.enc, host.member, host.dtype) == (ref_cb.dec.tolist(), ref_cb.enc.tolist(), ref_cb.member.tolist(), dtype)
    # a histogram with ties and fewer than 16 exponents seen
    h = torch.zeros(256, dtype=torch.int64)
    h[20] = h[9] = h[11] = 5
    h[15] = 9
    tied = sz.codebook_device(h.cuda(), dtype).to_host()
    assert tied.dec == sz.codebook_from_hist(h, dtype).dec == [15, 9, 11, 20, 0, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 13]
    # compress and decompress with it
    ref, m = oracle.compress(x, ref_cb)
    g = Gpu(n, dtype)
    g.out.fill_(POISON)
    xd = words_tensor(x)
    sz.compress_dcb(xd, dcb, g.out, g.ws, g.sizes)
    torch.cuda.synchronize()
    assert sz.read_sizes(g.sizes) == (ref.size, m, 0)
    assert np.array_equal(g.out[: ref.size].cpu().numpy(), ref), "stream differs from the oracle's"
    y = torch.zeros_like(xd)
    st = sz.new_sizes()
    sz.decompress_dcb(g.out, ref.size, n, dcb, y, st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0 and torch.equal(y, xd)


@pytest.mark.parametrize("dtype", DTYPES)
def test_batch_calibrated_on_the_device(dtype):
    """a codebook per tensor, counted and ranked on the device for the whole batch, then the batch calls under those
    codebooks: tables, streams and tensors are those of the oracle calibrated on each tensor itself"""
    sizes = [300 * 1024 + 5, 1, 0, 64 * 1024, 123457, 2048, 700 * 1024, 17]
    xs_np = []
    for k, n in enumerate(sizes):
        x = synth(dtype, (n + 1023) // 1024 + 1, 70 + k, layer=3 * k, kind="KV"[k % 2])[:n].copy()
        if k == 3:
            x[:] = x[0]                                    # one exponent only: fifteen unseen ones fill the codebook
        xs_np.append(x)
    xs = [words_tensor(x) for x in xs_np]
    dcbs = sz.DeviceCodebooks(len(xs), dtype)
    dcbs.hists.fill_(7)                                    # the call zeroes the counts itself
    sz.CalibrateBatchDevice(xs, dcbs).launch()
    outs = [torch.full((sz.compress_bound(x.size, dtype) + 512,), POISON, dtype=torch.uint8, device="cuda") for x in xs_np]
    ws = sz.Workspace(max(sizes), dtype)
    rec = sz.new_sizes_array(len(xs))
    sz.CompressBatchDcb(xs, dcbs, outs, capacities=[o.numel() - 512 for o in outs]).launch(ws, rec)
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    refs = []
    for k, x in enumerate(xs_np):
        print(f"case device-calibrated batch dtype={dtype} item {k} n={x.size}", flush=True)
        cb_or = oracle.calibrate(x, DT[dtype])
        host = dcbs.to_host(k)
        assert (host.dec, host.enc, host.member, host.dtype) == (cb_or.dec.tolist(), cb_or.enc.tolist(), cb_or.member.tolist(), dtype), f"item {k}: tables"
        ref, m = oracle.compress(x, cb_or)
        refs.append(ref)
        assert got[k] == (ref.size, m, 0), (k, got[k], ref.size, m)
        assert np.array_equal(outs[k][: ref.size].cpu().numpy(), ref), f"item {k}: stream differs from the oracle's"
        assert (outs[k][ref.size: ref.size + 512].cpu().numpy() == POISON).all()
    ys = [torch.zeros(max(x.size, 1), dtype=t.dtype, device="cuda") for x, t in zip(xs_np, xs)]
    st = sz.new_sizes()
    sz.DecompressBatchDcb(outs, [r.size for r in refs], [x.size for x in xs_np], dcbs, ys).launch(st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0
    for x, y, t in zip(xs_np, ys, xs):
        assert torch.equal(y[: x.size], t), "round trip differs"
    # a receiver without the codebooks: every stream decoded under the entries of its own header, batch and single
    for y in ys:
        y.fill_(0x55)
    st2 = sz.new_sizes()
    sz.DecompressBatchOwn(outs, [r.size for r in refs], [x.size for x in xs_np], dtype, ys).launch(st2)
    torch.cuda.synchronize()
    assert sz.read_sizes(st2)[2] == 0
    for k, (x, y, t) in enumerate(zip(xs_np, ys, xs)):
        assert torch.equal(y[: x.size], t), f"item {k}: decoded under its own header"
        y.fill_(0x55)
        st3 = sz.new_sizes()
        sz.decompress_own(outs[k], refs[k].size, x.size, dtype, y, st3)
        torch.cuda.synchronize()
        assert sz.read_sizes(st3) == (refs[k].size, got[k][1], 0) and torch.equal(y[: x.size], t), f"item {k}: single call"


@pytest.fixture
def hooks():
    """the library's test hooks (small staging and status areas); off again afterwards"""
    yield sz.internal_test_hooks
    sz.internal_test_hooks()


def test_compress_beside_other_work_on_the_device():
    """The compress calls wait for nothing -- no workgroup for another, no launch for room on the device: with a
    long run of elementwise kernels keeping the device busy on another stream (what a prefill worker's model does
    beside the codec), single and batch calls complete and give the streams they give on a quiet device."""
    dtype = sz.BF16
    n = 8 * 1024 * 1024
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    xs = [kv_synth.kv_bf16(n // 1024, 0, layer, "K", device="cuda") for layer in range(6)]
    refs = [oracle.compress(kv_synth.to_numpy_words(x), cb_or) for x in xs[:2]]
    outs = [torch.empty(sz.compress_bound(n, dtype), dtype=torch.uint8, device="cuda") for _ in xs]
    quiet = [torch.empty_like(o) for o in outs]
    ws = sz.Workspace(n, dtype)
    rec, rec_q, one = sz.new_sizes_array(len(xs)), sz.new_sizes_array(len(xs)), sz.new_sizes()
    sz.compress_batch(xs, [cb] * len(xs), quiet, ws, rec_q)
    torch.cuda.synchronize()
    want = sz.read_sizes_array(rec_q)
    busy = torch.ones(1 << 29, dtype=torch.float32, device="cuda")          # 2 GiB: each pass over it takes about a millisecond
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(40):
            busy.mul_(1.0001)
    for rep in range(10):
        sz.compress_batch(xs, [cb] * len(xs), outs, ws, rec)
        sz.compress(xs[0], cb, outs[0], ws, one)
    done_first = not side.query()                                            # the side stream is still busy: the calls ran beside it
    torch.cuda.synchronize()
    assert sz.read_sizes_array(rec) == want and sz.read_sizes(one) == want[0]
    for k in range(len(xs)):
        assert torch.equal(outs[k][: want[k][0]], quiet[k][: want[k][0]]), f"tensor {k} differs beside other work"
    for k, (ref, m) in enumerate(refs):
        assert want[k] == (ref.size, m, 0) and np.array_equal(outs[k][: ref.size].cpu().numpy(), ref)
    print("codec calls enqueued while the side stream was still running:", done_first, flush=True)


def test_two_compress_calls_on_two_streams_at_once():
    """two single-tensor compress calls, each with its own workspace, may run side by side on two streams (streams and
    results as in the serial case)"""
    n = 32768 * 1024 // 4
    cb_or = calibrated(sz.BF16)
    cb = gpu_codebook(cb_or)
    xs = [kv_synth.kv_bf16(n // 1024, 0, layer, "K", device="cuda") for layer in (2, 5)]
    refs = [oracle.compress(kv_synth.to_numpy_words(x), cb_or) for x in xs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [sz.Workspace(n, sz.BF16) for _ in range(2)]
    outs = [torch.empty(sz.compress_bound(n, sz.BF16), dtype=torch.uint8, device="cuda") for _ in range(2)]
    recs = [sz.new_sizes() for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(20):
        for k in range(2):
            sz.compress(xs[k], cb, outs[k], wss[k], recs[k], stream=streams[k])
    torch.cuda.synchronize()
    for k in range(2):
        ref, m = refs[k]
        assert sz.read_sizes(recs[k]) == (ref.size, m, 0)
        assert np.array_equal(outs[k][: ref.size].cpu().numpy(), ref)


@pytest.mark.parametrize("dtype", [sz.BF16, sz.FP8_E5M2])
def test_escape_values_beyond_the_staging_area(hooks, dtype):
    """a staging area of 4 KB: the slots of the tiles hold a record or two (none at all in the batch call, which
    shares the area between its tensors), so the finishing pass encodes most tiles once more from the words; the stream
    must still be the oracle's"""
    hooks(stage_bytes=4096)
    x = synth(dtype, 5 * 1024 + 3, 4)[:-517].copy()
    x[::997] = 0
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    ref, m = oracle.compress(x, cb_or)
    assert m > 1000
    out = torch.full((sz.compress_bound(x.size, dtype) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = sz.Workspace(x.size, dtype)
    sizes = sz.new_sizes()
    xd = words_tensor(x)
    for rep in range(2):
        sz.compress(xd, cb, out, ws, sizes)
        torch.cuda.synchronize()
        assert sz.read_sizes(sizes) == (ref.size, m, 0), (sz.read_sizes(sizes), ref.size, m)
        assert np.array_equal(out[: ref.size].cpu().numpy(), ref), "stream differs"
        assert (out[ref.size:].cpu().numpy() == 0xA5).all()
    small = [x[:70000].copy(), x[100:100 + 1025].copy()]
    xs = [words_tensor(small[0]), xd, words_tensor(small[1])]
    outs = [torch.empty(sz.compress_bound(t.numel(), dtype), dtype=torch.uint8, device="cuda") for t in xs]
    rec = sz.new_sizes_array(3)
    sz.compress_batch(xs, [cb] * 3, outs, ws, rec)
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    for k, src in enumerate((small[0], x, small[1])):
        r, mm = oracle.compress(src, cb_or)
        assert got[k] == (r.size, mm, 0), (k, got[k], r.size, mm)
        assert np.array_equal(outs[k][: r.size].cpu().numpy(), r), f"batch item {k} differs"


@pytest.mark.parametrize("dtype", [sz.BF16, sz.FP8_E5M2])
def test_batch_that_takes_several_launches(hooks, dtype):
    """a status area of 512 bytes holds the tile counts of a few of these tensors at a time (and only with larger tiles
    for the largest): the batch call splits into launches; every stream must still be the oracle's"""
    hooks(status_bytes=512)
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    sizes_tok = [40, 3, 700, 0, 129, 64, 1]
    xs_np = [synth(dtype, max(t, 1), 10 + k)[: t * 1024 - (k * 37 if t else 0)].copy() if t else synth(dtype, 1, 3)[:0].copy()
             for k, t in enumerate(sizes_tok)]
    xs = [words_tensor(x) if x.size else torch.empty(0, dtype=torch.int16 if dtype == sz.BF16 else torch.uint8, device="cuda") for x in xs_np]
    outs = [torch.empty(sz.compress_bound(x.size, dtype), dtype=torch.uint8, device="cuda") for x in xs_np]
    ws = sz.Workspace(max(x.size for x in xs_np), dtype)
    rec = sz.new_sizes_array(len(xs))
    for rep in range(2):
        sz.compress_batch(xs, [cb] * len(xs), outs, ws, rec)
        torch.cuda.synchronize()
        got = sz.read_sizes_array(rec)
        for k, x in enumerate(xs_np):
            r, mm = oracle.compress(x, cb_or)
            assert got[k] == (r.size, mm, 0), (k, got[k], r.size, mm)
            assert np.array_equal(outs[k][: r.size].cpu().numpy(), r), f"item {k} differs"


@pytest.mark.parametrize("dtype", [sz.BF16, sz.FP8_E5M2])
@pytest.mark.parametrize("groups,stage,direct", [(2, 0, 0), (4, 0, 1), (4, 8192, 0), (1, 0, 1), (2, 8192, 1)])
def test_finishing_pass_with_several_groups_per_workgroup(hooks, dtype, groups, stage, direct):
    """Large launches give every workgroup of the finishing pass two or four groups of 16 tiles; forced here on a
    batch of tensors whose group counts are everything but multiples of four (none, one, a group and a tile, ...),
    once with a staging area so small that tiles are encoded again by the finishing pass; direct = 1: the finishing
    pass is given sums of 64 tile counts (as in large launches) instead of reading the counts itself"""
    hooks(finish_groups=groups, stage_bytes=stage, direct_bytes=direct)
    cb_or = calibrated(dtype)
    cb = gpu_codebook(cb_or)
    per_group = 128 if dtype == sz.BF16 else 256     # chunks per group of 16 tiles
    chunks = [11 * per_group - 60, per_group - 1, per_group, per_group + 1, 1, 0, 4 * per_group + 9, 8 * per_group, 3]
    xs_np = []
    for k, c in enumerate(chunks):
        n = max(c * 1024 - (k * 53 if c else 0), 0)
        xs_np.append(synth(dtype, max(c, 1), 20 + k)[:n].copy())
    xs = [words_tensor(x) if x.size else torch.empty(0, dtype=torch.int16 if dtype == sz.BF16 else torch.uint8, device="cuda") for x in xs_np]
    outs = [torch.empty(sz.compress_bound(x.size, dtype), dtype=torch.uint8, device="cuda") for x in xs_np]
    ws = sz.Workspace(max(x.size for x in xs_np), dtype)
    rec = sz.new_sizes_array(len(xs))
    for rep in range(2):
        for o in outs:
            o.fill_(POISON)
        sz.compress_batch(xs, [cb] * len(xs), outs, ws, rec)
        torch.cuda.synchronize()
        got = sz.read_sizes_array(rec)
        for k, x in enumerate(xs_np):
            r, mm = oracle.compress(x, cb_or)
            assert got[k] == (r.size, mm, 0), (k, got[k], r.size, mm)
            assert np.array_equal(outs[k][: r.size].cpu().numpy(), r), f"item {k} differs"
    # and a single call, where the groups of one tensor are all there is
    one = sz.new_sizes()
    sz.compress(xs[0], cb, outs[0], ws, one)
    torch.cuda.synchronize()
    r, mm = oracle.compress(xs_np[0], cb_or)
    assert sz.read_sizes(one) == (r.size, mm, 0)
    assert np.array_equal(outs[0][: r.size].cpu().numpy(), r)


def test_tensor_of_many_chain_segments():
    """307 M BF16 elements (586 MiB, ragged): 37 500 tiles, so the finishing pass reads sums of 64 tile counts instead
    of every count; the offset table alone is 1.2 MB"""
    x_dev = kv_synth.kv_bf16(300007, 5, 9, "V", device="cuda")
    x = kv_synth.to_numpy_words(x_dev)[:-517].copy()
    del x_dev
    torch.cuda.empty_cache()
    g = Gpu(x.size, sz.BF16)
    total, m = check_parity(g, x, calibrated(sz.BF16, kind="V"), "large")
    print(f"large: n={x.size} eps={m / x.size:.5f} ratio={2 * x.size / total:.4f}", flush=True)


def test_escape_stress_full_size():
    """config 2 at its real tensor size [16384, 8, 128]: ~0.7 % escapes, bursts included"""
    x = kv_synth.to_numpy_words(kv_synth.kv_bf16_outliers(16384, 0, 3, device="cuda"))
    cb = calibrated(sz.BF16)
    g = Gpu(x.size, sz.BF16)
    total, m = check_parity(g, x, cb, "config2 L3")
    print(f"config2 L3: eps={m / x.size:.5f} ratio={2 * x.size / total:.4f}", flush=True)
    assert 0.004 < m / x.size < 0.05


def test_streaming_chunk_shape():
    """config 3's call shape: [2048, 8, 128] K and V of a deep layer, per-kind codebooks"""
    g = Gpu(2048 * 1024, sz.BF16)
    for layer, kind in ((79, "K"), (40, "V")):
        cb = calibrated(sz.BF16, seed=1, tokens=1024, layer=0, kind=kind)
        x = synth(sz.BF16, 2048, 0, layer, kind)
        check_parity(g, x, cb, f"config3 L{layer}{kind}")


def test_full_size_e5m2_tensor():
    """config 4 at its real tensor size [32768, 8, 128] E5M2 (32 MiB): V of layer 17"""
    n = 32768 * 1024
    g = Gpu(n, sz.FP8_E5M2)
    cb_or = calibrated(sz.FP8_E5M2, seed=1, tokens=1024, layer=0, kind="V")
    x = kv_synth.to_numpy_words(kv_synth.kv_e5m2(32768, 0, 17, "V", device="cuda"))
    total, m = check_parity(g, x, cb_or, "config4 L17V")
    print(f"config4 L17V: eps={m / n:.5f} ratio={n / total:.4f}", flush=True)


def test_full_size_tensors_of_the_benchmark_workload():
    """config 1 at its real tensor size [32768, 8, 128] (64 MiB), K of layer 0 and V of layer 31, with the
    per-kind codebooks from a seed-1 1024-token sample; whole stream and round trip compared."""
    n = 32768 * 1024
    g = Gpu(n, sz.BF16)
    for layer, kind in ((0, "K"), (31, "V")):
        cb_or = calibrated(sz.BF16, seed=1, tokens=1024, layer=0, kind=kind)
        x_dev = kv_synth.kv_bf16(32768, 0, layer, kind, device="cuda")
        x = kv_synth.to_numpy_words(x_dev)
        total, m = check_parity(g, x, cb_or, f"config1 L{layer}{kind}")
        print(f"config1 L{layer}{kind}: eps={m / n:.5f} ratio={2 * n / total:.4f}", flush=True)


@pytest.mark.parametrize("dtype", DTYPES)
def test_full_size_tensors_through_the_batch_calls(dtype):
    """the launch configuration the benchmark times, at its real tensor size: four [32768, 8, 128] tensors (K and V of
    two layers, per-kind codebooks) in one batch launch each way; every stream is the oracle's, byte for byte"""
    es = 2 if dtype == sz.BF16 else 1
    gen = kv_synth.kv_bf16 if dtype == sz.BF16 else kv_synth.kv_e5m2
    n = 32768 * 1024
    cbs_or = {k: calibrated(dtype, seed=1, tokens=1024, layer=0, kind=k) for k in "KV"}
    gcb = {k: gpu_codebook(c) for k, c in cbs_or.items()}
    items = [(0, "K"), (0, "V"), (31, "K"), (31, "V")]
    xs = [gen(32768, 0, layer, kind, device="cuda") for layer, kind in items]
    outs = [torch.full((sz.total_bytes(n, n // 20, dtype) + 512,), POISON, dtype=torch.uint8, device="cuda") for _ in items]
    ws = sz.Workspace(n, dtype)
    rec = sz.new_sizes_array(len(items))
    sz.compress_batch(xs, [gcb[k] for _, k in items], outs, ws, rec, capacities=[o.numel() - 512 for o in outs])
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    for i, (layer, kind) in enumerate(items):
        print(f"case full-size batch dtype={dtype} L{layer}{kind}", flush=True)
        ref, m = oracle.compress(kv_synth.to_numpy_words(xs[i]), cbs_or[kind])
        assert got[i] == (ref.size, m, 0), (i, got[i], ref.size, m)
        assert np.array_equal(outs[i][:ref.size].cpu().numpy(), ref), f"L{layer}{kind}: batch stream differs from the oracle's"
        assert (outs[i][ref.size:ref.size + 512].cpu().numpy() == POISON).all()
    ys = [torch.empty_like(x) for x in xs]
    st = sz.new_sizes()
    sz.decompress_batch(outs, [g[0] for g in got], [n] * len(items), [gcb[k] for _, k in items], ys, st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0
    for x, y in zip(xs, ys):
        assert torch.equal(x, y), "batch round trip differs"


def test_batch_tensor_larger_than_a_full_group():
    """an E5M2 tensor of 70 Mi elements has more chunks than the largest group the batch kernel forms can share at 64
    per workgroup: the grid is cut down to one group of that size; a small tensor rides in the same launch"""
    dtype = sz.FP8_E5M2
    cb_or = calibrated(dtype, seed=1, tokens=1024, layer=0, kind="K")
    cb = gpu_codebook(cb_or)
    xs = [kv_synth.kv_e5m2(70 * 1024, 0, 5, "K", device="cuda"), kv_synth.kv_e5m2(300, 0, 6, "K", device="cuda")[:-77].contiguous()]
    outs = [torch.full((sz.total_bytes(x.numel(), x.numel() // 20, dtype) + 512,), POISON, dtype=torch.uint8, device="cuda") for x in xs]
    ws = sz.Workspace(xs[0].numel(), dtype)
    rec = sz.new_sizes_array(2)
    sz.compress_batch(xs, [cb, cb], outs, ws, rec, capacities=[o.numel() - 512 for o in outs])
    torch.cuda.synchronize()
    got = sz.read_sizes_array(rec)
    ys = [torch.empty_like(x) for x in xs]
    st = sz.new_sizes()
    sz.decompress_batch(outs, [g[0] for g in got], [x.numel() for x in xs], [cb, cb], ys, st)
    torch.cuda.synchronize()
    assert sz.read_sizes(st)[2] == 0
    for i, x in enumerate(xs):
        ref, m = oracle.compress(kv_synth.to_numpy_words(x), cb_or)
        assert got[i] == (ref.size, m, 0), (i, got[i], ref.size, m)
        assert np.array_equal(outs[i][:ref.size].cpu().numpy(), ref), f"item {i}: stream differs from the oracle's"
        assert torch.equal(x, ys[i])


def test_more_tensors_than_one_launch_takes():
    """70 small tensors: the batch calls (host codebooks, device codebooks, own headers) split them over two launches
    of at most 64; every stream is the oracle's under the tensor's own codebook"""
    dtype = sz.BF16
    rng = np.random.default_rng(11)
    xs_np = [synth(dtype, 3, 200 + k, layer=k, kind="KV"[k % 2])[: int(rng.integers(1, 3000))].copy() for k in range(70)]
    xs = [words_tensor(x) for x in xs_np]
    cbs_or = [oracle.calibrate(x, DT[dtype]) for x in xs_np]
    refs = [oracle.compress(x, c) for x, c in zip(xs_np, cbs_or)]
    ws = sz.Workspace(4096, dtype)
    dcbs = sz.DeviceCodebooks(70, dtype)
    sz.CalibrateBatchDevice(xs, dcbs).launch()
    for how in ("host codebooks", "device codebooks"):
        outs = [torch.full((sz.compress_bound(x.size, dtype),), POISON, dtype=torch.uint8, device="cuda") for x in xs_np]
        rec = sz.new_sizes_array(70)
        if how == "host codebooks":
            sz.compress_batch(xs, [gpu_codebook(c) for c in cbs_or], outs, ws, rec)
        else:
            sz.CompressBatchDcb(xs, dcbs, outs).launch(ws, rec)
        torch.cuda.synchronize()
        got = sz.read_sizes_array(rec)
        for k, (ref, m) in enumerate(refs):
            assert got[k] == (ref.size, m, 0), (how, k, got[k], ref.size, m)
            assert np.array_equal(outs[k][: ref.size].cpu().numpy(), ref), f"{how}: item {k} differs from the oracle's stream"
        ys = [torch.zeros_like(t) for t in xs]
        st = sz.new_sizes()
        if how == "host codebooks":
            sz.DecompressBatchOwn(outs, [r[0].size for r in refs], [x.size for x in xs_np], dtype, ys).launch(st)
        else:
            sz.DecompressBatchDcb(outs, [r[0].size for r in refs], [x.size for x in xs_np], dcbs, ys).launch(st)
        torch.cuda.synchronize()
        assert sz.read_sizes(st)[2] == 0
        for k, (y, t) in enumerate(zip(ys, xs)):
            assert torch.equal(y, t), f"{how}: item {k} round trip"
