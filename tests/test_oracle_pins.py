"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
without any reference to the GPU path.  Run with -m "not gpu".

Each test names the statement of the paper it checks.  Expected values come
from the paper, from hand-assembled examples in tests/golden, from closed
forms, or from brute force written independently here in numpy.
"""
import os

import numpy as np
import pytest

import kv_synth
import oracle

BF16, E5M2 = oracle.BF16, oracle.E5M2


# --------------------------------------------------------------------------
# helpers that do NOT use the oracle
# --------------------------------------------------------------------------

def a256(x):
    return (x + 255) // 256 * 256


def bf16_fields_from_float_semantics(words):
    """sign / biased exponent / 7-bit mantissa of BF16 words from their VALUE
    (IEEE-754 binary32 with the low 16 bits dropped), via frexp -- no shifts of
    the encoding.  Only for finite normal numbers."""
    v = (words.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    sign = np.signbit(v).astype(np.uint8)
    frac, ex = np.frexp(np.abs(v))          # |v| = frac * 2**ex, frac in [0.5, 1)
    biased = ex - 1 + 127
    mant = np.rint((frac * 2.0 - 1.0) * 128.0).astype(np.int64)
    return sign, biased, mant


def parse_stream(blob, dtype):
    """Independent numpy parser of the stream layout."""
    assert bytes(blob[:4]) == b"SZP1"
    n = int(blob[16:24].view(np.uint64)[0])
    m = int(blob[24:32].view(np.uint64)[0])
    total = int(blob[32:40].view(np.uint64)[0])
    c = (n + 1023) // 1024
    sm_bytes = n if dtype == BF16 else (3 * n + 7) // 8
    o_tab = 64
    o_sm = a256(o_tab + 4 * (c + 1))
    o_code = o_sm + a256(sm_bytes)
    o_pos = o_code + a256((n + 1) // 2)
    o_val = o_pos + a256(2 * m)
    d = dict(n=n, m=m, total=total, c=c, dec=blob[40:56].copy(),
             chunk_off=blob[o_tab:o_tab + 4 * (c + 1)].copy().view(np.uint32),
             sm=blob[o_sm:o_sm + sm_bytes], code=blob[o_code:o_code + (n + 1) // 2],
             pos=blob[o_pos:o_pos + 2 * m].copy().view(np.uint16), val=blob[o_val:o_val + m],
             pads=[blob[o_tab + 4 * (c + 1):o_sm], blob[o_sm + sm_bytes:o_code],
                   blob[o_code + (n + 1) // 2:o_pos], blob[o_pos + 2 * m:o_val], blob[56:64], blob[12:16]],
             end=o_val + m)
    return d


def exponents_np(words, dtype):
    if dtype == BF16:
        return ((words >> 7) & 0xFF).astype(np.uint8)
    return ((words >> 2) & 0x1F).astype(np.uint8)


def read_golden(path):
    dec = words = None
    blob = []
    in_blob = False
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("dec:"):
            dec = [int(t) for t in line[4:].split()]
        elif line.startswith("words:"):
            words = [int(t, 16) for t in line[6:].split()]
        elif line.startswith("blob:"):
            in_blob = True
        elif in_blob and line.startswith("zeros"):
            blob += [0] * int(line.split()[1])          # "zeros n": n pad bytes
        elif in_blob:
            blob += [int(t, 16) for t in line.split()]
    return np.array(dec, np.uint8), words, np.array(blob, np.uint8)


SEQ_BF16 = np.array([127, 126, 128, 125, 129, 124, 130, 123, 131, 122, 132, 121, 133, 120, 134, 119], np.uint8)
SEQ_E5M2 = np.array([15, 14, 16, 13, 17, 12, 18, 11, 19, 10, 20, 9, 21, 8, 22, 7], np.uint8)


def codebooks(dtype):
    """calibrated-like, adversarial (nothing common covered), and one holding the extreme exponents"""
    if dtype == BF16:
        return [oracle.codebook_from_dec(SEQ_BF16, BF16),
                oracle.codebook_from_dec(np.arange(200, 216, dtype=np.uint8), BF16),
                oracle.codebook_from_dec(np.array([0, 255] + list(range(120, 134)), np.uint8), BF16)]
    return [oracle.codebook_from_dec(SEQ_E5M2, E5M2),
            oracle.codebook_from_dec(np.array([0, 31, 1, 30, 2, 29, 3, 28, 4, 27, 5, 26, 6, 25, 24, 23], np.uint8), E5M2),
            oracle.codebook_from_dec(np.arange(16, 32, dtype=np.uint8)[::-1].copy(), E5M2)]


# --------------------------------------------------------------------------
# eq. (1) / eq. (2)
# --------------------------------------------------------------------------

def test_eq1_matches_float_semantics_of_bf16():
    """Section 3.2 eq. (1): e is the exponent field and a holds sign and mantissa,
    checked against the VALUE of every finite normal BF16 number."""
    lib = oracle.load()
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    e_bits = (words >> 7) & 0xFF
    normal = (e_bits != 0) & (e_bits != 255)
    w = words[normal]
    sign, biased, mant = bf16_fields_from_float_semantics(w)
    for x, s, b, mt in zip(w.tolist(), sign.tolist(), biased.tolist(), mant.tolist()):
        assert lib.oracle_bf16_exponent(x) == b
        a = lib.oracle_bf16_signmant(x)
        assert a >> 7 == s and a & 0x7F == mt


def test_eq1_special_exponents():
    lib = oracle.load()
    # zero / subnormals have exponent field 0, Inf / NaN have 255, any sign and mantissa
    for x, e, a in [(0x0000, 0, 0x00), (0x8000, 0, 0x80), (0x0001, 0, 0x01), (0x807F, 0, 0xFF),
                    (0x7F80, 255, 0x00), (0xFF80, 255, 0x80), (0x7FC1, 255, 0x41), (0xFFFF, 255, 0xFF)]:
        assert lib.oracle_bf16_exponent(x) == e
        assert lib.oracle_bf16_signmant(x) == a


def test_eq2_inverts_eq1_for_every_pair():
    """Section 3.2 eq. (2) with the true exponent gives back x, for all 65 536 (a, e)."""
    lib = oracle.load()
    seen = set()
    for a in range(256):
        for e in range(256):
            x = lib.oracle_bf16_combine(a, e)
            assert lib.oracle_bf16_exponent(x) == e and lib.oracle_bf16_signmant(x) == a
            seen.add(x)
    assert len(seen) == 65536


def test_e5m2_fields_match_value_and_invert():
    """E5M2 = 1 sign, 5 exponent, 2 mantissa bits (appendix SplitZip on FP8); checked against
    torch's float8_e5m2 values for normal numbers, and combine(split(x)) == x for all 256 bytes."""
    import torch

    lib = oracle.load()
    allb = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    vals = allb.view(torch.float8_e5m2).to(torch.float64).numpy()
    for x in range(256):
        e, a = lib.oracle_e5m2_exponent(x), lib.oracle_e5m2_signmant(x)
        assert lib.oracle_e5m2_combine(a, e) == x
        assert 0 <= e < 32 and 0 <= a < 8
        if 0 < e < 31:
            frac, ex = np.frexp(abs(vals[x]))
            assert e == ex - 1 + 15
            assert a & 3 == int(round((frac * 2 - 1) * 4))
            assert a >> 2 == int(np.signbit(vals[x]))
    # exponent field 0 <=> zero or subnormal (|v| < 2^-14); 31 <=> inf / nan
    for x in range(256):
        e = lib.oracle_e5m2_exponent(x)
        v = vals[x]
        assert (e == 0) == (abs(v) < 2.0 ** -14)
        assert (e == 31) == (not np.isfinite(v))


# --------------------------------------------------------------------------
# sizes: section 3.2 closed form, the 4/3 limit, the paper's printed pairs
# --------------------------------------------------------------------------

def test_payload_closed_form():
    """B_SZ = N + N/2 + 3M (section 3.2) and 7 bits + 3 bytes per escape for E5M2."""
    for n in [0, 2, 8, 1024, 4096, 1 << 20, 33554432]:
        for m in [0, 1, 5, n // 100, n]:
            if m > n:
                continue
            assert oracle.payload_bytes(n, m, BF16) == n + n // 2 + 3 * m
            if n % 8 == 0:
                assert oracle.payload_bytes(n, m, E5M2) * 8 == 7 * n + 24 * m


def test_ratio_limit_is_four_thirds():
    """rho -> 4/3 as the escape rate goes to 0 (section 3.2); 8/7 for E5M2."""
    n = 1 << 20
    assert 2 * n * 3 == 4 * oracle.payload_bytes(n, 0, BF16)
    assert n * 7 == 8 * oracle.payload_bytes(n, 0, E5M2)


def test_printed_ratio_pairs(golden_dir):
    """The payload size function reproduces the (escape rate, ratio) pairs the paper prints."""
    n = 1 << 30
    rows, kinds = 0, {}
    for line in open(os.path.join(golden_dir, "paper_ratio_pairs.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        dt, eps_pct, eps_dec, printed, rdec, raw_bits, kind = line.split()[:7]
        dtype = BF16 if dt == "bf16" else E5M2
        eps, half = float(eps_pct) / 100, 0.5 * 10 ** (-int(eps_dec)) / 100
        printed, rdec, raw_bits = float(printed), int(rdec), int(raw_bits)

        def ratio(e):
            return raw_bits * n / 8 / oracle.payload_bytes(n, int(round(e * n)), dtype)

        lo, hi = ratio(eps + half), ratio(max(eps - half, 0.0))   # ratio falls as eps grows
        step = 0.5 * 10 ** (-rdec)
        if kind == "exact":
            assert lo - step <= printed <= hi + step, line
        elif kind == "all":
            assert round(ratio(eps), rdec) == printed and lo - step <= printed <= hi + step, line
        else:
            assert kind == "upper"
            assert printed <= hi + step and printed >= lo - step - 0.01, line
        rows += 1
        kinds[kind] = kinds.get(kind, 0) + 1
    assert rows == 8 and kinds == {"exact": 2, "all": 4, "upper": 2}


def test_printed_ratio_pins_reject_a_wrong_record_size():
    """The pins above bite: a payload function with 2, 4 or 5 bytes per escape instead of 3 (or a code plane of
    N instead of N/2 bytes) fails at least one of the printed pairs."""
    rows = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_ratio_pairs.txt")):
        line = line.split("#")[0].strip()
        if line:
            dt, eps_pct, eps_dec, printed, rdec, raw_bits, kind = line.split()[:7]
            rows.append((dt, float(eps_pct) / 100, 0.5 * 10 ** (-int(eps_dec)) / 100, float(printed), int(rdec), int(raw_bits), kind))

    def passes(payload_bits):          # payload_bits(dt, eps) -> bits per element
        for dt, eps, half, printed, rdec, raw_bits, kind in rows:
            lo, hi = raw_bits / payload_bits(dt, eps + half), raw_bits / payload_bits(dt, max(eps - half, 0.0))
            step = 0.5 * 10 ** (-rdec)
            if kind == "exact" and not (lo - step <= printed <= hi + step):
                return False
            if kind == "all" and not (round(raw_bits / payload_bits(dt, eps), rdec) == printed):
                return False
            if kind == "upper" and not (printed <= hi + step and printed >= lo - step - 0.01):
                return False
        return True

    dense = {"bf16": 12.0, "e5m2": 7.0}
    assert passes(lambda dt, e: dense[dt] + 24 * e)                    # the paper's B_SZ
    for wrong in (16, 32, 40):
        assert not passes(lambda dt, e: dense[dt] + wrong * e), wrong
    assert not passes(lambda dt, e: dense[dt] + 4 + 24 * e)            # codes not packed two per byte
    assert not passes(lambda dt, e: dense[dt] - 1 + 24 * e)


def test_total_bytes_itemised():
    """whole stream = header + offset table + planes + escapes, every section 256-byte aligned"""
    for dtype in (BF16, E5M2):
        for n in [0, 1, 2, 7, 8, 9, 15, 16, 17, 1023, 1024, 1025, 2047, 2048, 2049, 4096, 100000]:
            for m in sorted({0, 1, 7, 8, 9, min(n, 1000), n}):
                if m > n:
                    continue
                c = (n + 1023) // 1024
                sm = n if dtype == BF16 else (3 * n + 7) // 8
                want = a256(64 + 4 * (c + 1)) + a256(sm) + a256((n + 1) // 2) + a256(2 * m) + m
                assert oracle.total_bytes(n, m, dtype) == want


# --------------------------------------------------------------------------
# hand-assembled streams
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name,dtype", [("hand_stream_bf16.txt", BF16), ("hand_stream_e5m2.txt", E5M2)])
def test_hand_assembled_stream(golden_dir, name, dtype):
    dec, words, blob = read_golden(os.path.join(golden_dir, name))
    x = np.array(words, np.uint16 if dtype == BF16 else np.uint8)
    cb = oracle.codebook_from_dec(dec, dtype)
    got, m = oracle.compress(x, cb)
    assert m == 2
    assert got.tobytes() == blob.tobytes()
    assert np.array_equal(oracle.decompress(blob, x.size, cb), x)


def test_chunk_relative_positions_worked_example():
    """Escape positions are relative to 1024-element chunks, 16 bits each, with the raw
    exponent beside them (section 3.2; appendix on chunk size)."""
    n = 3 * 1024 + 7
    x = np.full(n, 0x3F80, np.uint16)          # 1.0 everywhere, exponent 127
    esc = {0: 0x0000, 1023: 0x7F80, 1024: 0x0280, 1029: 0x8000, 2047: 0xFFFF, 3072 + 6: 0x0001}
    for i, w in esc.items():
        x[i] = w
    cb = oracle.codebook_from_dec(SEQ_BF16, BF16)
    blob, m = oracle.compress(x, cb)
    p = parse_stream(blob, BF16)
    assert m == 6 and p["m"] == 6 and p["c"] == 4
    assert p["chunk_off"].tolist() == [0, 2, 5, 5, 6]          # chunk 2 has none
    assert p["pos"].tolist() == [0, 1023, 0, 5, 1023, 6]
    assert p["val"].tolist() == [0, 255, 5, 0, 255, 0]
    assert np.array_equal(oracle.decompress(blob, n, cb), x)


# --------------------------------------------------------------------------
# round trip, escape tally, structure
# --------------------------------------------------------------------------

def check_stream(x, cb, blob, m):
    dtype = cb.dtype
    n = x.size
    e = exponents_np(x, dtype)
    is_esc = ~np.isin(e, cb.dec)
    # |E| by brute force (section 3.2 definition of the escape set)
    assert m == int(is_esc.sum())
    p = parse_stream(blob, dtype)
    assert p["n"] == n and p["m"] == m and p["total"] == blob.size == p["end"]
    # closed-form sizes
    sm = n if dtype == BF16 else (3 * n + 7) // 8
    assert blob.size == a256(64 + 4 * (p["c"] + 1)) + a256(sm) + a256((n + 1) // 2) + a256(2 * m) + m
    assert all(not pad.any() for pad in p["pads"])
    # escapes: ascending element order, chunk-relative
    idx = np.flatnonzero(is_esc)
    assert np.array_equal(p["pos"], (idx % 1024).astype(np.uint16))
    assert np.array_equal(p["val"], e[idx])
    counts = np.bincount(idx // 1024, minlength=p["c"]) if n else np.zeros(0, np.int64)
    assert np.array_equal(p["chunk_off"], np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32))
    # codes: even element in the low nibble, dummy 0 for escapes, code k <-> dec[k]
    codes = np.empty(2 * p["code"].size, np.uint8)
    codes[0::2] = p["code"] & 0xF
    codes[1::2] = p["code"] >> 4
    assert not codes[n:].any()
    codes = codes[:n]
    assert not codes[is_esc].any()
    assert np.array_equal(cb.dec[codes[~is_esc]], e[~is_esc])
    # sign+mantissa plane
    if dtype == BF16:
        assert np.array_equal(p["sm"], (((x >> 8) & 0x80) | (x & 0x7F)).astype(np.uint8))
    else:
        bits = np.unpackbits(p["sm"], bitorder="little")
        assert not bits[3 * n:].any()
        a = bits[:3 * n].reshape(n, 3)
        a = a[:, 0] | (a[:, 1] << 1) | (a[:, 2] << 2)
        assert np.array_equal(a, ((x >> 5) & 4) | (x & 3))


@pytest.mark.parametrize("dtype", [BF16, E5M2])
def test_all_bit_patterns_round_trip(dtype):
    """Bitwise round-trip identity on every BF16 word (and every E5M2 byte, repeated), in a
    shuffled order, under several codebooks including one that covers nothing common."""
    rng = np.random.default_rng(7)
    if dtype == BF16:
        x = rng.permutation(65536).astype(np.uint16)
    else:
        x = rng.permutation(np.tile(np.arange(256), 20)).astype(np.uint8)
    for cb in codebooks(dtype):
        blob, m = oracle.compress(x, cb)
        check_stream(x, cb, blob, m)
        assert np.array_equal(oracle.decompress(blob, x.size, cb), x)


@pytest.mark.parametrize("dtype", [BF16, E5M2])
def test_every_small_length_round_trips(dtype):
    """every N in 0..2050: pack, chunk and alignment boundaries; escapes at the chunk edges"""
    rng = np.random.default_rng(11)
    cb = codebooks(dtype)[0]
    hot = cb.dec[:6]
    for n in range(0, 2051):
        e = hot[rng.integers(0, hot.size, n)].astype(np.uint16)
        for i in (0, 1, 1022, 1023, 1024, 1025, n - 2, n - 1):
            if 0 <= i < n and rng.random() < 0.7:
                e[i] = 0 if rng.random() < 0.5 else (255 if dtype == BF16 else 31)
        if dtype == BF16:
            x = ((rng.integers(0, 2, n) << 15) | (e << 7) | rng.integers(0, 128, n)).astype(np.uint16)
        else:
            x = ((rng.integers(0, 2, n) << 7) | (e << 2) | rng.integers(0, 4, n)).astype(np.uint8)
        blob, m = oracle.compress(x, cb)
        if n % 97 == 0 or n < 40 or 1020 <= n <= 1030 or n >= 2040:
            check_stream(x, cb, blob, m)
        assert blob.size == oracle.total_bytes(n, m, dtype)
        assert np.array_equal(oracle.decompress(blob, n, cb), x)


def test_no_escapes_gives_exact_ratio():
    """Every exponent in the codebook => M = 0 and payload ratio exactly 16/12."""
    rng = np.random.default_rng(3)
    n = 64 * 1024
    cb = codebooks(BF16)[0]
    x = ((rng.integers(0, 2, n) << 15) | (cb.dec[rng.integers(0, 16, n)].astype(np.uint16) << 7)
         | rng.integers(0, 128, n)).astype(np.uint16)
    blob, m = oracle.compress(x, cb)
    assert m == 0 and oracle.count_escapes(x, cb) == 0
    p = parse_stream(blob, BF16)
    assert (p["sm"].size + p["code"].size + 3 * m) * 4 == 2 * n * 3
    assert not p["chunk_off"].any()
    assert np.array_equal(oracle.decompress(blob, n, cb), x)


def test_all_escape_tensor():
    """codebook that covers nothing: M = N, every chunk full, still lossless"""
    rng = np.random.default_rng(5)
    n = 5 * 1024 + 123
    x = kv_synth.to_numpy_words(kv_synth.kv_bf16(8, 3))[:n].copy()
    cb = codebooks(BF16)[1]
    blob, m = oracle.compress(x, cb)
    assert m == n
    check_stream(x, cb, blob, m)
    assert np.array_equal(oracle.decompress(blob, n, cb), x)


@pytest.mark.parametrize("dtype", [BF16, E5M2])
def test_synthetic_kv_regime(dtype):
    """config-0 law: round trip, sizes, brute-force escape tally; statistics in the regime of the
    paper's Table 1 (top-16 coverage >= 99 %, exponent entropy about 3 bits)."""
    gen = kv_synth.kv_bf16 if dtype == BF16 else kv_synth.kv_e5m2
    x = kv_synth.to_numpy_words(gen(512, 0))
    cb = oracle.calibrate(kv_synth.to_numpy_words(gen(512, 1)), dtype)
    blob, m = oracle.compress(x, cb)
    check_stream(x, cb, blob, m)
    assert np.array_equal(oracle.decompress(blob, x.size, cb), x)
    assert m / x.size < 0.01
    h = cb.hist.astype(np.float64)
    p = h[h > 0] / h.sum()
    assert 2.5 < -(p * np.log2(p)).sum() < 4.0


def test_outlier_tensor_escapes():
    x = kv_synth.to_numpy_words(kv_synth.kv_bf16_outliers(256, 0))
    cb = oracle.calibrate(kv_synth.to_numpy_words(kv_synth.kv_bf16(256, 1)), BF16)
    blob, m = oracle.compress(x, cb)
    check_stream(x, cb, blob, m)
    assert 0.003 < m / x.size < 0.05
    assert np.array_equal(oracle.decompress(blob, x.size, cb), x)


# --------------------------------------------------------------------------
# calibration (section 3.3)
# --------------------------------------------------------------------------

def sample_with_counts(counts, dtype):
    """words whose exponent histogram is exactly `counts` (dict exponent -> count)"""
    es = np.concatenate([np.full(c, e, np.uint16) for e, c in counts.items()] or [np.zeros(0, np.uint16)])
    rng = np.random.default_rng(1)
    rng.shuffle(es)
    if dtype == BF16:
        return ((es << 7) | rng.integers(0, 128, es.size)).astype(np.uint16)
    return ((es << 2) | rng.integers(0, 4, es.size)).astype(np.uint8)


def test_calibrate_top16_hand_histogram():
    """top-16 by frequency; code k is the k-th most frequent exponent"""
    counts = {100 + i: 1000 - 10 * i for i in range(20)}      # strictly decreasing
    counts[7] = 5000
    cb = oracle.calibrate(sample_with_counts(counts, BF16), BF16)
    assert cb.dec.tolist() == [7] + [100 + i for i in range(15)]
    assert int(cb.hist[7]) == 5000 and int(cb.hist.sum()) == sum(counts.values())
    for k, e in enumerate(cb.dec.tolist()):
        assert cb.enc[e] == k and cb.member[e] == 1
    assert int(cb.member.sum()) == 16
    assert not cb.enc[cb.member == 0].any()


def test_calibrate_ties_and_few_values():
    # ties go to the smaller exponent; never-seen values fill the table in ascending order
    counts = {130: 50, 120: 50, 125: 70, 3: 50}
    cb = oracle.calibrate(sample_with_counts(counts, BF16), BF16)
    assert cb.dec.tolist() == [125, 3, 120, 130, 0, 1, 2, 4, 5, 6, 7, 8, 9, 10, 11, 12]
    cb0 = oracle.calibrate(np.zeros(0, np.uint16), BF16)
    assert cb0.dec.tolist() == list(range(16))
    cb8 = oracle.calibrate(sample_with_counts({31: 9, 30: 9, 2: 10}, E5M2), E5M2)
    assert cb8.dec.tolist() == [2, 30, 31, 0, 1, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13]


def test_calibrate_matches_numpy_sort():
    for dtype, gen in ((BF16, kv_synth.kv_bf16), (E5M2, kv_synth.kv_e5m2)):
        x = kv_synth.to_numpy_words(gen(128, 9))
        cb = oracle.calibrate(x, dtype)
        nv = 256 if dtype == BF16 else 32
        h = np.bincount(exponents_np(x, dtype), minlength=256)
        assert np.array_equal(h, cb.hist.astype(np.int64))
        order = sorted(range(nv), key=lambda v: (-h[v], v))[:16]
        assert cb.dec.tolist() == order


# --------------------------------------------------------------------------
# decoder input validation
# --------------------------------------------------------------------------

def test_decompress_rejects_malformed():
    x = kv_synth.to_numpy_words(kv_synth.kv_bf16(4, 0))
    cb = oracle.calibrate(x, BF16)
    x = x.copy()
    x[5] = 0          # make sure there is an escape
    x[3000] = 0x7F80
    blob, m = oracle.compress(x, cb)
    assert m >= 2
    n = x.size

    def bad(mut, n_=n, cb_=cb):
        b = blob.copy()
        b = mut(b) if mut else b
        with pytest.raises(ValueError):
            oracle.decompress(b, n_, cb_)

    def setb(i, v):
        def f(b):
            b[i] = v
            return b
        return f

    bad(setb(0, ord("X")))                    # magic
    bad(setb(4, 2))                           # version
    bad(setb(6, 1))                           # dtype
    bad(setb(16, int(blob[16]) ^ 1))          # N
    bad(setb(24, int(blob[24]) + 1))          # M inconsistent with total
    bad(lambda b: b[:-1])                     # truncated
    bad(None, n_=n - 1)                       # caller's N differs
    bad(None, cb_=oracle.codebook_from_dec(SEQ_BF16[::-1].copy(), BF16))   # other codebook
    p = parse_stream(blob, BF16)
    o_pos = blob.size - m - a256(2 * m)
    bad(setb(o_pos + 1, 0xFF))                # position outside its chunk
    bad(setb(64, 1))                          # chunk_off[0] != 0
