"""Pins of the format-variant oracle (oracle/splitzip_variants_oracle.c) to things other than itself:
hand-assembled streams, the paper's printed ratios for the ablated formats, closed forms, a decoder
written a second time in this file straight from the layout, the main-format oracle for the variant
that coincides with it, and round trips over every bit pattern.  CPU only."""
import os

import numpy as np
import pytest

import oracle
from oracle import variants as ov

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

SB = {ov.BF16: 8, ov.E5M2: 3, ov.E4M3: 4}            # bits of sign+mantissa per element
EXPS = {ov.BF16: 256, ov.E5M2: 32, ov.E4M3: 16}
WORD = {ov.BF16: np.uint16, ov.E5M2: np.uint8, ov.E4M3: np.uint8}


def a256(x):
    return (x + 255) // 256 * 256


def all_variants():
    """the formats of the ablations, per dtype"""
    out = []
    for dt in (ov.BF16, ov.E5M2):
        out += [ov.variant(dt, 4, 16, ov.ESC_POS, 1024),       # the main format
                ov.variant(dt, 4, 15, ov.ESC_SENTINEL, 1024),   # top-15 + sentinel
                ov.variant(dt, 3, 8, ov.ESC_POS, 1024),         # top-8, 3-bit codes
                ov.variant(dt, 4, 16, ov.ESC_POS, 256),         # chunk 256, 8-bit positions
                ov.variant(dt, 4, 16, ov.ESC_ABS32, 0)]         # absolute 32-bit positions
    out += [ov.variant(ov.E4M3, 3, 8, ov.ESC_POS, 1024),
            ov.variant(ov.E4M3, 3, 7, ov.ESC_SENTINEL, 256)]
    # escape values in the exponent's own width (the FP8 table's top-8 columns)
    out += [ov.variant(ov.E5M2, 3, 8, ov.ESC_POS, 1024, 5),
            ov.variant(ov.E4M3, 3, 8, ov.ESC_POS, 1024, 4),
            ov.variant(ov.E5M2, 4, 15, ov.ESC_SENTINEL, 256, 5),
            ov.variant(ov.E4M3, 3, 8, ov.ESC_ABS32, 0, 4)]
    return out


def vb_of(v):
    return v.value_bits or 8


def vid(v):
    return f"dt{v.dtype}-b{v.code_bits}-k{v.k}-m{v.escape_mode}-c{v.chunk}" + (f"-v{v.value_bits}" if v.value_bits else "")


def exponent_np(x, dt):
    x = x.astype(np.uint32)
    return (x >> 7) & 0xFF if dt == ov.BF16 else (x >> 2) & 0x1F if dt == ov.E5M2 else (x >> 3) & 0xF


def some_dec(dt, k, rng):
    """k distinct exponents around the middle of the range, shuffled"""
    mid = EXPS[dt] // 2
    vals = np.array([(mid - 4 + i) % EXPS[dt] for i in range(16)], np.uint8)[:k]
    rng.shuffle(vals)
    dec = np.zeros(16, np.uint8)
    dec[:k] = vals
    return dec


def random_words(dt, n, rng, spread=6):
    """words whose exponents cluster around the middle of the range, a few far away"""
    mid = EXPS[dt] // 2
    e = np.clip(np.rint(rng.normal(mid, spread / 3, n)), 0, EXPS[dt] - 1).astype(np.uint32)
    far = rng.random(n) < 0.01
    e[far] = rng.integers(0, EXPS[dt], far.sum())
    if dt == ov.BF16:
        return ((rng.integers(0, 2, n) << 15) | (e << 7) | rng.integers(0, 128, n)).astype(np.uint16)
    if dt == ov.E5M2:
        return ((rng.integers(0, 2, n) << 7) | (e << 2) | rng.integers(0, 4, n)).astype(np.uint8)
    return ((rng.integers(0, 2, n) << 7) | (e << 3) | rng.integers(0, 8, n)).astype(np.uint8)


# ---- a second decoder, written from the layout description only --------------------------------

def bits_at(plane, i, width):
    """element i of an LSB-first bit stream of `width`-bit fields"""
    value = 0
    for j in range(width):
        b = width * i + j
        value |= ((int(plane[b >> 3]) >> (b & 7)) & 1) << j
    return value


def field(blob, off, nbytes):
    return int.from_bytes(bytes(blob[off:off + nbytes]), "little")


def py_decode(blob, n, v, dec):
    """walks the stream as the layout says; no call into the oracle"""
    dt, cb, sb = v.dtype, v.code_bits, SB[v.dtype]
    assert bytes(blob[:4]) == b"SZP1" and field(blob, 4, 2) == 2
    m = field(blob, 24, 8)
    absolute = v.escape_mode == ov.ESC_ABS32
    c = 0 if absolute else -(-n // v.chunk)
    tab = 64
    off_sm = a256(64 + (0 if absolute else 4 * (c + 1)))
    off_code = off_sm + a256(-(-n * sb // 8))
    off_pos = off_code + a256(-(-n * cb // 8))
    pb = 0 if v.escape_mode == ov.ESC_SENTINEL else 4 if absolute else (2 if v.chunk > 256 else 1)
    off_val = off_pos + a256(m * pb)
    vb = vb_of(v)
    assert off_val + -(-m * vb // 8) == field(blob, 32, 8) == len(blob)
    sm, code, vals = blob[off_sm:], blob[off_code:], blob[off_val:]
    exps, next_val = [], 0
    for i in range(n):
        cde = bits_at(code, i, cb)
        if v.escape_mode == ov.ESC_SENTINEL and cde == (1 << cb) - 1:
            exps.append(bits_at(vals, next_val, vb))
            next_val += 1
        else:
            exps.append(int(dec[cde]))
    if v.escape_mode == ov.ESC_POS:
        for ch in range(c):
            lo, hi = field(blob, tab + 4 * ch, 4), field(blob, tab + 4 * ch + 4, 4)
            for j in range(lo, hi):
                exps[ch * v.chunk + field(blob, off_pos + pb * j, pb)] = bits_at(vals, j, vb)
    elif absolute:
        for j in range(m):
            exps[field(blob, off_pos + 4 * j, 4)] = bits_at(vals, j, vb)
    out = []
    for i in range(n):
        a, e = bits_at(sm, i, sb), exps[i]
        if dt == ov.BF16:
            out.append(((a & 0x80) << 8) | (e << 7) | (a & 0x7F))
        elif dt == ov.E5M2:
            out.append(((a & 4) << 5) | (e << 2) | (a & 3))
        else:
            out.append(((a & 8) << 4) | (e << 3) | (a & 7))
    return np.array(out, WORD[dt])


# ---- hand-assembled streams ----------------------------------------------------------------

def read_golden(path):
    var = dec = words = None
    escapes = 1
    blob, in_blob = [], False
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("variant:"):
            var = [int(t) for t in line[8:].split()]
        elif line.startswith("escapes:"):
            escapes = int(line[8:])
        elif line.startswith("dec:"):
            dec = [int(t) for t in line[4:].split()]
        elif line.startswith("words:"):
            words = [int(t, 16) for t in line[6:].split()]
        elif line.startswith("blob:"):
            in_blob = True
        elif in_blob and line.startswith("zeros"):
            blob += [0] * int(line.split()[1])
        elif in_blob:
            blob += [int(t, 16) for t in line.split()]
    d = np.zeros(16, np.uint8)
    d[:len(dec)] = dec
    return ov.variant(*var), d, words, np.array(blob, np.uint8), escapes


@pytest.mark.parametrize("name", ["hand_stream_variant_bf16_top3_chunk256.txt",
                                  "hand_stream_variant_e4m3_sentinel.txt",
                                  "hand_stream_variant_bf16_abs32.txt",
                                  "hand_stream_variant_e5m2_top2_values5.txt"])
def test_hand_assembled_variant_streams(name):
    v, dec, words, blob, escapes = read_golden(os.path.join(GOLDEN, name))
    x = np.array(words, WORD[v.dtype])
    got, m = ov.compress(x, v, dec)
    assert m == escapes
    assert got.size == blob.size and np.array_equal(got, blob), np.flatnonzero(got != blob)[:8]
    assert np.array_equal(ov.decompress(blob, x.size, v, dec), x)
    assert np.array_equal(py_decode(blob, x.size, v, dec), x)


# ---- sizes ------------------------------------------------------------------------------------

def test_printed_ratios_of_the_ablated_formats():
    """Section "Ablation on Top-k Exponent Coding": top-8 / 3 bits at a 7.89 % escape rate gives 1.241;
    section "Ablation on Escape-Position Metadata": top-15 + sentinel at 0.27 % gives 1.331 (payload bytes,
    as all of the paper's ratios)."""
    n = 1 << 26
    for v, eps, want in ((ov.variant(ov.BF16, 3, 8, ov.ESC_POS, 1024), 0.0789, 1.241),
                         (ov.variant(ov.BF16, 4, 15, ov.ESC_SENTINEL, 1024), 0.0027, 1.331)):
        ratio = 2 * n / ov.payload_bytes(n, round(eps * n), v)
        assert abs(ratio - want) < 0.0006, (vid(v), ratio)


def test_printed_fp8_ratios_fix_the_width_of_an_escape_value():
    """Table "FP8 codec throughput and compression ratio": E5M2 top-16 at 0.16 % escapes gives 1.136 -- only with
    whole-byte escape values; E5M2 top-8 at 7.72 % gives 1.049 and E4M3 top-8 at 7.83 % gives 0.933 -- only with the
    exponent in its own width (5 and 4 bits).  A printed ratio counts as reproduced if the payload ratio at some
    escape rate inside the rounding interval of the printed one rounds to it, or lies above it by less than 0.001
    (the paper's ratios include some metadata it does not itemise: its 1.324 is 1.329 by its own formula)."""
    n = 1 << 26

    def reproduced(v, eps, want):
        lo = n / ov.payload_bytes(n, round((eps + 0.00005) * n), v)      # ratio falls as the escape rate grows
        hi = n / ov.payload_bytes(n, round((eps - 0.00005) * n), v)
        return lo - 0.0005 - 0.001 <= want <= hi + 0.0005

    rows = ((ov.E5M2, 4, 16, 0.0016, 1.136, 8), (ov.E5M2, 3, 8, 0.0772, 1.049, 5), (ov.E4M3, 3, 8, 0.0783, 0.933, 4))
    for dt, cb, k, eps, want, vb in rows:
        assert reproduced(ov.variant(dt, cb, k, ov.ESC_POS, 1024, vb), eps, want), (dt, k, vb)
    # and the other width of each fails: the table needs both formats
    assert not reproduced(ov.variant(ov.E5M2, 3, 8, ov.ESC_POS, 1024, 8), 0.0772, 1.049)
    assert not reproduced(ov.variant(ov.E4M3, 3, 8, ov.ESC_POS, 1024, 8), 0.0783, 0.933)
    # (E5M2 top-16 with 5-bit values: 1.1374, which the slack for metadata would still let pass; what excludes it is
    # the main format's own pin, which has no slack: tests/golden/paper_ratio_pairs.txt, kind "exact")
    assert round(n / ov.payload_bytes(n, round(0.0016 * n), ov.variant(ov.E5M2, 4, 16, ov.ESC_POS, 1024, 5)), 3) == 1.137


def test_payload_and_total_closed_forms():
    """payload = ceil(N sb / 8) + ceil(N cb / 8) + M (position bytes + 1): the size formula of section 3.2
    with the widths of each ablation; total adds header, offset table and 256-byte alignment."""
    for v in all_variants():
        sb, cb = SB[v.dtype], v.code_bits
        pb = {ov.ESC_POS: 2 if v.chunk > 256 else 1, ov.ESC_SENTINEL: 0, ov.ESC_ABS32: 4}[v.escape_mode]
        for n, m in ((0, 0), (1, 0), (1, 1), (255, 3), (256, 256), (1023, 7), (1024, 0), (1025, 1025), (4099, 12),
                     (1 << 20, 1234)):
            assert ov.payload_bytes(n, m, v) == -(-n * sb // 8) + -(-n * cb // 8) + m * pb + -(-m * vb_of(v) // 8)
            tab = 0 if v.escape_mode == ov.ESC_ABS32 else 4 * (-(-n // v.chunk) + 1)
            assert ov.total_bytes(n, m, v) == (a256(64 + tab) + a256(-(-n * sb // 8)) + a256(-(-n * cb // 8))
                                               + a256(m * pb) + -(-m * vb_of(v) // 8))


def test_zero_escapes_give_the_dense_ratio():
    """no escapes: 16 / (8 + 4) and 16 / (8 + 3) for BF16, 8 / 7, 8 / 6 for E5M2, 8 / 7 for E4M3 with 3-bit codes"""
    n = 1 << 20
    for dt, cb, want in ((ov.BF16, 4, 16 / 12), (ov.BF16, 3, 16 / 11), (ov.E5M2, 4, 8 / 7), (ov.E5M2, 3, 8 / 6),
                         (ov.E4M3, 3, 8 / 7)):
        v = ov.variant(dt, cb, 8, ov.ESC_POS, 1024)
        bits = 16 if dt == ov.BF16 else 8
        assert abs(n * bits / 8 / ov.payload_bytes(n, 0, v) - want) < 1e-12


# ---- against the main-format oracle ----------------------------------------------------------

@pytest.mark.parametrize("dt", [ov.BF16, ov.E5M2])
def test_main_format_variant_equals_the_main_oracle_after_the_header(dt):
    rng = np.random.default_rng(5)
    for n in (0, 1, 2, 1023, 1024, 1025, 5000):
        x = random_words(dt, n, rng)
        cb = oracle.calibrate(random_words(dt, 4096, rng), dt)
        ref, m_ref = oracle.compress(x, cb)
        v = ov.variant(dt, 4, 16, ov.ESC_POS, 1024)
        got, m = ov.compress(x, v, cb.dec)
        assert m == m_ref and got.size == ref.size
        assert np.array_equal(got[64:], ref[64:])
        differ = np.flatnonzero(got[:64] != ref[:64]).tolist()
        assert differ == [4, 13]          # version 2 instead of 1, and the codebook size byte
        assert got[4] == 2 and got[13] == 16


def test_calibration_is_the_main_calibration_cut_at_k():
    rng = np.random.default_rng(6)
    for dt in (ov.BF16, ov.E5M2):
        x = random_words(dt, 50000, rng)
        full = oracle.calibrate(x, dt)
        for k in (1, 7, 8, 15, 16):
            dec, hist = ov.calibrate(x, dt, k)
            assert np.array_equal(dec[:k], full.dec[:k]) and not dec[k:].any()
            assert np.array_equal(hist, full.hist)
    # E4M3: ranks by count, ties towards the smaller exponent, unseen values ascending
    x = np.array([0x38] * 5 + [0x40] * 5 + [0x30] * 2, np.uint8)      # exponents 7, 8, 6
    dec, hist = ov.calibrate(x, ov.E4M3, 8)
    assert dec[:8].tolist() == [7, 8, 6, 0, 1, 2, 3, 4] and hist[7] == 5 and hist[8] == 5 and hist[6] == 2


# ---- round trips and structure ------------------------------------------------------------------

@pytest.mark.parametrize("v", all_variants(), ids=vid)
def test_every_bit_pattern_round_trips(v):
    dt = v.dtype
    words = np.arange(65536 if dt == ov.BF16 else 256, dtype=np.uint32).astype(WORD[dt])
    rng = np.random.default_rng(7)
    x = np.concatenate([words, rng.permutation(words)[: 1500 if dt == ov.BF16 else 256]])
    top = np.zeros(16, np.uint8)
    top[:v.k] = np.arange(EXPS[dt] - v.k, EXPS[dt])          # the extreme exponents
    for dec in (some_dec(dt, v.k, rng), top):
        blob, m = ov.compress(x, v, dec)
        e = exponent_np(x, dt)
        assert m == int((~np.isin(e, dec[:v.k])).sum())        # |E| of section 3.2, counted here
        assert blob.size == ov.total_bytes(x.size, m, v)
        assert np.array_equal(ov.decompress(blob, x.size, v, dec), x)


@pytest.mark.parametrize("v", all_variants(), ids=vid)
def test_second_decoder_agrees_on_small_inputs(v):
    rng = np.random.default_rng(8)
    for n in (0, 1, 7, 8, 9, 255, 256, 257, 1023, 1024, 1025, 2500):
        x = random_words(v.dtype, n, rng)
        dec = some_dec(v.dtype, v.k, rng)
        blob, m = ov.compress(x, v, dec)
        assert np.array_equal(py_decode(blob, n, v, dec), x), (vid(v), n)
        assert np.array_equal(ov.decompress(blob, n, v, dec), x)


def test_sentinel_codes_stand_exactly_where_the_escapes_are():
    rng = np.random.default_rng(9)
    v = ov.variant(ov.BF16, 4, 15, ov.ESC_SENTINEL, 1024)
    x = random_words(ov.BF16, 3000, rng)
    dec = some_dec(ov.BF16, 15, rng)
    blob, m = ov.compress(x, v, dec)
    c = 3
    off_code = a256(64 + 4 * (c + 1)) + a256(3000)
    codes = np.array([bits_at(blob[off_code:], i, 4) for i in range(3000)])
    esc = ~np.isin(exponent_np(x, ov.BF16), dec[:15])
    assert np.array_equal(codes == 15, esc) and m == esc.sum()
    # values in element order, and the table counts them per chunk
    off_val = off_code + a256(1500)
    assert np.array_equal(blob[off_val:off_val + m], exponent_np(x, ov.BF16)[esc].astype(np.uint8))
    tab = np.frombuffer(bytes(blob[64:64 + 16]), np.uint32)
    assert tab.tolist() == [0] + np.cumsum([esc[i * 1024:(i + 1) * 1024].sum() for i in range(3)]).tolist()


def test_positions_are_chunk_relative_or_absolute_as_the_variant_says():
    rng = np.random.default_rng(10)
    x = random_words(ov.BF16, 1000, rng)
    dec = some_dec(ov.BF16, 16, rng)
    esc = np.flatnonzero(~np.isin(exponent_np(x, ov.BF16), dec))
    for v, width, rel in ((ov.variant(ov.BF16, 4, 16, ov.ESC_POS, 256), 1, 256),
                          (ov.variant(ov.BF16, 4, 16, ov.ESC_POS, 1024), 2, 1024),
                          (ov.variant(ov.BF16, 4, 16, ov.ESC_ABS32, 0), 4, 1 << 32)):
        blob, m = ov.compress(x, v, dec)
        tab = 0 if v.escape_mode == ov.ESC_ABS32 else 4 * (-(-1000 // v.chunk) + 1)
        off_pos = a256(64 + tab) + a256(1000) + a256(500)
        pos = [field(blob, off_pos + width * j, width) for j in range(m)]
        assert pos == (esc % rel).tolist()


def test_bad_streams_are_refused():
    rng = np.random.default_rng(11)
    for v in all_variants():
        x = random_words(v.dtype, 2100, rng)
        dec = some_dec(v.dtype, v.k, rng)
        blob, m = ov.compress(x, v, dec)
        assert m > 0
        for off, val in ((0, 0x54), (4, 1), (7, v.code_bits ^ 7), (12, (v.escape_mode + 1) % 3), (13, v.k - 1),
                         (24, (m + 1) & 0xFF)):
            bad = blob.copy()
            bad[off] = val
            with pytest.raises(ValueError):
                ov.decompress(bad, x.size, v, dec)
        with pytest.raises(ValueError):
            ov.decompress(blob[:-1], x.size, v, dec)
        other = dec.copy()
        other[0], other[1] = dec[1], dec[0]
        with pytest.raises(ValueError):
            ov.decompress(blob, x.size, v, other)


def test_variant_validation():
    assert ov.valid(ov.variant(ov.BF16, 4, 16, ov.ESC_POS, 1024))
    assert not ov.valid(ov.variant(ov.BF16, 4, 16, ov.ESC_SENTINEL, 1024))    # no code left for the sentinel
    assert not ov.valid(ov.variant(ov.BF16, 3, 9, ov.ESC_POS, 1024))
    assert not ov.valid(ov.variant(ov.BF16, 5, 16, ov.ESC_POS, 1024))
    assert not ov.valid(ov.variant(ov.BF16, 4, 16, ov.ESC_POS, 1000))
    assert not ov.valid(ov.variant(3, 4, 16, ov.ESC_POS, 1024))
    assert ov.valid(ov.variant(ov.E4M3, 4, 16, ov.ESC_POS, 1024))             # valid, if pointless
    assert ov.valid(ov.variant(ov.BF16, 4, 16, ov.ESC_ABS32, 0))
