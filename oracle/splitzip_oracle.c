/*
 * SplitZip reference codec -- plain, slow, single-threaded C.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the oracle the GPU library is
 * checked against.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may build or call it; the product library never does, and
 * the two share no header, table generator or helper.  The format constants
 * below are typed in here on purpose instead of being included from the
 * product's header.
 *
 * What is computed (paper section 3.2 "Method", section 3.3 "Calibration",
 * section 3.4 "Top-16 Instead of Top-15", appendix "SplitZip on FP8",
 * appendix "Ablation on Chunk Size"):
 *
 *   - every 16-bit BF16 word is split by eq. (1) into the 8-bit exponent e and
 *     the sign+mantissa byte a; eq. (2) is the inverse given an exponent;
 *   - a is stored verbatim, one byte per element;
 *   - e goes through a calibrated top-16 codebook to a 4-bit code, two codes
 *     per byte; an exponent outside the codebook gets a dummy code and is
 *     recorded as an escape: 16-bit position relative to its 1024-element
 *     chunk plus the raw 8-bit exponent, kept in chunked position and value
 *     arrays in element order;
 *   - decoding unpacks, maps codes through the 16-entry table, recombines,
 *     then overwrites the exponent field at every recorded escape position;
 *   - the payload is N + N/2 + 3M bytes (section 3.2, the B_SZ formula).
 *   - FP8 E5M2 (appendix "SplitZip on FP8"): same scheme with the 5-bit
 *     exponent coded by a 4-bit top-16 code; the sign and the two mantissa bits
 *     form a 3-bit remainder, so a covered element costs 7 bits.  The printed
 *     ratio 1.136 at a 0.16 % escape rate fixes 7 bits per element and 3 bytes
 *     per escape.
 *
 * Byte-level conventions the paper leaves open (nibble order, dummy code
 * value, tie-breaking, metadata layout, 3-bit plane packing) are the readings
 * listed at each function.  The paper prints no worked example of a stream,
 * so those byte-level conventions are "parity unpinned" by the paper; they
 * are pinned by a hand-assembled example in tests/golden instead.
 *
 * Stream layout (little endian; the offset table follows the header directly,
 * every other section starts 256-byte aligned; pad bytes are zero; A(x) rounds
 * x up to a multiple of 256; C = ceil(N/1024)).  The paper fixes the payload
 * bytes only (section 3.2); header, table and padding are this build's
 * metadata:
 *
 *   header     64 B          see write_header()
 *   chunk_off  4*(C+1) B     u32 exclusive prefix sums of per-chunk escape
 *                            counts, chunk_off[C] = M
 *   sm plane   BF16: N B     byte i = a_i
 *              E5M2: ceil(3N/8) B, LSB-first bit stream, stream bit 3i+k is
 *              bit k of a_i (stream bit b lives in bit b&7 of byte b>>3)
 *   code plane ceil(N/2) B   byte j = code_{2j} | code_{2j+1} << 4
 *   esc_pos    2M B          u16 chunk-relative positions, element order
 *   esc_val    M B           u8 raw exponents, same order
 *
 *   total = A(64 + 4(C+1)) + A(sm) + A(ceil(N/2)) + A(2M) + M
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_BF16 0
#define ORACLE_E5M2 1

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_CAPACITY (-2)
#define ORACLE_ERR_FORMAT (-3)
#define ORACLE_ERR_NOMEM (-4)

#define CHUNK 1024u
#define HEADER_BYTES 64u

/* section alignment: 256 bytes (two 128-byte cache lines, one HBM channel granule) */
static uint64_t a256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

static int dtype_ok(int dtype) { return dtype == ORACLE_BF16 || dtype == ORACLE_E5M2; }

/* number of distinct exponent values of the format */
static unsigned exp_values(int dtype) { return dtype == ORACLE_BF16 ? 256u : 32u; }

/* ---- field split and recombination ------------------------------------ */

/* eq. (1): e = (x >> 7) & 0xff */
uint8_t oracle_bf16_exponent(uint16_t x) { return (uint8_t)((x >> 7) & 0xff); }

/* eq. (1): a = ((x >> 8) & 0x80) | (x & 0x7f) */
uint8_t oracle_bf16_signmant(uint16_t x) { return (uint8_t)(((x >> 8) & 0x80) | (x & 0x7f)); }

/* eq. (2): x = ((a & 0x80) << 8) | (e << 7) | (a & 0x7f) */
uint16_t oracle_bf16_combine(uint8_t a, uint8_t e) {
  return (uint16_t)((((unsigned)a & 0x80u) << 8) | ((unsigned)e << 7) | ((unsigned)a & 0x7fu));
}

/* E5M2 byte = s eeeee mm.  The paper gives no formula for FP8; these follow
 * eq. (1)/(2) with the field widths of the format: e is the 5-bit field, a is
 * the 3-bit remainder (sign, m1, m0). */
uint8_t oracle_e5m2_exponent(uint8_t x) { return (uint8_t)((x >> 2) & 0x1f); }
uint8_t oracle_e5m2_signmant(uint8_t x) { return (uint8_t)(((x >> 5) & 0x4) | (x & 0x3)); }
uint8_t oracle_e5m2_combine(uint8_t a, uint8_t e) {
  return (uint8_t)((((unsigned)a & 0x4u) << 5) | ((unsigned)e << 2) | ((unsigned)a & 0x3u));
}

/* ---- sizes -------------------------------------------------------------- */

/* bytes of the sign+mantissa plane */
uint64_t oracle_sm_bytes(uint64_t n, int dtype) {
  return dtype == ORACLE_BF16 ? n : (3u * n + 7u) / 8u;
}

/* Section 3.2, B_SZ = N + N/2 + 3M for BF16 (N/2 rounded up for odd N); for
 * E5M2 the first term is the 3-bit plane.  Metadata excluded. */
uint64_t oracle_payload_bytes(uint64_t n, uint64_t m, int dtype) {
  return oracle_sm_bytes(n, dtype) + (n + 1u) / 2u + 3u * m;
}

/* whole stream: payload + header + chunk offset table + alignment pads */
uint64_t oracle_total_bytes(uint64_t n, uint64_t m, int dtype) {
  uint64_t c = (n + CHUNK - 1u) / CHUNK;
  return a256(HEADER_BYTES + 4u * (c + 1u)) + a256(oracle_sm_bytes(n, dtype)) + a256((n + 1u) / 2u) +
         a256(2u * m) + m;
}

/* ---- calibration (section 3.3) ----------------------------------------- */

/* Count the exponent values of the sample, take the 16 most frequent, build
 * the encoding, decoding and membership tables.
 * Readings: ties are broken towards the smaller exponent value; values that
 * never occur fill the remaining slots in ascending order, so there are always
 * exactly 16 members; code k is the k-th most frequent exponent; a non-member
 * encodes to the dummy code 0. */
int oracle_calibrate(const void* sample, uint64_t n, int dtype, uint8_t dec[16], uint8_t enc[256],
                     uint8_t member[256], uint64_t hist[256]) {
  if (!dtype_ok(dtype) || (n && !sample) || !dec || !enc || !member) return ORACLE_ERR_ARG;
  uint64_t h[256];
  memset(h, 0, sizeof h);
  for (uint64_t i = 0; i < n; ++i) {
    unsigned e = dtype == ORACLE_BF16 ? oracle_bf16_exponent(((const uint16_t*)sample)[i])
                                      : oracle_e5m2_exponent(((const uint8_t*)sample)[i]);
    h[e]++;
  }
  unsigned nv = exp_values(dtype);
  uint8_t taken[256];
  memset(taken, 0, sizeof taken);
  memset(enc, 0, 256);
  memset(member, 0, 256);
  for (unsigned k = 0; k < 16; ++k) {
    /* selection: highest count among the values not taken yet; scanning in
     * ascending value order with a strict '>' keeps the smallest on ties */
    int best = -1;
    for (unsigned v = 0; v < nv; ++v) {
      if (taken[v]) continue;
      if (best < 0 || h[v] > h[best]) best = (int)v;
    }
    taken[best] = 1;
    dec[k] = (uint8_t)best;
    enc[best] = (uint8_t)k;
    member[best] = 1;
  }
  if (hist) memcpy(hist, h, sizeof h);
  return ORACLE_OK;
}

/* Tables from a given list of 16 distinct exponents (code k = dec[k]). */
int oracle_tables_from_dec(const uint8_t dec[16], int dtype, uint8_t enc[256], uint8_t member[256]) {
  if (!dtype_ok(dtype) || !dec || !enc || !member) return ORACLE_ERR_ARG;
  memset(enc, 0, 256);
  memset(member, 0, 256);
  for (unsigned k = 0; k < 16; ++k) {
    if (dec[k] >= exp_values(dtype) || member[dec[k]]) return ORACLE_ERR_ARG;
    member[dec[k]] = 1;
    enc[dec[k]] = (uint8_t)k;
  }
  return ORACLE_OK;
}

/* |E| of section 3.2: the number of elements whose exponent is outside C. */
uint64_t oracle_count_escapes(const void* in, uint64_t n, int dtype, const uint8_t member[256]) {
  uint64_t m = 0;
  for (uint64_t i = 0; i < n; ++i) {
    unsigned e = dtype == ORACLE_BF16 ? oracle_bf16_exponent(((const uint16_t*)in)[i])
                                      : oracle_e5m2_exponent(((const uint8_t*)in)[i]);
    if (!member[e]) ++m;
  }
  return m;
}

/* ---- little-endian stores / loads ------------------------------------- */

static void put16(uint8_t* p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put32(uint8_t* p, uint32_t v) { put16(p, (uint16_t)v); put16(p + 2, (uint16_t)(v >> 16)); }
static void put64(uint8_t* p, uint64_t v) { put32(p, (uint32_t)v); put32(p + 4, (uint32_t)(v >> 32)); }
static uint16_t get16(const uint8_t* p) { return (uint16_t)(p[0] | (p[1] << 8)); }
static uint32_t get32(const uint8_t* p) { return (uint32_t)get16(p) | ((uint32_t)get16(p + 2) << 16); }
static uint64_t get64(const uint8_t* p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }

/* header, 64 bytes:
 *   0  u32 magic 'S','Z','P','1'    4  u16 version = 1   6 u8 dtype   7 u8 code bits = 4
 *   8  u32 chunk elements = 1024   12  u32 reserved = 0
 *  16  u64 N   24  u64 M   32  u64 total bytes   40  u8 dec[16]   56  u8 reserved[8] = 0 */
static void write_header(uint8_t* out, uint64_t n, uint64_t m, uint64_t total, int dtype,
                         const uint8_t dec[16]) {
  memset(out, 0, HEADER_BYTES);
  out[0] = 'S'; out[1] = 'Z'; out[2] = 'P'; out[3] = '1';
  put16(out + 4, 1);
  out[6] = (uint8_t)dtype;
  out[7] = 4;
  put32(out + 8, CHUNK);
  put64(out + 16, n);
  put64(out + 24, m);
  put64(out + 32, total);
  memcpy(out + 40, dec, 16);
}

/* ---- compression (section 3.2, encoding path; section 3.4 dummy code) --- */

/* Stage 1: dense transform (split, encode table, nibble pack, store a).
 * Stage 2: scan the exponents again and compact the ones outside the codebook
 * into the chunked position / value arrays.
 * Readings: even element in the low nibble; missing high nibble of an odd N is
 * 0; escapes are listed in ascending element order; positions are relative to
 * 1024-element chunks; per-chunk metadata is a table of u32 exclusive offsets.
 * Returns ORACLE_ERR_CAPACITY (and still reports the sizes) if cap is too
 * small; nothing is written then. */
int oracle_compress(const void* in, uint64_t n, int dtype, const uint8_t dec[16],
                    const uint8_t enc[256], const uint8_t member[256], uint8_t* out, uint64_t cap,
                    uint64_t* total_bytes, uint64_t* n_escapes) {
  if (!dtype_ok(dtype) || (n && !in) || !dec || !enc || !member) return ORACLE_ERR_ARG;
  if (n >= ((uint64_t)1 << 32)) return ORACLE_ERR_ARG; /* u32 offsets */
  const uint16_t* x16 = (const uint16_t*)in;
  const uint8_t* x8 = (const uint8_t*)in;

  uint64_t m = oracle_count_escapes(in, n, dtype, member);
  uint64_t total = oracle_total_bytes(n, m, dtype);
  if (total_bytes) *total_bytes = total;
  if (n_escapes) *n_escapes = m;
  if (!out || cap < total) return ORACLE_ERR_CAPACITY;

  uint64_t c = (n + CHUNK - 1u) / CHUNK;
  uint64_t off_tab = HEADER_BYTES;
  uint64_t off_sm = a256(off_tab + 4u * (c + 1u));
  uint64_t off_code = off_sm + a256(oracle_sm_bytes(n, dtype));
  uint64_t off_pos = off_code + a256((n + 1u) / 2u);
  uint64_t off_val = off_pos + a256(2u * m);

  memset(out, 0, total); /* pads, unused nibbles and tail bits are zero */
  write_header(out, n, m, total, dtype, dec);

  /* stage 1: dense */
  for (uint64_t i = 0; i < n; ++i) {
    unsigned e, a;
    if (dtype == ORACLE_BF16) {
      e = oracle_bf16_exponent(x16[i]);
      a = oracle_bf16_signmant(x16[i]);
      out[off_sm + i] = (uint8_t)a;
    } else {
      e = oracle_e5m2_exponent(x8[i]);
      a = oracle_e5m2_signmant(x8[i]);
      for (unsigned k = 0; k < 3; ++k) {
        uint64_t b = 3u * i + k;
        out[off_sm + (b >> 3)] |= (uint8_t)(((a >> k) & 1u) << (b & 7u));
      }
    }
    unsigned code = member[e] ? enc[e] : 0u; /* dummy code for escapes */
    out[off_code + (i >> 1)] |= (uint8_t)((i & 1u) ? (code << 4) : code);
  }

  /* stage 2: escapes */
  uint64_t k = 0;
  for (uint64_t ch = 0; ch < c; ++ch) {
    put32(out + off_tab + 4u * ch, (uint32_t)k);
    uint64_t lo = ch * CHUNK, hi = lo + CHUNK < n ? lo + CHUNK : n;
    for (uint64_t i = lo; i < hi; ++i) {
      unsigned e = dtype == ORACLE_BF16 ? oracle_bf16_exponent(x16[i]) : oracle_e5m2_exponent(x8[i]);
      if (!member[e]) {
        put16(out + off_pos + 2u * k, (uint16_t)(i - lo));
        out[off_val + k] = (uint8_t)e;
        ++k;
      }
    }
  }
  put32(out + off_tab + 4u * c, (uint32_t)k);
  return ORACLE_OK;
}

/* ---- decompression (section 3.2, decoding path) ------------------------- */

/* Dense pass: unpack nibbles, 16-entry table, recombine with a.  Sparse pass:
 * for every recorded escape overwrite the exponent field of the reconstructed
 * word with the raw exponent.  The stream is validated first (magic, version,
 * dtype, N against the caller's, section sizes, monotone offsets, positions
 * inside their chunk); a bad stream returns ORACLE_ERR_FORMAT and leaves out
 * untouched.  The decoding table is the caller's; the copy in the header must
 * equal it. */
int oracle_decompress(const uint8_t* blob, uint64_t blob_bytes, uint64_t n, int dtype,
                      const uint8_t dec[16], void* out) {
  if (!dtype_ok(dtype) || !blob || !dec || (n && !out)) return ORACLE_ERR_ARG;
  if (blob_bytes < HEADER_BYTES) return ORACLE_ERR_FORMAT;
  if (memcmp(blob, "SZP1", 4) != 0 || get16(blob + 4) != 1 || blob[6] != dtype || blob[7] != 4 ||
      get32(blob + 8) != CHUNK || get32(blob + 12) != 0 || get64(blob + 16) != n)
    return ORACLE_ERR_FORMAT;
  uint64_t m = get64(blob + 24), total = get64(blob + 32);
  if (m > n || total != oracle_total_bytes(n, m, dtype) || total > blob_bytes) return ORACLE_ERR_FORMAT;
  if (memcmp(blob + 40, dec, 16) != 0) return ORACLE_ERR_FORMAT;
  for (unsigned i = 56; i < 64; ++i)
    if (blob[i]) return ORACLE_ERR_FORMAT;

  uint64_t c = (n + CHUNK - 1u) / CHUNK;
  uint64_t off_tab = HEADER_BYTES;
  uint64_t off_sm = a256(off_tab + 4u * (c + 1u));
  uint64_t off_code = off_sm + a256(oracle_sm_bytes(n, dtype));
  uint64_t off_pos = off_code + a256((n + 1u) / 2u);
  uint64_t off_val = off_pos + a256(2u * m);

  if (get32(blob + off_tab) != 0 || get32(blob + off_tab + 4u * c) != m) return ORACLE_ERR_FORMAT;
  for (uint64_t ch = 0; ch < c; ++ch) {
    uint64_t lo = get32(blob + off_tab + 4u * ch), hi = get32(blob + off_tab + 4u * (ch + 1u));
    uint64_t len = (ch + 1u) * CHUNK <= n ? CHUNK : n - ch * CHUNK;
    if (hi < lo || hi - lo > len || hi > m) return ORACLE_ERR_FORMAT;
    for (uint64_t j = lo; j < hi; ++j) {
      unsigned pos = get16(blob + off_pos + 2u * j);
      if (pos >= len) return ORACLE_ERR_FORMAT;
      if (j > lo && pos <= get16(blob + off_pos + 2u * (j - 1u))) return ORACLE_ERR_FORMAT;
      if (blob[off_val + j] >= exp_values(dtype)) return ORACLE_ERR_FORMAT;
    }
  }

  uint16_t* y16 = (uint16_t*)out;
  uint8_t* y8 = (uint8_t*)out;

  /* dense pass */
  for (uint64_t i = 0; i < n; ++i) {
    unsigned byte = blob[off_code + (i >> 1)];
    unsigned code = (i & 1u) ? (byte >> 4) : (byte & 0xfu);
    uint8_t e = dec[code];
    if (dtype == ORACLE_BF16) {
      y16[i] = oracle_bf16_combine(blob[off_sm + i], e);
    } else {
      unsigned a = 0;
      for (unsigned k = 0; k < 3; ++k) {
        uint64_t b = 3u * i + k;
        a |= ((blob[off_sm + (b >> 3)] >> (b & 7u)) & 1u) << k;
      }
      y8[i] = oracle_e5m2_combine((uint8_t)a, e);
    }
  }

  /* sparse overwrite of the exponent field */
  for (uint64_t ch = 0; ch < c; ++ch) {
    uint64_t lo = get32(blob + off_tab + 4u * ch), hi = get32(blob + off_tab + 4u * (ch + 1u));
    for (uint64_t j = lo; j < hi; ++j) {
      uint64_t i = ch * CHUNK + get16(blob + off_pos + 2u * j);
      unsigned e = blob[off_val + j];
      if (dtype == ORACLE_BF16)
        y16[i] = (uint16_t)((y16[i] & ~(0xffu << 7)) | (e << 7));
      else
        y8[i] = (uint8_t)((y8[i] & ~(0x1fu << 2)) | (e << 2));
    }
  }
  return ORACLE_OK;
}
