/*
 * SplitZip format variants of the paper's ablations -- plain, slow,
 * single-threaded C.
 *
 * THIS FILE IS TEST INFRASTRUCTURE, like splitzip_oracle.c beside it: the
 * oracle the GPU library's variant kernels are checked against.  Only the
 * tests and the benchmark's cpu_baseline leg may build or call it.  It shares
 * nothing with the product: the constants are typed in here.
 *
 * What is computed.  The codec of section 3.2 with its knobs turned the way
 * the ablations turn them:
 *
 *   - section "Ablation on Top-k Exponent Coding": a top-8 codebook and 3-bit
 *     codes instead of top-16 and 4-bit codes;
 *   - section "Ablation on Escape-Position Metadata": 15 codebook entries and
 *     the remaining 4-bit code as a sentinel that marks an escaped element;
 *     escaped exponents are kept in element order and no position is stored;
 *   - appendix "Ablation on Chunk Size": chunks of 256 elements with 8-bit
 *     chunk-relative positions; and, in place of chunk-relative positions,
 *     32-bit absolute element indices (no chunking at all);
 *   - appendix "SplitZip on FP8": E5M2 and E4M3 with a 3-bit top-8 code (E5M2
 *     with the 4-bit top-16 code is the main format).
 *
 * A variant is (dtype, code bits, codebook entries k, escape mode, chunk
 * elements, bits per escape value).  Field split, dense coding, escape order and the decoding rule
 * are those of the main format; only widths and the escape representation
 * change.  E4M3 byte = s eeee mmm: e = (x >> 3) & 15, a = ((x >> 4) & 8) |
 * (x & 7), by analogy with eq. (1) (the paper prints no FP8 formula).
 *
 * Stream layout, version 2 (little endian; the offset table follows the
 * header directly, every other section starts 256-byte aligned, pad bytes are
 * zero; A(x) rounds up to 256; C = ceil(N / chunk); sb = bits of a per
 * element: 8, 3, 4 for BF16, E5M2, E4M3; cb = code bits):
 *
 *   header     64 B            see v_write_header()
 *   chunk_off  4*(C+1) B       u32 exclusive prefix sums of per-chunk escape
 *                              counts; absent in the absolute-position mode
 *   sm plane   ceil(N*sb/8) B  LSB-first bit stream: stream bit sb*i+j is bit
 *                              j of a_i (stream bit b = bit b&7 of byte b>>3)
 *   code plane ceil(N*cb/8) B  the same packing with cb bits per element
 *   esc_pos    positions       u16[M] (chunk > 256) or u8[M] chunk-relative;
 *                              nothing in the sentinel mode; u32[M] absolute
 *                              element indices in the absolute mode
 *   esc_val    ceil(M*vb/8) B  raw exponents, element order: whole bytes (vb = 8)
 *                              or an LSB-first bit stream of vb = the exponent
 *                              field's own width (5 for E5M2, 4 for E4M3)
 *
 *   total = A(64 + table) + A(sm) + A(code) + A(positions) + ceil(M*vb/8)
 *
 * With (BF16 or E5M2, 4 bits, k = 16, chunk-relative, 1024) every byte after
 * the header equals the main format's stream; the header differs in the
 * version and the variant bytes only.
 *
 * Readings where the paper is silent: as in splitzip_oracle.c (ties towards
 * the smaller exponent, dummy code 0, ascending element order); codebook
 * slots >= k are written as 0 in the header; the sentinel is the all-ones
 * code; the sentinel mode keeps the per-chunk offset table, because without
 * it no decoder can start anywhere but at element 0 (the paper's size figure
 * for this variant, like all its ratios, counts payload only).
 *
 * Width of an escape value.  Section 3.2 stores the raw exponent of a BF16
 * escape "as an 8-bit integer", which is its own width; the FP8 appendix does
 * not say.  Its table pins both readings: E5M2 top-16 at 0.16 % escapes gives
 * 1.136 only with 24-bit records (16-bit position + a whole byte: 8 / (7 + 24
 * x 0.0016) = 1.1366; 21 bits would give 1.1374), while E5M2 top-8 at 7.72 %
 * and E4M3 top-8 at 7.83 % give 1.049 and 0.933 only with 21 and 20 bits per
 * escape (8 / (6 + 21 x 0.0772) = 1.0497, 8 / (7 + 20 x 0.0783) = 0.9339;
 * whole bytes would give 1.019 and 0.901), i.e. the exponent in its own
 * width.  Both are formats here: vb = 8 (the main format's records) and vb =
 * the exponent's width.  Every printed ratio is matched by one of them to
 * within 0.001 (the paper's ratios include some metadata it does not itemise).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define V_BF16 0
#define V_E5M2 1
#define V_E4M3 2

#define V_ESC_POS 0      /* chunk-relative positions */
#define V_ESC_SENTINEL 1 /* reserved code, values only */
#define V_ESC_ABS32 2    /* absolute u32 positions, no chunks */

#define V_OK 0
#define V_ERR_ARG (-1)
#define V_ERR_CAPACITY (-2)
#define V_ERR_FORMAT (-3)

#define V_HEADER 64u

typedef struct {
  uint32_t dtype;       /* V_BF16 / V_E5M2 / V_E4M3 */
  uint32_t code_bits;   /* 3 or 4 */
  uint32_t k;           /* codebook entries in use */
  uint32_t escape_mode; /* V_ESC_* */
  uint32_t chunk;       /* elements per chunk (power of two, 64..65536); ignored in the absolute mode */
  uint32_t value_bits;  /* bits per escape value: 0 or 8 = whole bytes, else the exponent field's width (5 / 4 for E5M2 / E4M3) */
} oracle_variant;

static uint64_t v_a256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

static unsigned v_elem_bytes(uint32_t dtype) { return dtype == V_BF16 ? 2u : 1u; }
static unsigned v_exp_values(uint32_t dtype) { return dtype == V_BF16 ? 256u : dtype == V_E5M2 ? 32u : 16u; }
static unsigned v_sm_bits(uint32_t dtype) { return dtype == V_BF16 ? 8u : dtype == V_E5M2 ? 3u : 4u; }
static unsigned v_exp_bits(uint32_t dtype) { return dtype == V_BF16 ? 8u : dtype == V_E5M2 ? 5u : 4u; }
static unsigned v_value_bits(const void* vv);

int oracle_v_valid(const oracle_variant* v) {
  if (!v || v->dtype > V_E4M3) return 0;
  if (v->code_bits != 3 && v->code_bits != 4) return 0;
  if (v->escape_mode > V_ESC_ABS32) return 0;
  unsigned codes = 1u << v->code_bits;
  unsigned kmax = v->escape_mode == V_ESC_SENTINEL ? codes - 1u : codes;
  if (v->k < 1 || v->k > kmax || v->k > v_exp_values(v->dtype)) return 0;
  if (v->escape_mode != V_ESC_ABS32) {
    if (v->chunk < 64 || v->chunk > 65536 || (v->chunk & (v->chunk - 1u))) return 0;
  }
  if (v->value_bits != 0 && v->value_bits != 8 && v->value_bits != v_exp_bits(v->dtype)) return 0;
  return 1;
}
static unsigned v_value_bits(const void* vv) {
  const oracle_variant* v = (const oracle_variant*)vv;
  return v->value_bits ? v->value_bits : 8u;
}

/* exponent field and the remaining sign+mantissa bits of one element */
static unsigned v_exponent(uint32_t dtype, unsigned x) {
  return dtype == V_BF16 ? (x >> 7) & 0xffu : dtype == V_E5M2 ? (x >> 2) & 0x1fu : (x >> 3) & 0xfu;
}
static unsigned v_signmant(uint32_t dtype, unsigned x) {
  if (dtype == V_BF16) return ((x >> 8) & 0x80u) | (x & 0x7fu);
  if (dtype == V_E5M2) return ((x >> 5) & 0x4u) | (x & 0x3u);
  return ((x >> 4) & 0x8u) | (x & 0x7u);
}
static unsigned v_combine(uint32_t dtype, unsigned a, unsigned e) {
  if (dtype == V_BF16) return ((a & 0x80u) << 8) | (e << 7) | (a & 0x7fu);
  if (dtype == V_E5M2) return ((a & 0x4u) << 5) | (e << 2) | (a & 0x3u);
  return ((a & 0x8u) << 4) | (e << 3) | (a & 0x7u);
}
static unsigned v_load(const void* p, uint32_t dtype, uint64_t i) {
  return dtype == V_BF16 ? ((const uint16_t*)p)[i] : ((const uint8_t*)p)[i];
}
static void v_store(void* p, uint32_t dtype, uint64_t i, unsigned x) {
  if (dtype == V_BF16) ((uint16_t*)p)[i] = (uint16_t)x;
  else ((uint8_t*)p)[i] = (uint8_t)x;
}

/* ---- sizes ---------------------------------------------------------------- */

static unsigned v_pos_bytes(const oracle_variant* v) {
  if (v->escape_mode == V_ESC_SENTINEL) return 0u;
  if (v->escape_mode == V_ESC_ABS32) return 4u;
  return v->chunk > 256u ? 2u : 1u;
}
static uint64_t v_chunks(uint64_t n, const oracle_variant* v) {
  return v->escape_mode == V_ESC_ABS32 ? 0u : (n + v->chunk - 1u) / v->chunk;
}
static uint64_t v_table_bytes(uint64_t n, const oracle_variant* v) {
  return v->escape_mode == V_ESC_ABS32 ? 0u : 4u * (v_chunks(n, v) + 1u);
}
static uint64_t v_plane_bytes(uint64_t n, unsigned bits) { return (n * bits + 7u) / 8u; }

/* what the paper's size formulas count (section 3.2 and the ablations): the
 * two planes and the escape records */
uint64_t oracle_v_payload_bytes(uint64_t n, uint64_t m, const oracle_variant* v) {
  if (!oracle_v_valid(v)) return 0;
  return v_plane_bytes(n, v_sm_bits(v->dtype)) + v_plane_bytes(n, v->code_bits) + m * v_pos_bytes(v) +
         v_plane_bytes(m, v_value_bits(v));
}

uint64_t oracle_v_total_bytes(uint64_t n, uint64_t m, const oracle_variant* v) {
  if (!oracle_v_valid(v)) return 0;
  return v_a256(V_HEADER + v_table_bytes(n, v)) + v_a256(v_plane_bytes(n, v_sm_bits(v->dtype))) +
         v_a256(v_plane_bytes(n, v->code_bits)) + v_a256(m * v_pos_bytes(v)) + v_plane_bytes(m, v_value_bits(v));
}

/* ---- calibration (section 3.3, with k entries) ------------------------------ */

/* The k most frequent exponent values of the sample, most frequent first; ties
 * towards the smaller value; values that never occur fill up in ascending
 * order.  dec[k..15] = 0. */
int oracle_v_calibrate(const void* sample, uint64_t n, uint32_t dtype, uint32_t k, uint8_t dec[16],
                       uint64_t hist[256]) {
  if (dtype > V_E4M3 || (n && !sample) || !dec || k < 1 || k > 16 || k > v_exp_values(dtype)) return V_ERR_ARG;
  uint64_t h[256];
  memset(h, 0, sizeof h);
  for (uint64_t i = 0; i < n; ++i) h[v_exponent(dtype, v_load(sample, dtype, i))]++;
  uint8_t taken[256];
  memset(taken, 0, sizeof taken);
  memset(dec, 0, 16);
  for (uint32_t j = 0; j < k; ++j) {
    int best = -1;
    for (unsigned e = 0; e < v_exp_values(dtype); ++e) {
      if (taken[e]) continue;
      if (best < 0 || h[e] > h[best]) best = (int)e;
    }
    taken[best] = 1;
    dec[j] = (uint8_t)best;
  }
  if (hist) memcpy(hist, h, sizeof h);
  return V_OK;
}

/* code of every exponent value, or -1 for an exponent outside the codebook */
static int v_tables(const oracle_variant* v, const uint8_t dec[16], int code_of[256]) {
  for (unsigned e = 0; e < 256; ++e) code_of[e] = -1;
  for (uint32_t j = 0; j < v->k; ++j) {
    if (dec[j] >= v_exp_values(v->dtype) || code_of[dec[j]] >= 0) return V_ERR_ARG;
    code_of[dec[j]] = (int)j;
  }
  return V_OK;
}

/* ---- bit streams and little-endian fields ----------------------------------- */

static void put_bits(uint8_t* plane, uint64_t bit0, unsigned nbits, unsigned value) {
  for (unsigned j = 0; j < nbits; ++j) {
    uint64_t b = bit0 + j;
    plane[b >> 3] |= (uint8_t)(((value >> j) & 1u) << (b & 7u));
  }
}
static unsigned get_bits(const uint8_t* plane, uint64_t bit0, unsigned nbits) {
  unsigned value = 0;
  for (unsigned j = 0; j < nbits; ++j) {
    uint64_t b = bit0 + j;
    value |= ((plane[b >> 3] >> (b & 7u)) & 1u) << j;
  }
  return value;
}
static void v_put(uint8_t* p, unsigned bytes, uint64_t x) {
  for (unsigned i = 0; i < bytes; ++i) p[i] = (uint8_t)(x >> (8u * i));
}
static uint64_t v_get(const uint8_t* p, unsigned bytes) {
  uint64_t x = 0;
  for (unsigned i = 0; i < bytes; ++i) x |= (uint64_t)p[i] << (8u * i);
  return x;
}

/* header, 64 bytes:
 *   0  u32 magic 'S','Z','P','1'   4  u16 version = 2   6  u8 dtype   7  u8 code bits
 *   8  u32 chunk elements (0 in the absolute mode)   12  u8 escape mode   13  u8 k
 *  14  u8 bits per escape value if not 8, else 0   15  u8 0
 *  16  u64 N   24  u64 M   32  u64 total bytes   40  u8 dec[16] (slots >= k are 0)   56  u8 reserved[8] = 0 */
static void v_write_header(uint8_t* out, uint64_t n, uint64_t m, uint64_t total, const oracle_variant* v,
                           const uint8_t dec[16]) {
  memset(out, 0, V_HEADER);
  memcpy(out, "SZP1", 4);
  v_put(out + 4, 2, 2);
  out[6] = (uint8_t)v->dtype;
  out[7] = (uint8_t)v->code_bits;
  v_put(out + 8, 4, v->escape_mode == V_ESC_ABS32 ? 0u : v->chunk);
  out[12] = (uint8_t)v->escape_mode;
  out[13] = (uint8_t)v->k;
  out[14] = (uint8_t)(v_value_bits(v) == 8u ? 0u : v_value_bits(v));
  v_put(out + 16, 8, n);
  v_put(out + 24, 8, m);
  v_put(out + 32, 8, total);
  memcpy(out + 40, dec, v->k);
}

typedef struct { uint64_t tab, sm, code, pos, val; } v_offsets;
static v_offsets v_layout(uint64_t n, uint64_t m, const oracle_variant* v) {
  v_offsets o;
  o.tab = V_HEADER;
  o.sm = v_a256(V_HEADER + v_table_bytes(n, v));
  o.code = o.sm + v_a256(v_plane_bytes(n, v_sm_bits(v->dtype)));
  o.pos = o.code + v_a256(v_plane_bytes(n, v->code_bits));
  o.val = o.pos + v_a256(m * v_pos_bytes(v));
  return o;
}

/* ---- compression ------------------------------------------------------------ */

/* One pass over the elements in order: a to the sign+mantissa plane, the code
 * (the dummy code 0 for an escape, or the sentinel in the sentinel mode) to the
 * code plane, and for an escape the record its mode asks for.  Returns
 * V_ERR_CAPACITY, with the sizes still reported, if cap is too small. */
int oracle_v_compress(const void* in, uint64_t n, const oracle_variant* v, const uint8_t dec[16], uint8_t* out,
                      uint64_t cap, uint64_t* total_bytes, uint64_t* n_escapes) {
  if (!oracle_v_valid(v) || (n && !in) || !dec) return V_ERR_ARG;
  if (n >= ((uint64_t)1 << 32)) return V_ERR_ARG;
  int code_of[256];
  if (v_tables(v, dec, code_of) != V_OK) return V_ERR_ARG;

  uint64_t m = 0;
  for (uint64_t i = 0; i < n; ++i)
    if (code_of[v_exponent(v->dtype, v_load(in, v->dtype, i))] < 0) ++m;
  uint64_t total = oracle_v_total_bytes(n, m, v);
  if (total_bytes) *total_bytes = total;
  if (n_escapes) *n_escapes = m;
  if (!out || cap < total) return V_ERR_CAPACITY;

  const v_offsets o = v_layout(n, m, v);
  const unsigned sb = v_sm_bits(v->dtype), cb = v->code_bits, pb = v_pos_bytes(v), vb = v_value_bits(v);
  const unsigned sentinel = (1u << cb) - 1u;
  memset(out, 0, total);
  v_write_header(out, n, m, total, v, dec);

  uint64_t r = 0; /* escapes so far */
  for (uint64_t i = 0; i < n; ++i) {
    if (v->escape_mode != V_ESC_ABS32 && i % v->chunk == 0) v_put(out + o.tab + 4u * (i / v->chunk), 4, r);
    const unsigned x = v_load(in, v->dtype, i);
    const unsigned e = v_exponent(v->dtype, x);
    put_bits(out + o.sm, (uint64_t)sb * i, sb, v_signmant(v->dtype, x));
    if (code_of[e] >= 0) {
      put_bits(out + o.code, (uint64_t)cb * i, cb, (unsigned)code_of[e]);
    } else {
      put_bits(out + o.code, (uint64_t)cb * i, cb, v->escape_mode == V_ESC_SENTINEL ? sentinel : 0u);
      if (v->escape_mode == V_ESC_POS) v_put(out + o.pos + (uint64_t)pb * r, pb, i % v->chunk);
      if (v->escape_mode == V_ESC_ABS32) v_put(out + o.pos + 4u * r, 4, i);
      put_bits(out + o.val, (uint64_t)vb * r, vb, e);   /* vb = 8: the byte out[o.val + r] */
      ++r;
    }
  }
  if (v->escape_mode != V_ESC_ABS32) v_put(out + o.tab + 4u * v_chunks(n, v), 4, r);
  return V_OK;
}

/* ---- decompression ---------------------------------------------------------- */

/* Validates the stream (header fields against the caller's variant, N and
 * table, sizes, monotone offsets, positions in range and ascending, values in
 * the format's exponent range; in the sentinel mode the sentinels of every
 * chunk are counted against the table), then decodes: every element through
 * the table, and escapes either by overwriting the exponent field at the
 * recorded positions or, in the sentinel mode, by taking the next recorded
 * exponent wherever the sentinel stands.  A bad stream returns V_ERR_FORMAT
 * and leaves out untouched. */
int oracle_v_decompress(const uint8_t* blob, uint64_t blob_bytes, uint64_t n, const oracle_variant* v,
                        const uint8_t dec[16], void* out) {
  if (!oracle_v_valid(v) || !blob || !dec || (n && !out)) return V_ERR_ARG;
  int code_of[256];
  if (v_tables(v, dec, code_of) != V_OK) return V_ERR_ARG;
  if (blob_bytes < V_HEADER) return V_ERR_FORMAT;
  if (memcmp(blob, "SZP1", 4) != 0 || v_get(blob + 4, 2) != 2 || blob[6] != v->dtype || blob[7] != v->code_bits ||
      v_get(blob + 8, 4) != (v->escape_mode == V_ESC_ABS32 ? 0u : v->chunk) || blob[12] != v->escape_mode ||
      blob[13] != v->k || blob[14] != (v_value_bits(v) == 8u ? 0u : v_value_bits(v)) || blob[15] != 0 ||
      v_get(blob + 16, 8) != n)
    return V_ERR_FORMAT;
  const uint64_t m = v_get(blob + 24, 8), total = v_get(blob + 32, 8);
  if (m > n || total != oracle_v_total_bytes(n, m, v) || total > blob_bytes) return V_ERR_FORMAT;
  for (unsigned j = 0; j < 16; ++j)
    if (blob[40 + j] != (j < v->k ? dec[j] : 0)) return V_ERR_FORMAT;
  for (unsigned i = 56; i < 64; ++i)
    if (blob[i]) return V_ERR_FORMAT;

  const v_offsets o = v_layout(n, m, v);
  const unsigned sb = v_sm_bits(v->dtype), cb = v->code_bits, pb = v_pos_bytes(v), vb = v_value_bits(v);
  const unsigned sentinel = (1u << cb) - 1u;
  const uint64_t c = v_chunks(n, v);

  for (uint64_t j = 0; j < m; ++j)
    if (get_bits(blob + o.val, (uint64_t)vb * j, vb) >= v_exp_values(v->dtype)) return V_ERR_FORMAT;
  /* the unused bits of the last value byte are zero */
  if ((m * vb) % 8u && (blob[o.val + (m * vb) / 8u] >> ((m * vb) % 8u))) return V_ERR_FORMAT;
  if (v->escape_mode == V_ESC_ABS32) {
    for (uint64_t j = 0; j < m; ++j) {
      const uint64_t p = v_get(blob + o.pos + 4u * j, 4);
      if (p >= n || (j && p <= v_get(blob + o.pos + 4u * (j - 1u), 4))) return V_ERR_FORMAT;
    }
  } else {
    if (v_get(blob + o.tab, 4) != 0 || v_get(blob + o.tab + 4u * c, 4) != m) return V_ERR_FORMAT;
    for (uint64_t ch = 0; ch < c; ++ch) {
      const uint64_t lo = v_get(blob + o.tab + 4u * ch, 4), hi = v_get(blob + o.tab + 4u * (ch + 1u), 4);
      const uint64_t first = ch * v->chunk, len = first + v->chunk <= n ? v->chunk : n - first;
      if (hi < lo || hi - lo > len || hi > m) return V_ERR_FORMAT;
      if (v->escape_mode == V_ESC_POS) {
        for (uint64_t j = lo; j < hi; ++j) {
          const uint64_t p = v_get(blob + o.pos + (uint64_t)pb * j, pb);
          if (p >= len || (j > lo && p <= v_get(blob + o.pos + (uint64_t)pb * (j - 1u), pb))) return V_ERR_FORMAT;
        }
      } else {
        uint64_t seen = 0;
        for (uint64_t i = first; i < first + len; ++i)
          if (get_bits(blob + o.code, (uint64_t)cb * i, cb) == sentinel) ++seen;
        if (seen != hi - lo) return V_ERR_FORMAT;
      }
    }
  }
  /* codes beyond the codebook (other than the sentinel) cannot be decoded */
  for (uint64_t i = 0; i < n; ++i) {
    const unsigned code = get_bits(blob + o.code, (uint64_t)cb * i, cb);
    if (code >= v->k && !(v->escape_mode == V_ESC_SENTINEL && code == sentinel)) return V_ERR_FORMAT;
  }

  /* dense pass */
  uint64_t r = 0;
  for (uint64_t i = 0; i < n; ++i) {
    const unsigned a = get_bits(blob + o.sm, (uint64_t)sb * i, sb);
    const unsigned code = get_bits(blob + o.code, (uint64_t)cb * i, cb);
    unsigned e;
    if (v->escape_mode == V_ESC_SENTINEL && code == sentinel) e = get_bits(blob + o.val, (uint64_t)vb * r++, vb);
    else e = dec[code];
    v_store(out, v->dtype, i, v_combine(v->dtype, a, e));
  }
  /* sparse overwrite of the exponent field */
  if (v->escape_mode == V_ESC_POS) {
    for (uint64_t ch = 0; ch < c; ++ch) {
      const uint64_t lo = v_get(blob + o.tab + 4u * ch, 4), hi = v_get(blob + o.tab + 4u * (ch + 1u), 4);
      for (uint64_t j = lo; j < hi; ++j) {
        const uint64_t i = ch * v->chunk + v_get(blob + o.pos + (uint64_t)pb * j, pb);
        const unsigned a = v_signmant(v->dtype, v_load(out, v->dtype, i));
        v_store(out, v->dtype, i, v_combine(v->dtype, a, get_bits(blob + o.val, (uint64_t)vb * j, vb)));
      }
    }
  } else if (v->escape_mode == V_ESC_ABS32) {
    for (uint64_t j = 0; j < m; ++j) {
      const uint64_t i = v_get(blob + o.pos + 4u * j, 4);
      const unsigned a = v_signmant(v->dtype, v_load(out, v->dtype, i));
      v_store(out, v->dtype, i, v_combine(v->dtype, a, get_bits(blob + o.val, (uint64_t)vb * j, vb)));
    }
  }
  return V_OK;
}

unsigned oracle_v_elem_bytes(uint32_t dtype) { return v_elem_bytes(dtype); }
