// SplitZip for MI355X: the compress kernels (dense transform of both formats, escape staging, the exchange between workgroups, single-tensor and batch kernels).
// Part of the single translation unit splitzip.hip (included inside its anonymous namespace).
#ifndef SPLITZIP_COMPRESS_HPP
#define SPLITZIP_COMPRESS_HPP

// ---------------------------------------------------------------------------
// compress
// ---------------------------------------------------------------------------

// what the dense pass and the trailer need to know of one tensor and its stream
struct Planes {
  Words w;        // the tensor's words (read only here)
  uint8_t* out;
  uint64_t n, capacity;
  uint64_t off_tab, off_sm, off_code, off_pos, sm_bytes, code_bytes;
  uint32_t n_chunks, dtype;
};

__host__ __device__ inline Planes make_planes(const Words& in, void* out, uint64_t n, uint64_t capacity, int dtype) {
  const Layout L = make_layout(n, dtype);
  Planes p;
  p.w = in;
  p.out = static_cast<uint8_t*>(out);
  p.n = n;
  p.capacity = capacity;
  p.off_tab = L.off_tab; p.off_sm = L.off_sm; p.off_code = L.off_code; p.off_pos = L.off_pos;
  p.sm_bytes = L.sm_bytes; p.code_bytes = L.code_bytes;
  p.n_chunks = (uint32_t)L.n_chunks;
  p.dtype = (uint32_t)dtype;
  return p;
}

struct CompressArgs {
  Planes p;
  uint32_t* ws_hdr;      // [0] epoch of this launch, [1] escapes of the earlier segments, [2] sticky error flags
  uint64_t* state;       // one word per workgroup: epoch << 32 | escapes in its range
  uint8_t* val_stage;    // n bytes: escape values of a call of several launches, until M is known
  splitzip_sizes* sizes;
  uint64_t spin_ticks;
  uint32_t seg_chunk0, seg_chunks;   // the chunks this launch covers
  uint32_t flags;        // kSegFirst | kSegLast
  uint32_t expect_wgs;   // workgroups whose counts are awaited (= the grid size)
  const splitzip_codebook* d_cb;   // nullable: a codebook in device memory, used instead of dec / lut below
  uint8_t dec[16];
  uint16_t lut[256];     // exponent -> code | (non-member ? 0x100 : 0)   (the "marked" table of appendix A)
};

// where a chunk's escape records go: LDS staging (first pass) or their final place
struct LdsSink {
  uint16_t* pos;
  uint8_t* val;
  uint32_t tag;   // OR-ed into the position: which of the wave's chunks the record belongs to
  uint32_t cap;   // records the staging holds
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < cap) {
      pos[r] = (uint16_t)(p | tag);
      val[r] = (uint8_t)e;
    }
  }
};
struct GlobalSink {
  uint16_t* pos;
  uint8_t* val;
  uint64_t pos_room, val_room;   // records that fit below the capacity
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < pos_room) pos[r] = (uint16_t)p;
    if (r < val_room) val[r] = (uint8_t)e;
  }
};

// Dense transform of 8 BF16 elements held in four dwords.
//   sm   : 8 sign+mantissa bytes, a = ((x >> 8) & 0x80) | (x & 0x7f)        (eq. (1))
//   code : 8 nibbles, element j in nibble j
//   F    : 8 nibbles, nibble j = 1 if element j is an escape
__device__ inline void encode8_bf16(const uint32_t (&w)[4], const uint16_t* lut, u32x2& sm,
                                    uint32_t& code, uint32_t& F) {
  uint32_t t[4], u[4];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    // bytes 0 and 2 of t hold a of the low / high half-word
    t[d] = (w[d] & 0x007f007fu) | ((w[d] >> 8) & 0x00800080u);
    const uint32_t e0 = (w[d] >> 7) & 0xffu, e1 = (w[d] >> 23) & 0xffu;
    // low byte: code pair; high byte: flag pair in the same nibble layout
    u[d] = (uint32_t)lut[e0] + ((uint32_t)lut[e1] << 4);
  }
  sm.x = byte_perm(t[1], t[0], 0x06040200u);
  sm.y = byte_perm(t[3], t[2], 0x06040200u);
  // x = [code(u_lo), code(u_hi), flag(u_lo), flag(u_hi)]
  const uint32_t x01 = byte_perm(u[1], u[0], 0x05010400u), x23 = byte_perm(u[3], u[2], 0x05010400u);
  code = byte_perm(x23, x01, 0x05040100u);
  F = byte_perm(x23, x01, 0x07060302u);
}

// escape records of one lane's 8 elements (flag nibbles in m), ranks r, r+1, ...
// The lane parks its four dwords in its own 16 bytes of LDS so that the escaping element can be
// picked with a run-time index (registers cannot be indexed that way).
template <typename Sink>
__device__ inline void emit_half_bf16(uint32_t* park, const uint32_t (&w)[4], uint32_t m, uint32_t r,
                                      uint32_t pos0, const Sink& sink) {
  if (m) {
    *reinterpret_cast<u32x4*>(park) = u32x4{w[0], w[1], w[2], w[3]};
    const uint16_t* x = reinterpret_cast<const uint16_t*>(park);
    do {
      const uint32_t jj = (uint32_t)(__ffs(m) - 1) >> 2;
      m &= m - 1;
      sink.put(r, pos0 + jj, ((uint32_t)x[jj] >> 7) & 0xffu);
      ++r;
    } while (m);
  }
}

// One chunk's words into registers: lane l holds elements [8 l, 8 l + 8) of each half-chunk.
// Elements past N read as zero.
template <bool FULL>
__device__ inline void load_chunk_bf16(const Planes& a, const uint8_t* cptr, uint64_t cbase, int lane, uint32_t (&w)[2][4]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;   // first element of this lane's group
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL) {
      // chunk pointer (wave-uniform) + a 32-bit lane offset: no 64-bit vector arithmetic
      const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(cptr) + (uint32_t)(h * 64 + lane));
      w[h][0] = v.x; w[h][1] = v.y; w[h][2] = v.z; w[h][3] = v.w;
    } else if (nvalid == 8) {
      const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(cptr + 2 * (g0 - cbase)));
      w[h][0] = v.x; w[h][1] = v.y; w[h][2] = v.z; w[h][3] = v.w;
    } else {
      const uint16_t* p = reinterpret_cast<const uint16_t*>(cptr + 2 * (g0 - cbase));
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const uint32_t lo = (uint32_t)(2 * d) < nvalid ? p[2 * d] : 0u;
        const uint32_t hi = (uint32_t)(2 * d + 1) < nvalid ? p[2 * d + 1] : 0u;
        w[h][d] = lo | (hi << 16);
      }
    }
  }
}

// One chunk by one wave, its words in w: dense transform, (optionally) plane stores, escape
// ranks inside the chunk, escape records into `sink` starting at rank `base`.
// Returns the chunk's escape count (wave-uniform).
template <bool FULL, bool STORE, typename Sink>
__device__ inline uint32_t process_chunk_bf16(const Planes& a, const uint16_t* lut, uint32_t* park,
                                              uint64_t cbase, int lane, const uint32_t (&w)[2][4], uint32_t base,
                                              const Sink& sink) {
  uint32_t F[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    u32x2 sm;
    uint32_t code;
    encode8_bf16(w[h], lut, sm, code, F[h]);
    if (!FULL) {
      const uint32_t nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
      // elements past N contribute zero nibbles (their sm bytes are already 0)
      const uint32_t keep = nvalid == 8 ? ~0u : ((1u << (4 * nvalid)) - 1u);
      code &= keep;
      F[h] &= keep;
    }
    if (STORE) {
      // Sections are padded to 256 bytes and a lane's group never straddles the padded end, so
      // whole-group stores also write the zero padding.
      if (FULL) {
        st_stream(reinterpret_cast<u32x2*>(a.out + a.off_sm + cbase) + (uint32_t)(h * 64 + lane), sm);
        st_stream(reinterpret_cast<uint32_t*>(a.out + a.off_code + (cbase >> 1)) + (uint32_t)(h * 64 + lane), code);
      } else {
        if (g0 < a256(a.sm_bytes)) st_stream(reinterpret_cast<u32x2*>(a.out + a.off_sm + g0), sm);
        if ((g0 >> 1) < a256(a.code_bytes)) st_stream(reinterpret_cast<uint32_t*>(a.out + a.off_code + (g0 >> 1)), code);
      }
    }
  }
  // escapes per lane; both halves scanned at once (16 bits each: a half has at most 512)
  const uint32_t packed = __popc(F[0]) | (__popc(F[1]) << 16);
  const uint32_t incl = wave_incl_scan(packed);
  const uint32_t tot = wave_last(incl);
  const uint32_t excl = incl - packed;
  const uint32_t tot0 = tot & 0xffffu, total = tot0 + (tot >> 16);
  if (total) {
    // element order inside the chunk: half, lane, element
    emit_half_bf16(park, w[0], F[0], base + (excl & 0xffffu), lane * 8, sink);
    emit_half_bf16(park, w[1], F[1], base + tot0 + (excl >> 16), kHalf + lane * 8, sink);
  }
  return total;
}

// ---- FP8 E5M2 (appendix "SplitZip on FP8"): byte = s eeeee mm, e = (x >> 2) & 31, a = s m1 m0 ----
// One chunk by one wave; lane l owns the 16 consecutive elements [16 l, 16 l + 16): one 16-byte
// load, 8 bytes of codes, 6 bytes of the 3-bit plane (lanes 2p and 2p+1 share 12 bytes: the even
// lane stores 8 of them, the odd lane 4).

// a of the four bytes of w, packed LSB first into 12 bits
__device__ inline uint32_t pack3_e5m2(uint32_t w) {
  const uint32_t t = ((w >> 5) & 0x04040404u) | (w & 0x03030303u);
  const uint32_t x = t + (t << 5);   // bytes 0|1 meet in bits 5..10, bytes 2|3 in bits 21..26; no field overlaps another
  return ((x >> 5) & 0x3fu) | ((x >> 15) & 0xfc0u);
}
// inverse: 12 bits -> the sign and mantissa bits of four bytes, exponent field zero
__device__ inline uint32_t unpack3_e5m2(uint32_t r) {
  const uint32_t u = (r | (r << 10)) & 0x003f003fu;
  const uint32_t t = (u | (u << 5)) & 0x07070707u;
  return ((t & 0x04040404u) << 5) | (t & 0x03030303u);
}

template <bool FULL>
__device__ inline void load_chunk_e5m2(const Planes& a, const uint8_t* cptr, uint64_t cbase, int lane, uint32_t (&w)[4]) {
  const uint64_t g0 = cbase + lane * 16;
  uint32_t nvalid = 16;
  if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 16 ? a.n - g0 : 16);
  if (FULL) {
    const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(cptr) + (uint32_t)lane);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if (nvalid == 16) {
    const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(cptr + (g0 - cbase)));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else {
    const uint8_t* p = cptr + (g0 - cbase);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      uint32_t x = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((uint32_t)(4 * d + j) < nvalid) x |= (uint32_t)p[4 * d + j] << (8 * j);
      w[d] = x;
    }
  }
}

template <bool FULL, bool STORE, typename Sink>
__device__ inline uint32_t process_chunk_e5m2(const Planes& a, const uint16_t* lut, uint32_t* park,
                                              uint64_t cbase, int lane, const uint32_t (&w)[4], uint32_t base,
                                              const Sink& sink) {
  const uint64_t g0 = cbase + lane * 16;
  uint32_t r[4], u[8];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    r[d] = pack3_e5m2(w[d]);
    // entry of a byte: at byte offset (byte & 0x7c) of the table (see kLutShift)
    const uint8_t* lb = reinterpret_cast<const uint8_t*>(lut);
    const uint32_t t0 = *reinterpret_cast<const uint16_t*>(lb + (w[d] & 0x7cu));
    const uint32_t t1 = *reinterpret_cast<const uint16_t*>(lb + ((w[d] >> 8) & 0x7cu));
    const uint32_t t2 = *reinterpret_cast<const uint16_t*>(lb + ((w[d] >> 16) & 0x7cu));
    const uint32_t t3 = *reinterpret_cast<const uint16_t*>(lb + ((w[d] >> 24) & 0x7cu));
    // low byte: code pair; high byte: flag pair in the same nibble layout
    u[2 * d] = t0 + (t1 << 4);
    u[2 * d + 1] = t2 + (t3 << 4);
  }
  // the lane's 48 plane bits: lo holds bits 0..31, hi bits 32..47
  uint32_t lo = r[0] | (r[1] << 12) | (r[2] << 24), hi = (r[2] >> 8) | (r[3] << 4);
  uint32_t code[2], F[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const uint32_t x01 = byte_perm(u[4 * q + 1], u[4 * q], 0x05010400u), x23 = byte_perm(u[4 * q + 3], u[4 * q + 2], 0x05010400u);
    code[q] = byte_perm(x23, x01, 0x05040100u);
    F[q] = byte_perm(x23, x01, 0x07060302u);
  }
  if (!FULL) {
    // elements past N contribute zero nibbles (their plane bits are already 0)
    const uint32_t nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 16 ? a.n - g0 : 16);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const uint32_t nv = nvalid > (uint32_t)(8 * q) ? nvalid - 8 * q : 0u;
      const uint32_t keep = nv >= 8 ? ~0u : ((1u << (4 * nv)) - 1u);
      code[q] &= keep;
      F[q] &= keep;
    }
  }
  if (STORE) {
    // plane bytes of this lane pair: [12 p, 12 p + 12) of the chunk's 384
    // quad_perm [1,1,3,3]: the odd neighbour's bits
    const uint32_t lo_up = __builtin_amdgcn_update_dpp(0u, lo, 0xF5, 0xf, 0xf, false);
    const uint32_t hi_up = __builtin_amdgcn_update_dpp(0u, hi, 0xF5, 0xf, 0xf, false);
    const uint64_t sm_off = (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12;
    uint8_t* sm_dst = a.out + a.off_sm + (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12;   // uniform pointer + lane offset
    // the pair's 12 bytes, all in the even lane
    uint32_t d0 = lo, d1 = (hi & 0xffffu) | (lo_up << 16), d2 = (lo_up >> 16) | (hi_up << 16);
    if (FULL) {
      // Both lanes of a pair write the pair's 12 bytes (quad_perm [0,0,2,2]: the even neighbour's bits): one
      // instruction writes the chunk's 384 bytes back to back, and it is issued whatever the lane -- so the
      // compiler can count on it when it works out how long a wave must wait for the loads issued before it.
      const uint32_t lo_dn = __builtin_amdgcn_update_dpp(0u, lo, 0xA0, 0xf, 0xf, false);
      const uint32_t hi_dn = __builtin_amdgcn_update_dpp(0u, hi, 0xA0, 0xf, 0xf, false);
      d0 = lo_dn; d1 = (hi_dn & 0xffffu) | (lo_up << 16);
      st_stream(reinterpret_cast<u32x3*>(sm_dst), u32x3{d0, d1, d2});
      st_stream(reinterpret_cast<u32x2*>(a.out + a.off_code + (cbase >> 1)) + (uint32_t)lane, u32x2{code[0], code[1]});
    } else {
      // dword by dword up to the padded end of each plane; the pad can reach 128 bytes past the
      // chunk's own 384 plane bytes
      const uint64_t sm_end = a256(a.sm_bytes);
      if (!(lane & 1)) {
        if (sm_off < sm_end) *reinterpret_cast<uint32_t*>(sm_dst) = d0;
        if (sm_off + 4 < sm_end) *reinterpret_cast<uint32_t*>(sm_dst + 4) = d1;
        if (sm_off + 8 < sm_end) *reinterpret_cast<uint32_t*>(sm_dst + 8) = d2;
      }
      const uint64_t past = (cbase / 8) * 3 + 384 + 4 * (uint32_t)lane;
      if (lane < 32 && past < sm_end) *reinterpret_cast<uint32_t*>(a.out + a.off_sm + past) = 0;
      if ((g0 >> 1) < a256(a.code_bytes))
        *reinterpret_cast<u32x2*>(a.out + a.off_code + (g0 >> 1)) = u32x2{code[0], code[1]};
    }
  }
  const uint32_t mine = __popc(F[0]) + __popc(F[1]);
  const uint32_t incl = wave_incl_scan(mine);
  const uint32_t total = wave_last(incl);
  if (total && mine) {
    // element order inside the chunk: lane, element
    *reinterpret_cast<u32x4*>(park) = u32x4{w[0], w[1], w[2], w[3]};
    const uint8_t* x = reinterpret_cast<const uint8_t*>(park);
    uint32_t rr = base + incl - mine;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      uint32_t m = F[q];
      while (m) {
        const uint32_t jj = 8 * q + ((uint32_t)(__ffs(m) - 1) >> 2);
        m &= m - 1;
        sink.put(rr, lane * 16 + jj, ((uint32_t)x[jj] >> 2) & 0x1fu);
        ++rr;
      }
    }
  }
  return total;
}

// the two formats as seen by the compress kernel
struct Bf16 {
  static constexpr int ES = 2;   // bytes per word
  struct Regs { uint32_t w[2][4]; };
  __device__ static inline void arrived(Regs& r) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int d = 0; d < 4; ++d) asm volatile("" : "+v"(r.w[h][d]));
  }
  // batch kernel: two workgroups of 512 per CU, 512 staged escapes per wave.  Against one workgroup of 1024: the
  // same on 64 MiB tensors, 2 to 4 % faster on 4 to 32 MiB ones; four workgroups of 512 (eight waves per SIMD) are
  // no faster, eight of 256 are 3 % slower.
  static constexpr int kBatchThreads = 512, kBatchWgsPerCu = 2, kBatchWavesPerSimd = 4;
  static constexpr uint32_t kBatchStageCap = kStageCap;
  static constexpr int kLutShift = 0;       // the LDS encode table holds the entry of exponent e in slot e
  // a chunk goes the fast way if it is complete (then nothing of a pad is its business: N is a multiple of 1024 there)
  __device__ static inline bool full(const Planes& a, uint64_t cbase) { return cbase + kChunk <= a.n; }
  template <bool FULL>
  __device__ static inline void load(const Planes& a, const uint8_t* cptr, uint64_t cbase, int lane, Regs& r) { load_chunk_bf16<FULL>(a, cptr, cbase, lane, r.w); }
  template <bool FULL, bool STORE, typename Sink>
  __device__ static inline uint32_t process(const Planes& a, const uint16_t* lut, uint32_t* park, uint64_t cbase,
                                            int lane, const Regs& r, uint32_t base, const Sink& sink) {
    return process_chunk_bf16<FULL, STORE>(a, lut, park, cbase, lane, r.w, base, sink);
  }
};
struct E5m2 {
  static constexpr int ES = 1;
  struct Regs { uint32_t w[4]; };
  __device__ static inline void arrived(Regs& r) {
#pragma unroll
    for (int d = 0; d < 4; ++d) asm volatile("" : "+v"(r.w[d]));
  }
  // batch kernel: eight workgroups of 256 per CU, eight waves per SIMD at 64 registers.  Many small workgroups
  // matter more than the wave count: while one of them exchanges counts and writes escape records out, the others
  // keep the CU's memory pipeline busy (measured on 64 tensors of 32 MiB: 1 x 1024 threads 2.2 TB/s, 4 x 256 and
  // 4 x 512 2.45, 8 x 256 2.65).  256 staged escapes per wave are plenty: FP8 exponents miss the codebook far less
  // often than BF16 ones, and a wave that does overflow takes the second pass of write_out.
  static constexpr int kBatchThreads = 256, kBatchWgsPerCu = 8, kBatchWavesPerSimd = 8;
  static constexpr uint32_t kBatchStageCap = 256;
  // The LDS encode table holds the entry of exponent e in slots 2 e and 2 e + 1: its byte offset is then
  // the word's byte with the sign and mantissa bits masked off, one instruction per element.
  static constexpr int kLutShift = 1;
  // the tensor's last chunk always goes the careful way: 384 plane bytes per chunk leave a pad behind an odd chunk count
  __device__ static inline bool full(const Planes& a, uint64_t cbase) { return cbase + kChunk < a.n; }
  template <bool FULL>
  __device__ static inline void load(const Planes& a, const uint8_t* cptr, uint64_t cbase, int lane, Regs& r) { load_chunk_e5m2<FULL>(a, cptr, cbase, lane, r.w); }
  template <bool FULL, bool STORE, typename Sink>
  __device__ static inline uint32_t process(const Planes& a, const uint16_t* lut, uint32_t* park, uint64_t cbase,
                                            int lane, const Regs& r, uint32_t base, const Sink& sink) {
    return process_chunk_e5m2<FULL, STORE>(a, lut, park, cbase, lane, r.w, base, sink);
  }
};

// header, sizes record and the zero padding behind the positions: one wave, once M is known
__device__ void compress_write_trailer(const Planes& a, const uint8_t* dec, splitzip_sizes* sizes, uint32_t M,
                                       uint32_t err_flags, int lane) {
  const uint64_t off_val = a.off_pos + a256(2ull * M);
  const uint64_t total = off_val + M;
  for (uint64_t i = 2ull * M + lane; i < a256(2ull * M); i += 64)
    if (a.off_pos + i < a.capacity) a.out[a.off_pos + i] = 0;
  // chunk_off[C] = M, then zero padding up to the sign+mantissa plane
  uint32_t* tab = reinterpret_cast<uint32_t*>(a.out + a.off_tab);
  for (uint64_t i = (uint64_t)a.n_chunks + lane; a.off_tab + 4 * i < a.off_sm; i += 64) tab[i] = i == a.n_chunks ? M : 0u;
  if (lane == 0) {
    uint32_t h[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) h[i] = 0;
    h[0] = 0x31505a53u;                           // "SZP1"
    h[1] = 1u | (a.dtype << 16) | (4u << 24);      // version, dtype, code bits
    h[2] = kChunk;
    h[4] = (uint32_t)a.n; h[5] = (uint32_t)(a.n >> 32);
    h[6] = M;
    h[8] = (uint32_t)total; h[9] = (uint32_t)(total >> 32);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      h[10 + i] = dec[4 * i] | (dec[4 * i + 1] << 8) | (dec[4 * i + 2] << 16) | ((uint32_t)dec[4 * i + 3] << 24);
    uint4* ho = reinterpret_cast<uint4*>(a.out);
#pragma unroll
    for (int i = 0; i < 4; ++i) ho[i] = make_uint4(h[4 * i], h[4 * i + 1], h[4 * i + 2], h[4 * i + 3]);
    sizes->total_bytes = total;
    sizes->n_escapes = M;
    sizes->status = (total > a.capacity ? SPLITZIP_STATUS_OVERFLOW : 0u) | err_flags;
    sizes->reserved = 0;
  }
}

// ---- building blocks of the compress kernels ----
// A workgroup owns a contiguous range [r0, r0 + nb) of a tensor's chunks, nb <= kMaxRange, dealt
// round-robin to its NW waves (chunk k of the range belongs to wave k mod NW).  LDS per range:
//   stage_pk/val[wave][.]  the wave's escape records, position | (k / NW) << 10 and exponent
//   s_off[k]               escapes of chunk k, after the scan: escapes of the chunks before it
//   s_wstart[k]            records its wave had staged before chunk k
struct RangeLds {
  uint16_t* stage_pk;    // this wave's `cap` entries
  uint8_t* stage_val;
  uint32_t* s_off;       // kMaxRange + 1
  uint16_t* s_wstart;    // kMaxRange
  uint32_t cap;          // escape records a wave can stage
};

// this workgroup's share of `chunks` chunks starting at chunk0: dealt evenly, the first `rem`
// workgroups get one more
__device__ inline void my_range(uint32_t chunk0, uint32_t chunks, uint32_t wgs, uint32_t b, uint32_t& r0, uint32_t& nb) {
  const uint32_t per = chunks / wgs, rem = chunks % wgs;
  nb = per + (b < rem ? 1u : 0u);
  r0 = chunk0 + b * per + (b < rem ? b : rem);
}

struct NoHook {
  __device__ inline void operator()() const {}
};

// dense pass of one wave over its chunks of the range; the loads of the next chunk are issued before
// this chunk is worked on (what a wave has in flight at that point is what keeps the memory system
// busy: 1 to 2 KB per wave).  `mid` is called once, half way through (not at all by a wave without
// chunks).  Returns the wave's escape count.
template <int NW, typename F, typename Hook>
__device__ inline uint32_t dense_pass(const Planes& P, const uint16_t* lut, uint32_t* park, const RangeLds& L,
                                      uint32_t r0, uint32_t nb, int wave, int lane, Hook& mid) {
  uint32_t wave_count = 0;
  const uint32_t mine = nb > (uint32_t)wave ? (nb - wave + NW - 1) / NW : 0u;   // chunks of this wave
  const uint32_t mid_it = mine / 2;
  typename F::Regs w, nx;
  // paged tensor: the pool pages of all of the wave's chunks at once (lane it <-> its it-th chunk), so that no
  // table read stands in front of a chunk's loads later
  uint32_t my_pages = 0;
  if (P.w.table && (uint32_t)lane < mine) my_pages = page_of_chunk(P.w, r0 + wave + (uint32_t)lane * NW);
  // the wave's it-th chunk into r (nothing if it has no such chunk)
  auto fetch = [&](uint32_t it, typename F::Regs& r) {
    if (it < mine) {
      const uint64_t cbase = (uint64_t)(r0 + wave + it * NW) * kChunk;
      const uint8_t* cptr = chunk_at<F::ES>(P.w, cbase, __builtin_amdgcn_readlane(my_pages, it));
      if (F::full(P, cbase)) F::template load<true>(P, cptr, cbase, lane, r);
      else F::template load<false>(P, cptr, cbase, lane, r);
    }
  };
  // Only the tensor's last chunk can be ragged, and it is the last of its wave: the loop takes complete chunks
  // only (no branch between two ways of storing stands between a chunk's loads and the wait for them), the
  // ragged one comes after it.
  const bool last_ragged = mine > 0 && !F::full(P, (uint64_t)(r0 + wave + (mine - 1) * NW) * kChunk);
  const uint32_t fast = mine - (last_ragged ? 1u : 0u);
  auto chunk = [&](uint32_t it, auto complete) {
    const uint32_t k = wave + it * NW;
    const uint64_t cbase = (uint64_t)(r0 + k) * kChunk;
    if (it == mid_it) mid();
    const LdsSink lds{L.stage_pk, L.stage_val, it << 10, L.cap};
    const uint32_t cnt = F::template process<decltype(complete)::value, true>(P, lut, park, cbase, lane, w, wave_count, lds);
    if (lane == 0) {
      L.s_off[k] = cnt;
      L.s_wstart[k] = (uint16_t)(wave_count < 0xffffu ? wave_count : 0xffffu);
    }
    wave_count += cnt;
  };
  fetch(0, w);
  // The first chunk has to be there before the loop is entered: a load still pending on entry would put the
  // compiler's wait into the loop header, where every iteration pays it in full (all loads and stores issued
  // so far), the next chunk's loads included.
  F::arrived(w);
  for (uint32_t it = 0; it < fast; ++it) {
    fetch(it + 1, nx);
    chunk(it, std::true_type{});
    w = nx;
  }
  if (last_ragged) chunk(mine - 1, std::false_type{});
  return wave_count;
}

// one wave: exclusive offsets of the range's chunks, four per lane, in place; s_off[nb] = total
__device__ inline void scan_range(uint32_t* s_off, uint32_t nb, int lane) {
  uint32_t v[4], sum = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t q = 4 * lane + j;
    v[j] = q < nb ? s_off[q] : 0u;
    sum += v[j];
  }
  const uint32_t incl = wave_incl_scan(sum);
  uint32_t run = incl - sum;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t q = 4 * lane + j;
    if (q < nb) s_off[q] = run;
    run += v[j];
  }
  if (lane == 63) s_off[nb] = incl;
}

// one wave: wait until the words of all `wgs` workgroups carry `tag`, then sum the counts of the
// workgroups before b (lower) and of all.  Returns false if the wait was given up: it is bounded
// by spin_ticks of the 100 MHz wall clock (or not begun at all if `dead`).
__device__ inline bool exchange(const uint64_t* state, uint32_t tag, uint32_t wgs, uint32_t b, int lane,
                                uint64_t spin_ticks, bool dead, uint32_t& lower, uint32_t& all) {
  uint32_t lo = 0, al = 0, spins = 0;
  bool ok = !dead;
  const uint64_t t0 = wall_clock64();
  while (ok) {
    lo = 0;
    al = 0;
    int ready = 1;
    for (uint32_t i = lane; i < wgs; i += 64) {
      const uint64_t s = ld_agent(&state[i]);
      if ((uint32_t)(s >> 32) != tag) ready = 0;
      al += (uint32_t)s;
      lo += i < b ? (uint32_t)s : 0u;
    }
    if (__ballot(ready) == ~0ull) break;
    if ((++spins & 15u) == 0 && (uint64_t)(wall_clock64() - t0) > spin_ticks) ok = false;
    else __builtin_amdgcn_s_sleep(1);
  }
  lower = wave_last(wave_incl_scan(lo));
  all = wave_last(wave_incl_scan(al));
  return ok;
}

// all waves: the range's entries of the stream's offset table and this wave's escape records to
// their final rank.  `prefix` = escapes before the range in the whole tensor.
template <int NW, typename F>
__device__ inline void write_out(const Planes& P, const uint16_t* lut, uint32_t* park, const RangeLds& L,
                                 uint32_t r0, uint32_t nb, uint32_t wave_count, uint32_t prefix,
                                 const GlobalSink& g, int tid, int wave, int lane) {
  uint32_t* tab = reinterpret_cast<uint32_t*>(P.out + P.off_tab);
  if ((uint32_t)tid < nb) tab[r0 + tid] = prefix + L.s_off[tid];
  if (wave_count <= L.cap) {
    // staged record i of this wave belongs to chunk k and is the (i - s_wstart[k])-th of it
    for (uint32_t i = lane; i < wave_count; i += 64) {
      const uint32_t pk = L.stage_pk[i], k = (pk >> 10) * NW + wave;
      g.put(prefix + L.s_off[k] + (i - L.s_wstart[k]), pk & 1023u, L.stage_val[i]);
    }
  } else {
    // more escapes than the staging holds: go over this wave's chunks again and write the
    // records straight to their place
    typename F::Regs w;
    for (uint32_t k = wave; k < nb; k += NW) {
      const uint64_t cbase = (uint64_t)(r0 + k) * kChunk;
      const uint32_t r = prefix + L.s_off[k];
      const uint8_t* cptr = chunk_at<F::ES>(P.w, cbase, P.w.table ? page_of_chunk(P.w, r0 + k) : 0u);
      if (F::full(P, cbase)) {
        F::template load<true>(P, cptr, cbase, lane, w);
        F::template process<true, false>(P, lut, park, cbase, lane, w, r, g);
      } else {
        F::template load<false>(P, cptr, cbase, lane, w);
        F::template process<false, false>(P, lut, park, cbase, lane, w, r, g);
      }
    }
  }
}

// where escape records of a tensor go when M is final: positions and, behind them, values
__device__ inline GlobalSink final_sink(const Planes& P, uint32_t M) {
  const uint64_t off_val = P.off_pos + a256(2ull * M);
  GlobalSink g;
  g.pos = reinterpret_cast<uint16_t*>(P.out + P.off_pos);
  g.pos_room = P.capacity > P.off_pos ? (P.capacity - P.off_pos) / 2 : 0;
  g.val = P.out + off_val;
  g.val_room = P.capacity > off_val ? P.capacity - off_val : 0;
  return g;
}

// One launch covers the chunks [seg_chunk0, seg_chunk0 + seg_chunks) with a grid in which every
// workgroup is resident at the same time.  After its dense pass a workgroup publishes the escape
// count of its range in state[b] (tagged with the launch's epoch, so that the words never need
// clearing) and one wave reads the words of all workgroups: the counts before b give its offset,
// all of them give M.  The wait ends when the slowest workgroup has published.
template <int T, typename F>
__global__ __launch_bounds__(T, (T == 1024 ? 8 : 1)) void compress_kernel(const CompressArgs a) {
  constexpr int NW = T / 64;
  static_assert(kMaxRange <= 256 && NW >= 4 && NW <= 16, "one wave scans the range, four chunks per lane");
  __shared__ uint16_t lut[256];
  __shared__ uint16_t stage_pk[NW][kStageCap];
  __shared__ uint8_t stage_val[NW][kStageCap];
  __shared__ uint32_t s_off[kMaxRange + 1];
  __shared__ uint16_t s_wstart[kMaxRange];
  __shared__ u32x4 s_park[T];
  __shared__ uint32_t s_red[16];
  __shared__ uint32_t s_misc[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: loops over chunks stay scalar
  const uint32_t b = blockIdx.x;
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);
  const RangeLds L{stage_pk[wave], stage_val[wave], s_off, s_wstart, kStageCap};

  if (tid < 256) {
    const int e = tid >> F::kLutShift;   // LDS slot tid holds the entry of exponent e
    lut[tid] = a.d_cb ? (a.d_cb->member[e] ? (uint16_t)a.d_cb->enc[e] : (uint16_t)0x100u) : a.lut[e];
  }
  const uint8_t* dec = a.d_cb ? a.d_cb->dec : a.dec;
  const uint32_t epoch = ld_agent(&a.ws_hdr[0]);
  const uint32_t base = (a.flags & kSegFirst) ? 0u : ld_agent(&a.ws_hdr[1]);
  const uint32_t err_before = b == 0 ? ld_agent(&a.ws_hdr[2]) : 0u;   // sticky flags of earlier launches
  const bool single = (a.flags & (kSegFirst | kSegLast)) == (kSegFirst | kSegLast);
  __syncthreads();

  uint32_t r0, nb;
  my_range(a.seg_chunk0, a.seg_chunks, gridDim.x, b, r0, nb);
  NoHook no_hook;
  const uint32_t wave_count = dense_pass<NW, F>(a.p, lut, park, L, r0, nb, wave, lane, no_hook);
  if (lane == 0) s_red[wave] = wave_count;
  __syncthreads();

  if (wave == 0) {
    const uint32_t agg = wave_last(wave_incl_scan(lane < NW ? s_red[lane] : 0u));
    if (lane == 0) st_agent(&a.state[b], ((uint64_t)epoch << 32) | agg);
    uint32_t lo, al;
    const bool ok = exchange(a.state, epoch, a.expect_wgs, b, lane, a.spin_ticks, false, lo, al);
    if (lane == 0) {
      s_misc[0] = base + lo;
      s_misc[1] = base + al;
      s_misc[2] = ok ? 0u : 1u;
    }
    // workgroup 0 closes the launch: it has seen every workgroup's word, so all of them have
    // read the header words
    if (b == 0) {
      const uint32_t err = err_before | (ok ? 0u : (uint32_t)SPLITZIP_STATUS_INTERNAL);
      if (lane == 0) {
        st_agent(&a.ws_hdr[0], epoch + 1u);
        st_agent(&a.ws_hdr[1], base + al);
        st_agent(&a.ws_hdr[2], single ? 0u : err);   // a call of several launches reports in its finishing launch
      }
      if (single) compress_write_trailer(a.p, dec, a.sizes, base + al, err, lane);
    }
  } else if (wave == 1) {
    scan_range(s_off, nb, lane);   // meanwhile
  }
  __syncthreads();
  const uint32_t prefix = s_misc[0], M = s_misc[1];
  const bool timed_out = s_misc[2] != 0;

  if (!timed_out) {
    // values go behind the positions when M is final, else into the workspace
    GlobalSink g = final_sink(a.p, M);
    if (!single) {
      g.val = a.val_stage;
      g.val_room = ~0ull;
    }
    write_out<NW, F>(a.p, lut, park, L, r0, nb, wave_count, prefix, g, tid, wave, lane);
  } else if (tid == 0) {
    __hip_atomic_fetch_or(&a.ws_hdr[2], (uint32_t)SPLITZIP_STATUS_INTERNAL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// ---- several tensors in one launch ----
constexpr uint32_t kBatchMax = 64;     // tensors per launch: their descriptors travel as kernel arguments
constexpr uint32_t kRing = 4;          // exchange slots: a workgroup can be two tensors ahead of the slowest
constexpr uint32_t kRingWgs = 2048;    // words per slot

struct BatchItem {
  const uint8_t* in;
  uint8_t* out;
  uint64_t n, capacity;
};
struct CompressBatchArgs {
  BatchItem item[kBatchMax];
  splitzip_sizes* sizes;     // n_items records
  uint32_t* ws_hdr;          // [0] epoch, [2] sticky error flags, [3] groups that are through
  uint64_t* state;           // per group kRing slots of group_wgs words: (epoch + item) << 32 | escapes in the range
  uint64_t spin_ticks;
  uint32_t n_items, dtype;
  uint32_t group_wgs;        // workgroups that share one tensor; the grid is n_groups * group_wgs
  uint32_t await_extra;      // error-path tests: words awaited beyond the group's
  Words paging;              // table and page geometry shared by all tensors (table null: contiguous tensors); base unused
  uint8_t dec[kBatchMax][16];   // every tensor's codebook, as its 16 decode entries: the kernel builds the encode table from them
  const splitzip_codebook* d_cbs;   // nullable: n_items codebooks in device memory, used instead of dec
  __device__ inline const uint8_t* dec_of(uint32_t k) const { return d_cbs ? d_cbs[k].dec : dec[k]; }
};

// entry of the LDS encode table for exponent e under the codebook dec (wave-uniform): its code, or the escape mark
__device__ inline uint16_t encode_entry(const uint8_t* dec, uint32_t e) {
  uint32_t entry = 0x100u;
#pragma unroll
  for (uint32_t k = 0; k < 16; ++k) entry = dec[k] == e ? k : entry;
  return (uint16_t)entry;
}

// Half way through a dense pass: the loads of the previous tensor's exchange words, so that their
// latency is hidden.  Wave w of the first few waves (one per 256 workgroups a group can have, four at most)
// fetches the words [256 w, 256 w + 256) of the group, four per lane, reduces them at the end of its pass,
// and wave 0 puts the parts together.  A larger group goes without: wave 0 reads its words when it needs them.
struct ExchangePrefetch {
  const uint64_t* slot;
  uint32_t first, wgs;
  int lane;
  bool enabled, issued;
  uint64_t v[4];
  __device__ inline void operator()() {
    if (!enabled) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t i = first + lane + 64 * j;
      v[j] = i < wgs ? ld_agent(&slot[i]) : 0ull;
    }
    issued = true;
  }
  // the wave's part: true if all of its words carry the tag; lower = counts of the workgroups before b, all = of all
  __device__ inline bool reduce(uint32_t tag, uint32_t b, uint32_t& lower, uint32_t& all) const {
    uint32_t lo = 0, al = 0;
    int ready = 1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t q = first + lane + 64 * j;
      if (q < wgs) {
        if ((uint32_t)(v[j] >> 32) != tag) ready = 0;
        al += (uint32_t)v[j];
        lo += q < b ? (uint32_t)v[j] : 0u;
      }
    }
    lower = wave_last(wave_incl_scan(lo));
    all = wave_last(wave_incl_scan(al));
    return __ballot(ready) == ~0ull;
  }
};

// The same persistent grid works through the tensors one after the other, and the exchange of
// tensor i is taken out of the critical path: a workgroup publishes its count for tensor i, then
// completes tensor i - 1 (whose counts every workgroup published a whole dense pass ago; the words
// are even fetched half way through the dense pass of tensor i, so the read costs nothing) and
// goes on to tensor i + 1.  Staging in LDS has three sets (tensor i + 1 may be staged while i - 1 is still written out).  What a single launch pays per
// tensor -- the wait for the slowest workgroup, the exchange, the write-out and the launch itself
// -- is paid once per batch here.  Small tensors are shared by a group of workgroups only; the
// groups work on different tensors at the same time (tensor i belongs to group i mod n_groups).
template <int T, typename F>
__global__ __launch_bounds__(T, F::kBatchWavesPerSimd) void compress_batch_kernel(const CompressBatchArgs a) {
  constexpr int NW = T / 64;
  constexpr uint32_t CAP = F::kBatchStageCap;
  constexpr int PFW = F::kBatchWgsPerCu < 4 ? F::kBatchWgsPerCu : 4;   // waves that fetch exchange words ahead, 256 each: for groups of up to 256 PFW workgroups
  static_assert(PFW <= NW && PFW <= 4, "prefetching waves");
  __shared__ uint32_t s_pf[4][4];          // parts of the waves 1 .. PFW - 1: ready, lower, all
  // the table of the tensor whose dense pass is running, at an address the compiler knows: its lookups carry
  // the table's place as an immediate, one address instruction less per element
  __shared__ uint16_t lut_now[256];
  // the tables of the two tensors before it (a wave whose staging overflowed encodes its chunks again in write_out)
  __shared__ uint16_t lut_old[2][256];
  __shared__ uint16_t stage_pk[3][NW][CAP];   // three sets: a wave may stage tensor i + 1 while another still writes out i - 1
  __shared__ uint8_t stage_val[3][NW][CAP];
  __shared__ uint32_t s_off[3][kMaxRange + 1];
  __shared__ uint16_t s_wstart[3][kMaxRange];
  __shared__ u32x4 s_park[T];
  __shared__ uint32_t s_red[16];
  __shared__ uint32_t s_misc[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t G = a.group_wgs, n_groups = gridDim.x / G;
  const uint32_t grp = blockIdx.x / G, b = blockIdx.x % G;
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);

  if (grp < a.n_items)
    for (int i = tid; i < 256; i += T) lut_now[i] = encode_entry(a.dec_of(grp), (uint32_t)i >> F::kLutShift);
  const uint32_t epoch = ld_agent(&a.ws_hdr[0]);
  const uint32_t err_before = b == 0 ? ld_agent(&a.ws_hdr[2]) : 0u;
  if (tid == 0) s_misc[3] = 0;   // set once an exchange was given up: later ones are not waited for
  __syncthreads();

  uint64_t* const ring = a.state + (uint64_t)grp * kRing * G;   // this group's slots
  Planes Pprev = make_planes(contiguous_words(nullptr), nullptr, 0, 0, (int)a.dtype);
  uint32_t prev_count = 0, prev_r0 = 0, prev_nb = 0, prev_item = 0;
  // this group's tensors: grp, grp + n_groups, ...; seq counts them
  for (uint32_t seq = 0;; ++seq) {
    const uint32_t i = grp + seq * n_groups;
    const bool have = i < a.n_items;
    if (!have && seq == 0) break;   // a group without tensors
    const uint32_t set = seq % 3u;
    const RangeLds L{stage_pk[set][wave], stage_val[set][wave], s_off[set], s_wstart[set], CAP};
    Planes P = Pprev;
    uint32_t r0 = 0, nb = 0, wave_count = 0;
    ExchangePrefetch pf;
    pf.slot = ring + ((seq + kRing - 1) % kRing) * G;
    pf.first = 256u * (uint32_t)wave;
    pf.wgs = G;
    pf.lane = lane;
    pf.enabled = wave < PFW && seq > 0 && G <= 256u * PFW && a.await_extra == 0;
    pf.issued = false;
    if (have) {
      P = make_planes(item_words(a.paging, a.item[i].in), a.item[i].out, a.item[i].n, a.item[i].capacity, (int)a.dtype);
      my_range(0, P.n_chunks, G, b, r0, nb);
      wave_count = dense_pass<NW, F>(P, lut_now, park, L, r0, nb, wave, lane, pf);
      if (lane == 0) s_red[wave] = wave_count;
    }
    if (PFW > 1 && wave > 0 && wave < PFW) {
      uint32_t lo = 0, al = 0;
      // a wave whose words lie beyond the group has nothing to wait for
      const bool ready = pf.first >= G || (pf.issued && pf.reduce(epoch + prev_item, b, lo, al));
      if (lane == 0) {
        s_pf[wave][0] = ready ? 1u : 0u;
        s_pf[wave][1] = lo;
        s_pf[wave][2] = al;
      }
    }
    __syncthreads();
    if (wave == 0) {
      if (have) {
        const uint32_t agg = wave_last(wave_incl_scan(lane < NW ? s_red[lane] : 0u));
        if (lane == 0) st_agent(&ring[(seq % kRing) * G + b], ((uint64_t)(epoch + i) << 32) | agg);
      }
      if (seq > 0) {
        // complete the previous tensor: from the prefetched words if they were all there
        const uint32_t tag = epoch + prev_item;
        uint32_t lo = 0, al = 0;
        bool ok = true, done = false;
        if (pf.issued) {
          done = pf.reduce(tag, b, lo, al);
#pragma unroll
          for (int w = 1; w < PFW; ++w) {
            done = done && s_pf[w][0] != 0;
            lo += s_pf[w][1];
            al += s_pf[w][2];
          }
        }
        if (!done)
          ok = exchange(ring + ((seq - 1) % kRing) * G, tag, G + a.await_extra, b, lane, a.spin_ticks, s_misc[3] != 0, lo, al);
        if (lane == 0) {
          s_misc[0] = lo;
          s_misc[1] = al;
          s_misc[2] = ok ? 0u : 1u;
          if (!ok) s_misc[3] = 1;
        }
        if (b == 0) {
          const uint32_t err = err_before | (ok ? 0u : (uint32_t)SPLITZIP_STATUS_INTERNAL);
          compress_write_trailer(Pprev, a.dec_of(prev_item), a.sizes + prev_item, al, err, lane);
          if (!have && lane == 0) {
            // this group is through.  The last group to get here closes the launch: by then every
            // workgroup has read the header words, because each group completed an exchange.
            const uint32_t through = __hip_atomic_fetch_add(&a.ws_hdr[3], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t active = a.n_items < n_groups ? a.n_items : n_groups;
            if (through + 1 == active) {
              st_agent(&a.ws_hdr[3], 0u);
              st_agent(&a.ws_hdr[2], 0u);
              st_agent(&a.ws_hdr[0], epoch + a.n_items);
            }
          }
        }
      }
    } else if (wave == 1 && have) {
      scan_range(s_off[set], nb, lane);
    } else if (wave == 2 && have) {
      // Every dense pass of tensor i is over: its table is kept for its write-out, and the table of this group's
      // next tensor takes its place -- every entry the escape mark, then the 16 codes by the lanes that own them.
      // One wave does all of it: its LDS accesses are carried out in program order.
      const bool more = i + n_groups < a.n_items;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        lut_old[seq & 1u][4 * lane + q] = lut_now[4 * lane + q];
        if (more) lut_now[4 * lane + q] = 0x100u;
      }
      if (more && lane < 16) {
        const uint32_t e = a.dec_of(i + n_groups)[lane] & ((256u >> F::kLutShift) - 1u);   // whatever a device codebook holds, the table is not left
#pragma unroll
        for (int q = 0; q < (1 << F::kLutShift); ++q) lut_now[(e << F::kLutShift) + q] = (uint16_t)lane;
      }
    }
    __syncthreads();
    if (seq > 0 && s_misc[2] == 0) {
      const uint32_t pset = (seq + 2u) % 3u;
      const RangeLds Lp{stage_pk[pset][wave], stage_val[pset][wave], s_off[pset], s_wstart[pset], CAP};
      write_out<NW, F>(Pprev, lut_old[(seq + 1u) & 1u], park, Lp, prev_r0, prev_nb, prev_count, s_misc[0],
                       final_sink(Pprev, s_misc[1]), tid, wave, lane);
    }
    if (!have) break;
    // no barrier here: the next tensor is staged in the third LDS set, and s_misc / s_red are only
    // rewritten behind the next barrier, which every wave reaches after its write-out
    Pprev = P;
    prev_count = wave_count;
    prev_r0 = r0;
    prev_nb = nb;
    prev_item = i;
  }
}

// Last launch of a call that took several: M is known now.  Moves the staged escape values
// behind the position array and writes the trailer.
__global__ __launch_bounds__(kThreads) void compress_finish_kernel(const CompressArgs a) {
  const uint32_t M = ld_agent(&a.ws_hdr[1]);
  const uint64_t off_val = a.p.off_pos + a256(2ull * M);
  const uint64_t room = a.p.capacity > off_val ? a.p.capacity - off_val : 0;
  const uint64_t m = M < room ? M : room;
  const uint64_t nvec = m / 16;
  const u32x4* src = reinterpret_cast<const u32x4*>(a.val_stage);
  u32x4* dst = reinterpret_cast<u32x4*>(a.p.out + off_val);
  const uint64_t gtid = blockIdx.x * (uint64_t)kThreads + threadIdx.x, gsz = (uint64_t)gridDim.x * kThreads;
  for (uint64_t i = gtid; i < nvec; i += gsz) dst[i] = src[i];
  for (uint64_t i = nvec * 16 + gtid; i < m; i += gsz) a.p.out[off_val + i] = a.val_stage[i];
  if (blockIdx.x == 0 && threadIdx.x < 64) {
    uint32_t err = 0;
    if (threadIdx.x == 0) {
      err = ld_agent(&a.ws_hdr[2]);
      st_agent(&a.ws_hdr[2], 0u);
    }
    compress_write_trailer(a.p, a.d_cb ? a.d_cb->dec : a.dec, a.sizes, M, err, threadIdx.x);
  }
}

#endif  // SPLITZIP_COMPRESS_HPP
