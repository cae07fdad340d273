// SplitZip for MI355X: the compress kernels (dense transform of both formats with escape staging, one tile per workgroup; the finishing pass that ranks and places the escape records; the trailer).
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
// a tile's slot in the staging area: records in the order of the tile's elements, position | exponent << 16
struct SlotSink {
  uint32_t* slot;
  uint32_t cap;   // records the slot holds
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < cap) slot[r] = p | (e << 16);
  }
};
// the final place of the records of a tensor: positions and, behind them, values
struct FinalSink {
  uint16_t* pos;
  uint8_t* val;
  uint64_t pos_room, val_room;   // records that fit below the capacity
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < pos_room) pos[r] = (uint16_t)p;
    if (r < val_room) val[r] = (uint8_t)e;
  }
};
// counting only
struct NullSink {
  __device__ inline void put(uint32_t, uint32_t, uint32_t) const {}
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
  // escapes per lane and half, ranked over the wave; element order inside the chunk: half, lane, element
  uint32_t excl0, excl1;
  const uint32_t tot0 = wave_sparse_excl(__popc(F[0]), excl0), tot1 = wave_sparse_excl(__popc(F[1]), excl1);
  const uint32_t total = tot0 + tot1;
  if (total) {
    emit_half_bf16(park, w[0], F[0], base + excl0, lane * 8, sink);
    emit_half_bf16(park, w[1], F[1], base + tot0 + excl1, kHalf + lane * 8, sink);
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
    // (a quad permute reads lanes of its own quad only: every lane gets a value, the old one is never kept)
    const uint32_t lo_up = __builtin_amdgcn_mov_dpp(lo, 0xF5, 0xf, 0xf, false);
    const uint32_t hi_up = __builtin_amdgcn_mov_dpp(hi, 0xF5, 0xf, 0xf, false);
    const uint64_t sm_chunk = (uint64_t)(uint32_t)(cbase >> 10) * 384u;   // the chunk's plane bytes start here: a scalar product
    const uint64_t sm_off = sm_chunk + (uint32_t)(lane >> 1) * 12;
    uint8_t* sm_chunk_ptr = a.out + a.off_sm + sm_chunk;
    uint8_t* sm_dst = sm_chunk_ptr + (uint32_t)(lane >> 1) * 12;
    // the pair's 12 bytes, all in the even lane
    uint32_t d0 = lo, d1 = (hi & 0xffffu) | (lo_up << 16), d2 = (lo_up >> 16) | (hi_up << 16);
    if (FULL) {
      // Both lanes of a pair write the pair's 12 bytes (quad_perm [0,0,2,2]: the even neighbour's bits): one
      // instruction writes the chunk's 384 bytes back to back, and it is issued whatever the lane -- so the
      // compiler can count on it when it works out how long a wave must wait for the loads issued before it.
      const uint32_t lo_dn = __builtin_amdgcn_mov_dpp(lo, 0xA0, 0xf, 0xf, false);
      const uint32_t hi_dn = __builtin_amdgcn_mov_dpp(hi, 0xA0, 0xf, 0xf, false);
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
      const uint64_t past = sm_chunk + 384 + 4 * (uint32_t)lane;
      if (lane < 32 && past < sm_end) *reinterpret_cast<uint32_t*>(a.out + a.off_sm + past) = 0;
      if ((g0 >> 1) < a256(a.code_bytes))
        *reinterpret_cast<u32x2*>(a.out + a.off_code + (g0 >> 1)) = u32x2{code[0], code[1]};
    }
  }
  const uint32_t mine = __popc(F[0]) + __popc(F[1]);
  uint32_t excl;
  const uint32_t total = wave_sparse_excl(mine, excl);
  if (total && mine) {
    // element order inside the chunk: lane, element
    *reinterpret_cast<u32x4*>(park) = u32x4{w[0], w[1], w[2], w[3]};
    const uint8_t* x = reinterpret_cast<const uint8_t*>(park);
    uint32_t rr = base + excl;
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
  // A workgroup of four waves takes a tile of 4 x kCpt chunks (16 KB of words).  Four workgroups per CU serve BF16
  // best (one launch pair over 64 tensors of 64 MiB: 1245-1259 us against 1266-1268 us with five, 1298 us with
  // eight and 1306 us with three); unused LDS asked for at the launch sets the number.
  static constexpr uint32_t kCpt = 2;
  static constexpr int kWavesPerSimd = 8;
  static constexpr uint32_t kTileLdsPad = 28000;
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
  // a tile of 4 x kCpt chunks is 16 KB of words here too; eight workgroups per CU (730 us for 64 tensors of 32 MiB
  // against 750 us with six and 790 us with five)
  static constexpr uint32_t kCpt = 4;
  static constexpr int kWavesPerSimd = 8;
  static constexpr uint32_t kTileLdsPad = 0;
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

// ---- the two passes of a compress call ----
// Pass 1, compress_tile_kernel: one workgroup of four waves per tile of 4 x cpt chunks (16 KB of words), started by
// the hardware in the order of the tiles -- the access pattern the memory system likes best, see
// traffic_shape_kernel.  A workgroup waits for nobody: planes out; escapes of the tile staged in LDS, then written
// as (position | exponent << 16) records, in element order, to the tile's slot of the staging area; the tile's
// entries of the offset table as offsets inside the tile; the tile's escape count to the status area.
// Pass 2, compress_finish_kernel: one workgroup per group of 16 tiles.  It sums the counts (all of the tensor's:
// M; those before the group: its first rank), adds what lies before each tile to the tile's table entries and
// moves the records from the slots to their ranks in the position and value arrays.  A tile with more escapes
// than its slot (or its LDS staging) holds is encoded once more from the words, straight to the final place.
// Between the passes lies a kernel boundary: no workgroup ever waits for another, nothing needs to be resident
// together, and no word of the workspace needs a defined value before a call.
constexpr uint32_t kTileThreads = 256;
constexpr uint32_t kGroup = 16;             // tiles per group of the finishing pass
constexpr uint32_t kFinishMost = 4;         // groups per workgroup of the finishing pass, at most
constexpr uint32_t kSlotAhead = 16;         // threads per tile that fetch records before the finishing pass knows the counts, two records each
constexpr uint32_t kTileStageCap = 256;     // escapes a wave can stage in LDS
constexpr uint32_t kSlotCapMost = 1024;     // records per tile slot, at most
constexpr uint32_t kDirectTiles = 4096;     // up to this many tiles per tensor the finishing pass sums the tile counts itself ...
constexpr uint64_t kDirectBytes = 128ull << 20;   // ... if all its workgroups together read no more than this many bytes of counts
constexpr uint32_t kSumGroup = 64;          // beyond: sums of this many tile counts, by tile_group_sum_kernel
constexpr uint32_t kBatchMax = 64;          // tensors per launch: their descriptors travel as kernel arguments
constexpr uint32_t kRedo = 0x80000000u;     // in a tile's count: its records are not in its slot
static_assert(kGroup * kSlotAhead == kTileThreads, "every thread fetches records of one tile ahead");

struct TileItem {
  const uint8_t* in;
  uint8_t* out;
  uint64_t n, capacity;
};
struct TileArgs {
  TileItem item[kBatchMax];
  splitzip_sizes* sizes;          // n_items records
  uint8_t* status;                // per tensor: u32 count of every tile, then u32 sum of every kSumGroup tiles
  uint8_t* stage;                 // per tensor stage_cap bytes: the tiles' slots
  uint64_t stage_cap;
  uint32_t status_off[kBatchMax]; // where a tensor's counts start in `status`
  uint32_t n_items, dtype;
  uint32_t cpt;                   // chunks per wave and tile, a power of two
  uint32_t tile_shift;            // log2 of the chunks per tile (4 cpt)
  uint32_t slot_cap;              // records per tile slot (the same for all tensors of the launch)
  uint32_t finish_groups;         // groups of kGroup tiles per workgroup of the finishing pass, 1 to kFinishMost
  uint32_t use_group_sums;        // the finishing pass reads sums of kSumGroup tile counts (tile_group_sum_kernel) instead of all tile counts
  Words paging;                   // table and page geometry shared by all tensors (table null: contiguous tensors); base unused
  const splitzip_codebook* d_cbs; // nullable: n_items codebooks in device memory, used instead of dec
  uint8_t dec[kBatchMax][16];     // every tensor's codebook, as its 16 decode entries: the kernels build the encode table from them
  __device__ inline const uint8_t* dec_of(uint32_t k) const { return d_cbs ? d_cbs[k].dec : dec[k]; }
  __device__ inline u32x4 dec16_of(uint32_t k) const { return d_cbs ? load_dec16(d_cbs[k].dec) : dec16_from(dec[k]); }
};

// what both passes derive from the arguments for one tensor
struct TileGeom {
  Planes P;
  uint32_t tile_chunks, n_tiles;
  uint32_t* counts;      // n_tiles
  uint32_t* group_sums;  // ceil(n_tiles / kSumGroup)
  uint32_t* slots;       // n_tiles x slot_cap records
};
__device__ inline TileGeom tile_geom(const TileArgs& a, uint32_t item) {
  TileGeom g;
  const TileItem it = a.item[item];
  g.P = make_planes(item_words(a.paging, it.in), it.out, it.n, it.capacity, (int)a.dtype);
  g.tile_chunks = 1u << a.tile_shift;
  g.n_tiles = (g.P.n_chunks + g.tile_chunks - 1) >> a.tile_shift;
  g.counts = reinterpret_cast<uint32_t*>(a.status + a.status_off[item]);
  g.group_sums = g.counts + g.n_tiles;
  g.slots = reinterpret_cast<uint32_t*>(a.stage + (uint64_t)item * a.stage_cap);
  return g;
}

// The LDS encode table (exponent e in slots e << shift ... : its code, or the escape mark 0x100) from the 16 decode
// entries of the codebook, by the first wave of the workgroup alone: escape marks everywhere, then the 16 codes on
// top (the LDS takes a wave's writes in order); the caller's barrier makes it visible to the others.  Entries that
// are no exponent of the format (a codebook in device memory is not the host's to check) are left out.
__device__ inline void build_encode_table(uint16_t* lut, const u32x4& d, int tid, int shift) {
  if (tid < 64) {
#pragma unroll
    for (int q = 0; q < 4; ++q) lut[q * 64 + tid] = 0x100u;
    const uint32_t k = (uint32_t)tid >> shift, sub = (uint32_t)tid & ((1u << shift) - 1u);
    const uint32_t e = dec16_at(d, k & 15u);
    if (k < 16 && e < (256u >> shift)) lut[(e << shift) + sub] = (uint16_t)k;
  }
}

// a barrier for LDS traffic only: global loads that are on their way stay on their way
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// CPT: chunks of a wave whose loads are issued together, before anything else happens in the workgroup.  Wave w of
// the tile owns the chunks [w cpt, w cpt + cpt) of the tile.
template <typename F, int CPT>
__global__ __launch_bounds__(kTileThreads, F::kWavesPerSimd) void compress_tile_kernel(const TileArgs a) {
  constexpr int NW = kTileThreads / 64;
  __shared__ uint16_t lut[256];
  __shared__ uint16_t stage_pk[NW][kTileStageCap];
  __shared__ uint8_t stage_val[NW][kTileStageCap];
  __shared__ u32x4 s_park[kTileThreads];
  __shared__ uint32_t s_cnt[NW];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t item = blockIdx.y;
  const TileGeom G = tile_geom(a, item);
  const Planes& P = G.P;
  const uint32_t t = blockIdx.x;
  if (t >= G.n_tiles) return;
  const uint32_t r0 = t << a.tile_shift, nb = P.n_chunks - r0 < G.tile_chunks ? P.n_chunks - r0 : G.tile_chunks;
  const uint32_t w0 = (uint32_t)wave * a.cpt;                                   // the wave's first chunk inside the tile
  const uint32_t mine = nb > w0 ? (nb - w0 < a.cpt ? nb - w0 : a.cpt) : 0u;     // and how many it has
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);

  uint32_t wave_count = 0, my_start = 0;   // lane it: escapes of the wave before its it-th chunk
  const LdsSink lds{stage_pk[wave], stage_val[wave], 0u, kTileStageCap};
  typename F::Regs w[CPT];
  // A tile all of whose chunks are complete (every tile but a tensor's last, as a rule) takes a path without a
  // condition per chunk: nothing stands between the loads, and the compiler need not merge the registers of two
  // ways of loading a chunk.
  const uint32_t r_last = r0 + G.tile_chunks - 1;
  if (nb == G.tile_chunks && F::full(P, (uint64_t)r_last * kChunk)) {
    auto fetch = [&](uint32_t it0) {
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        const uint64_t cbase = (uint64_t)(r0 + w0 + it0 + j) * kChunk;
        const uint8_t* cptr = chunk_at<F::ES>(P.w, cbase, P.w.table ? page_of_chunk(P.w, r0 + w0 + it0 + j) : 0u);
        F::template load<true>(P, cptr, cbase, lane, w[j]);
      }
    };
    // the words first: the table is built while they are on their way
    fetch(0);
    build_encode_table(lut, a.dec16_of(item), tid, F::kLutShift);
    lds_barrier();
    for (uint32_t it0 = 0; it0 < a.cpt; it0 += CPT) {
      if (it0 > 0) fetch(it0);   // tiles of more than CPT chunks per wave (very large tensors)
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        if ((uint32_t)lane == it0 + j) my_start = wave_count;
        wave_count += F::template process<true, true>(P, lut, park, (uint64_t)(r0 + w0 + it0 + j) * kChunk, lane, w[j], wave_count, lds);
      }
    }
  } else {
    // the wave's chunks [it0, it0 + CPT) into w (nothing for chunks it does not have)
    auto fetch = [&](uint32_t it0) {
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        const uint32_t it = it0 + j;
        if (it < mine) {
          const uint64_t cbase = (uint64_t)(r0 + w0 + it) * kChunk;
          const uint8_t* cptr = chunk_at<F::ES>(P.w, cbase, P.w.table ? page_of_chunk(P.w, r0 + w0 + it) : 0u);
          if (F::full(P, cbase)) F::template load<true>(P, cptr, cbase, lane, w[j]);
          else F::template load<false>(P, cptr, cbase, lane, w[j]);
        }
      }
    };
    fetch(0);
    build_encode_table(lut, a.dec16_of(item), tid, F::kLutShift);
    lds_barrier();
    // dense pass; the wave's escape records into its LDS staging in element order, the chunks' counts kept in lanes
    for (uint32_t it0 = 0; it0 < mine; it0 += CPT) {
      if (it0 > 0) fetch(it0);
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        const uint32_t it = it0 + j;
        if (it >= mine) break;
        const uint64_t cbase = (uint64_t)(r0 + w0 + it) * kChunk;
        if ((uint32_t)lane == it) my_start = wave_count;
        wave_count += F::full(P, cbase) ? F::template process<true, true>(P, lut, park, cbase, lane, w[j], wave_count, lds)
                                        : F::template process<false, true>(P, lut, park, cbase, lane, w[j], wave_count, lds);
      }
    }
  }
  if (lane == 0) s_cnt[wave] = wave_count;
  lds_barrier();
  uint32_t before = 0, total = 0;
  bool redo = false;
#pragma unroll
  for (int q = 0; q < NW; ++q) {
    const uint32_t c = s_cnt[q];
    before += q < wave ? c : 0u;
    total += c;
    redo = redo || c > kTileStageCap;
  }
  redo = redo || total > a.slot_cap;
  // the tile's entries of the offset table, for now as offsets inside the tile
  uint32_t* tab = reinterpret_cast<uint32_t*>(P.out + P.off_tab);
  if ((uint32_t)lane < mine) tab[r0 + w0 + lane] = before + my_start;
  if (!redo) {
    uint32_t* slot = G.slots + (uint64_t)t * a.slot_cap + before;   // staged record i of this wave is the (before + i)-th of the tile
    for (uint32_t i = lane; i < wave_count; i += 64) slot[i] = (uint32_t)stage_pk[wave][i] | ((uint32_t)stage_val[wave][i] << 16);
  }
  if (tid == 0) G.counts[t] = total | (redo ? kRedo : 0u);
}

// sums of kSumGroup tile counts each, for tensors of more than kDirectTiles tiles (one wave per sum)
__global__ __launch_bounds__(64) void tile_group_sum_kernel(const TileArgs a) {
  const TileGeom G = tile_geom(a, blockIdx.y);
  const uint32_t g = blockIdx.x, t = g * kSumGroup + threadIdx.x;
  if (g * kSumGroup >= G.n_tiles) return;
  const uint32_t sum = wave_last(wave_incl_scan(t < G.n_tiles ? G.counts[t] & ~kRedo : 0u));
  if (threadIdx.x == 0) G.group_sums[g] = sum;
}

template <typename F>
__global__ __launch_bounds__(kTileThreads) void compress_finish_kernel(const TileArgs a) {
  constexpr int NW = kTileThreads / 64;
  static_assert(kFinishMost <= NW, "one wave scans the counts of one group");
  __shared__ uint16_t lut[256];
  __shared__ u32x4 s_park[kTileThreads];
  __shared__ uint32_t s_cnt[kFinishMost][kGroup];       // the counts of the groups' tiles, redo mark included
  __shared__ uint32_t s_tp[kFinishMost][kGroup + 1];    // escapes of a group's tiles before each tile
  __shared__ uint32_t s_red[2 * NW];
  __shared__ uint32_t s_more[kFinishMost];              // a group has a tile with more records than were fetched ahead
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t item = blockIdx.y;
  const TileGeom G = tile_geom(a, item);
  const Planes& P = G.P;
  const uint32_t n_groups = (G.n_tiles + kGroup - 1) / kGroup;
  // the workgroup's groups: [g0, g0 + ng) -- a.finish_groups of them in a row (1 to kFinishMost: a launch of many
  // groups gives every workgroup several, so that fewer rounds of workgroups pass through the chip; each round
  // costs the same few trips to memory whatever it carries)
  const uint32_t g0 = blockIdx.x * a.finish_groups;
  if (g0 >= (n_groups ? n_groups : 1u)) return;   // a tensor without elements still gets its header
  const uint32_t ng = n_groups - g0 < a.finish_groups ? (n_groups > g0 ? n_groups - g0 : 1u) : a.finish_groups;
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);
  uint32_t* tab = reinterpret_cast<uint32_t*>(P.out + P.off_tab);
  const uint32_t group_entries = kGroup << a.tile_shift;

  // Everything whose address does not depend on the counts is fetched at once: the counts themselves, the
  // groups' table entries (one per thread and group, or a few) and the first 2 kSlotAhead records of every tile's slot
  // (two per thread: hardly a tile has more, so hardly a workgroup has to go to memory once more after the barrier).
  const uint32_t sl = (uint32_t)tid / kSlotAhead, sj = (uint32_t)tid % kSlotAhead;   // tile of a group, record of the tile
  uint32_t my_entry[kFinishMost], rec_ahead[kFinishMost], rec_ahead2[kFinishMost];
#pragma unroll
  for (uint32_t q = 0; q < kFinishMost; ++q) {
    my_entry[q] = 0;
    rec_ahead[q] = 0;
    rec_ahead2[q] = 0;
    if (q < ng) {
      const uint32_t t0 = (g0 + q) * kGroup, c0 = t0 << a.tile_shift;
      if (c0 + tid < P.n_chunks && (uint32_t)tid < group_entries) my_entry[q] = tab[c0 + tid];
      if (t0 + sl < G.n_tiles && sj < a.slot_cap) rec_ahead[q] = G.slots[(uint64_t)(t0 + sl) * a.slot_cap + sj];
      if (t0 + sl < G.n_tiles && sj + kSlotAhead < a.slot_cap) rec_ahead2[q] = G.slots[(uint64_t)(t0 + sl) * a.slot_cap + sj + kSlotAhead];
    }
  }
  const uint32_t t_first = g0 * kGroup;   // the first tile of the workgroup's first group
  uint32_t before = 0, all = 0;
  if (a.use_group_sums) {
    const uint32_t n_sums = (G.n_tiles + kSumGroup - 1) / kSumGroup, whole = t_first / kSumGroup;   // sums that lie before the first group entirely
    for (uint32_t i = tid; i < n_sums; i += kTileThreads) {
      const uint32_t c = G.group_sums[i];
      all += c;
      before += i < whole ? c : 0u;
    }
    for (uint32_t i = whole * kSumGroup + tid; i < t_first; i += kTileThreads) before += G.counts[i] & ~kRedo;
  } else {
    // four counts per load, four loads per thread on their way at a time (the counts start 256-byte aligned and
    // the sums behind them pad the last vector)
    const u32x4* cv = reinterpret_cast<const u32x4*>(G.counts);
    const uint32_t nvec = (G.n_tiles + 3) / 4;
    for (uint32_t v0 = 0; v0 < nvec; v0 += 4 * kTileThreads) {
      u32x4 v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t idx = v0 + q * kTileThreads + tid;
        v[q] = idx < nvec ? cv[idx] : u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t e = 4 * (v0 + q * kTileThreads + tid);
        const uint32_t c[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
        for (int z = 0; z < 4; ++z) {
          const uint32_t cz = e + z < G.n_tiles ? c[z] & ~kRedo : 0u;
          all += cz;
          before += e + z < t_first ? cz : 0u;
        }
      }
    }
  }
  before = wave_last(wave_incl_scan(before));
  all = wave_last(wave_incl_scan(all));
  if (lane == 0) {
    s_red[wave] = before;
    s_red[NW + wave] = all;
  }
  if ((uint32_t)wave < ng) {
    // wave q: the counts of the tiles of group q, and what lies before each inside the group
    const uint32_t t0 = (g0 + (uint32_t)wave) * kGroup;
    const uint32_t c = (uint32_t)lane < kGroup && t0 + lane < G.n_tiles ? G.counts[t0 + lane] : 0u;
    const uint32_t incl = wave_incl_scan(c & ~kRedo);
    if ((uint32_t)lane < kGroup) {
      s_cnt[wave][lane] = c;
      s_tp[wave][lane] = incl - (c & ~kRedo);
    }
    if (lane == 63) s_tp[wave][kGroup] = incl;
    const uint64_t more = __ballot((c & ~kRedo) > 2 * kSlotAhead && !(c & kRedo));
    if (lane == 0) s_more[wave] = more != 0;
  }
  build_encode_table(lut, a.dec16_of(item), tid, F::kLutShift);
  __syncthreads();
  uint32_t first = 0, M = 0;   // the rank of the first record of the group at hand; all records of the tensor
#pragma unroll
  for (int q = 0; q < NW; ++q) {
    first += s_red[q];
    M += s_red[NW + q];
  }
  const uint64_t off_val = P.off_pos + a256(2ull * M);
  FinalSink fin;
  fin.pos = reinterpret_cast<uint16_t*>(P.out + P.off_pos);
  fin.pos_room = P.capacity > P.off_pos ? (P.capacity - P.off_pos) / 2 : 0;
  fin.val = P.out + off_val;
  fin.val_room = P.capacity > off_val ? P.capacity - off_val : 0;

#pragma unroll
  for (uint32_t q = 0; q < kFinishMost; ++q) {
    if (q >= ng) break;
    const uint32_t t0 = (g0 + q) * kGroup, c0 = t0 << a.tile_shift;
    const uint32_t entries = P.n_chunks > c0 ? (P.n_chunks - c0 < group_entries ? P.n_chunks - c0 : group_entries) : 0u;
    const uint32_t* cnt = s_cnt[q];
    const uint32_t* tp = s_tp[q];
    // tiles whose records are not in their slots: once more from the words, by the offsets inside the tile that the
    // first pass left in the table
    bool any_redo = false;
    for (uint32_t l = 0; l < kGroup; ++l) {
      if (!(cnt[l] & kRedo)) continue;   // uniform: the counts are the same for every thread
      any_redo = true;
      const uint32_t r0 = (t0 + l) << a.tile_shift;
      const uint32_t nb = P.n_chunks - r0 < G.tile_chunks ? P.n_chunks - r0 : G.tile_chunks;
      typename F::Regs w;
      for (uint32_t k = wave; k < nb; k += NW) {
        const uint64_t cbase = (uint64_t)(r0 + k) * kChunk;
        const uint32_t base = first + tp[l] + tab[r0 + k];
        const uint8_t* cptr = chunk_at<F::ES>(P.w, cbase, P.w.table ? page_of_chunk(P.w, r0 + k) : 0u);
        if (F::full(P, cbase)) {
          F::template load<true>(P, cptr, cbase, lane, w);
          F::template process<true, false>(P, lut, park, cbase, lane, w, base, fin);
        } else {
          F::template load<false>(P, cptr, cbase, lane, w);
          F::template process<false, false>(P, lut, park, cbase, lane, w, base, fin);
        }
      }
    }
    if (any_redo) __syncthreads();   // the table has been read by whoever needed its entries as offsets inside a tile
    // the table entries: what lies before the tile added to the offsets inside the tile
    if ((uint32_t)tid < entries) tab[c0 + tid] = my_entry[q] + first + tp[(uint32_t)tid >> a.tile_shift];
    for (uint32_t e = tid + kTileThreads; e < entries; e += kTileThreads) tab[c0 + e] += first + tp[e >> a.tile_shift];
    // the records fetched ahead
    const uint32_t cl = cnt[sl];
    if (!(cl & kRedo) && sj < cl) fin.put(first + tp[sl] + sj, rec_ahead[q] & 0xffffu, rec_ahead[q] >> 16);
    if (!(cl & kRedo) && sj + kSlotAhead < cl) fin.put(first + tp[sl] + sj + kSlotAhead, rec_ahead2[q] & 0xffffu, rec_ahead2[q] >> 16);
    // The rest of the slots of tiles with more records than that: rank r of the group belongs to the last tile that
    // starts at or before r.  Two records per thread are on their way at a time.
    const uint32_t group_total = tp[kGroup];
    if (s_more[q]) {   // a tile of the group has more records than were fetched ahead
      auto locate = [&](uint32_t r, uint32_t& l, uint32_t& j) -> bool {
        l = 0;
#pragma unroll
        for (uint32_t step = kGroup / 2; step; step >>= 1)
          if (tp[l + step] <= r) l += step;
        j = r - tp[l];
        return r < group_total && j >= 2 * kSlotAhead && !(cnt[l] & kRedo);
      };
      for (uint32_t r = tid; r < group_total; r += 2 * kTileThreads) {
        uint32_t l0, j0, l1, j1, rec0 = 0, rec1 = 0;
        const bool take0 = locate(r, l0, j0), take1 = locate(r + kTileThreads, l1, j1);
        if (take0) rec0 = G.slots[(uint64_t)(t0 + l0) * a.slot_cap + j0];
        if (take1) rec1 = G.slots[(uint64_t)(t0 + l1) * a.slot_cap + j1];
        if (take0) fin.put(first + r, rec0 & 0xffffu, rec0 >> 16);
        if (take1) fin.put(first + r + kTileThreads, rec1 & 0xffffu, rec1 >> 16);
      }
    }
    first += group_total;
  }
  if (g0 == 0 && wave == 0) compress_write_trailer(P, a.dec_of(item), a.sizes + item, M, 0u, lane);
}

#endif  // SPLITZIP_COMPRESS_HPP
