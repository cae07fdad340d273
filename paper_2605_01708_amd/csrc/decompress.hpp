// SplitZip for MI355X: the decompress kernels (dense decode of both formats, scatter correction in registers, single-tensor and batch kernels).
// Part of the single translation unit splitzip.hip (included inside its anonymous namespace).
#ifndef SPLITZIP_DECOMPRESS_HPP
#define SPLITZIP_DECOMPRESS_HPP

// ---------------------------------------------------------------------------
// decompress
// ---------------------------------------------------------------------------

struct DecompressArgs {
  const uint8_t* comp;
  Words w;                 // where the decoded words go
  uint64_t n, comp_bytes;
  splitzip_sizes* sizes;   // nullable
  uint64_t off_tab, off_sm, off_code, off_pos, sm_bytes, code_bytes;
  uint32_t n_chunks, n_tiles, cpw, dtype;
  uint32_t reg_patch_max;  // chunks with at most this many escapes are corrected in registers, the others in an LDS tile
  const uint8_t* d_dec;    // nullable: the 16 decode entries in device memory, used instead of dec
  uint8_t dec[16];
};

__device__ inline void flag_bad(const DecompressArgs& a) {
  if (a.sizes) atomicOr(&a.sizes->status, SPLITZIP_STATUS_BAD_STREAM);
}

// header checks: one thread of workgroup 0
// dec: the 16 decode entries the caller's codebook has, four to a word
__device__ void decompress_check_header(const DecompressArgs& a, const u32x4& dec, uint32_t M) {
  const uint32_t* h = reinterpret_cast<const uint32_t*>(a.comp);
  const uint64_t n = h[4] | ((uint64_t)h[5] << 32), m = h[6] | ((uint64_t)h[7] << 32);
  const uint64_t total = h[8] | ((uint64_t)h[9] << 32);
  bool ok = h[0] == 0x31505a53u && h[1] == (1u | (a.dtype << 16) | (4u << 24)) && h[2] == kChunk &&
            h[3] == 0 && n == a.n && m == M && total == a.off_pos + a256(2 * m) + m &&
            total <= a.comp_bytes && h[14] == 0 && h[15] == 0;
  ok = ok && h[10] == dec.x && h[11] == dec.y && h[12] == dec.z && h[13] == dec.w;   // the 16 entries, four to a word
  if (!ok) flag_bad(a);
  if (a.sizes) {
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = m;
  }
}

// BF16: the plane words of one chunk as a wave holds them, two half-chunks of 8 elements per lane each
struct PlanesBf16 {
  u32x2 sm[2];
  uint32_t cd[2];
};
template <bool FULL>
__device__ inline void load_planes_bf16(const DecompressArgs& a, uint64_t cbase, int lane, PlanesBf16& in) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    in.sm[h] = u32x2{0u, 0u};
    in.cd[h] = 0;
    if (FULL || g0 < a256(a.sm_bytes)) in.sm[h] = ld_stream(reinterpret_cast<const u32x2*>(a.comp + a.off_sm + g0));
    if (FULL || (g0 >> 1) < a256(a.code_bytes))
      in.cd[h] = ld_stream(reinterpret_cast<const uint32_t*>(a.comp + a.off_code + (g0 >> 1)));
  }
}
// dense decode into registers: o[4 h + d] holds elements 2 d and 2 d + 1 of the lane's group in half h
__device__ inline void decode_chunk_bf16(const PlanesBf16& in, const uint32_t* tbl, uint32_t (&o)[8]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t smw[2] = {in.sm[h].x, in.sm[h].y};
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      // code byte b -> both exponents already in place (bits 7..14 and 23..30)
      const uint32_t cb = (in.cd[h] >> (8 * b)) & 0xffu;
      // [a0, a0, a1, a1], then keep mantissa in the low and sign in the high byte of each half-word (eq. (2))
      const uint32_t p = byte_perm(0u, smw[b >> 1], (b & 1) ? 0x03030202u : 0x01010000u);
      o[4 * h + b] = (p & 0x807f807fu) | tbl[cb];
    }
  }
}

template <bool FULL>
__device__ inline void store_chunk_bf16(const DecompressArgs& a, uint8_t* cptr, uint64_t cbase, int lane, const uint32_t (&o)[8]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL || nvalid == 8) {
      st_stream(reinterpret_cast<u32x4*>(cptr) + (uint32_t)(h * 64 + lane), u32x4{o[4 * h], o[4 * h + 1], o[4 * h + 2], o[4 * h + 3]});
    } else {
      uint16_t* q = reinterpret_cast<uint16_t*>(cptr + 2 * (g0 - cbase));
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if ((uint32_t)(2 * d) < nvalid) q[2 * d] = (uint16_t)o[4 * h + d];
        if ((uint32_t)(2 * d + 1) < nvalid) q[2 * d + 1] = (uint16_t)(o[4 * h + d] >> 16);
      }
    }
  }
}

// E5M2: the plane words of one chunk as a wave holds them, 16 elements per lane.  Lanes 2p and 2p+1 share 12
// bytes of the 3-bit plane: the even lane loads bytes 0..7 of them, the odd lane bytes 4..11 -- the same
// instruction for every lane (no branch, no register written from two places), the overlap costs nothing.
struct PlanesE5m2 {
  u32x2 sm, cd;
};
template <bool FULL>
__device__ inline void load_planes_e5m2(const DecompressArgs& a, uint64_t cbase, int lane, PlanesE5m2& in) {
  const uint64_t g0 = cbase + lane * 16;
  const uint64_t off = (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12 + ((lane & 1) ? 4u : 0u);
  const uint8_t* src = a.comp + a.off_sm + off;
  const uint64_t sm_end = a256(a.sm_bytes);   // a multiple of 256; off is a multiple of 4
  in.sm = u32x2{0u, 0u};
  in.cd = u32x2{0u, 0u};
  if (FULL || off + 8 <= sm_end) in.sm = ld_stream(reinterpret_cast<const u32x2*>(src));
  else if (off + 4 <= sm_end) in.sm.x = ld_stream(reinterpret_cast<const uint32_t*>(src));
  if (FULL || (g0 >> 1) < a256(a.code_bytes)) in.cd = ld_stream(reinterpret_cast<const u32x2*>(a.comp + a.off_code + (g0 >> 1)));
}
// dense decode into registers: o[d] holds elements 4 d .. 4 d + 3
__device__ inline void decode_chunk_e5m2(const PlanesE5m2& in, const uint32_t* tbl, int lane, uint32_t (&o)[4]) {
  // the lane's 48 plane bits: the even lane's start at its first byte, the odd lane's two bytes further on
  const uint32_t lo = (lane & 1) ? (in.sm.x >> 16) | (in.sm.y << 16) : in.sm.x;
  const uint32_t hi = (lane & 1) ? in.sm.y >> 16 : in.sm.y & 0xffffu;
  const uint32_t r[4] = {lo & 0xfffu, (lo >> 12) & 0xfffu, (lo >> 24) | ((hi & 0xfu) << 8), (hi >> 4) & 0xfffu};
  const uint32_t cdw[2] = {in.cd.x, in.cd.y};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    // two code bytes -> four exponents already in place (bits 2..6 of each byte)
    const uint32_t c01 = (cdw[d >> 1] >> (16 * (d & 1))) & 0xffu, c23 = (cdw[d >> 1] >> (16 * (d & 1) + 8)) & 0xffu;
    o[d] = unpack3_e5m2(r[d]) | tbl[c01] | (tbl[c23] << 16);
  }
}

template <bool FULL>
__device__ inline void store_chunk_e5m2(const DecompressArgs& a, uint8_t* cptr, uint64_t cbase, int lane, const uint32_t (&o)[4]) {
  const uint64_t g0 = cbase + lane * 16;
  uint32_t nvalid = 16;
  if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 16 ? a.n - g0 : 16);
  if (FULL || nvalid == 16) {
    st_stream(reinterpret_cast<u32x4*>(cptr) + (uint32_t)lane, u32x4{o[0], o[1], o[2], o[3]});
  } else {
    uint8_t* q = cptr + (g0 - cbase);
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if ((uint32_t)j < nvalid) q[j] = (uint8_t)(o[j >> 2] >> (8 * (j & 3)));
  }
}

// in-register scatter correction: dword r of the owning lane gets (o & ~mask) | bits; r is
// wave-uniform, so the choice of the register is a scalar branch
template <int R>
__device__ inline void patch_regs(uint32_t (&o)[R], uint32_t r, bool mine, uint32_t mask, uint32_t bits) {
#pragma unroll
  for (int q = 0; q < R; ++q)
    if (r == (uint32_t)q && mine) o[q] = (o[q] & ~mask) | bits;
}

// the two formats as seen by the decompress kernel
struct DBf16 {
  static constexpr int ES = 2;   // bytes per word
  static constexpr int kPlanesAhead = 2;   // chunks whose planes are on their way while one is decoded
  struct Out { uint32_t o[8]; };
  // table entry for a code byte: both exponents in place for one dword of output
  __device__ static inline uint32_t table(int cb, const u32x4& dec) { return (dec16_at(dec, cb & 15) << 7) | (dec16_at(dec, cb >> 4) << 23); }
  __device__ static inline uint32_t table(int cb, const uint8_t* dec) { return ((uint32_t)dec[cb & 15] << 7) | ((uint32_t)dec[cb >> 4] << 23); }
  // The decode table is built from entries held in scalar registers: it is ready, and the barrier behind it
  // passed, while the table entries and planes are still on their way (a 64 MiB tensor: 23.1 us against 23.8 us
  // with the entries read by vector loads, which return behind everything asked for before them).
  static constexpr bool kScalarDec = true;
  __device__ static inline bool full(const DecompressArgs& a, uint64_t cbase) { return cbase + kChunk <= a.n; }
  typedef PlanesBf16 In;
  template <bool FULL>
  __device__ static inline void load(const DecompressArgs& a, uint64_t cbase, int lane, In& in) { load_planes_bf16<FULL>(a, cbase, lane, in); }
  __device__ static inline void decode(const In& in, const uint32_t* tbl, int lane, Out& r) { decode_chunk_bf16(in, tbl, r.o); }
  __device__ static inline void arrived(In& in) {
    asm volatile("" : "+v"(in.sm[0].x), "+v"(in.sm[0].y), "+v"(in.sm[1].x), "+v"(in.sm[1].y), "+v"(in.cd[0]), "+v"(in.cd[1]));
  }
  template <bool FULL>
  __device__ static inline void store(const DecompressArgs& a, uint8_t* cptr, uint64_t cbase, int lane, const Out& r) { store_chunk_bf16<FULL>(a, cptr, cbase, lane, r.o); }
  // the scatter correction of the element at chunk position pos (wave-uniform), in the registers of the lane that holds it
  __device__ static inline bool patch_reg(Out& r, int lane, uint32_t pos, uint32_t val) {
    const uint32_t q = pos & 511u, e = q & 7u, sh = 16u * (e & 1u);
    patch_regs<8>(r.o, 4u * (pos >> 9) + (e >> 1), (uint32_t)lane == (q >> 3), 0x7f80u << sh, val << (7u + sh));
    return true;
  }
  // The chunk as an LDS tile in element order (2 KB), for chunks with many escapes: registers -> tile, the
  // correction of one element by one lane, tile -> registers.
  static constexpr uint32_t kTileDwords = 512;
  __device__ static inline void to_tile(const Out& r, uint32_t* tile, int lane) {
#pragma unroll
    for (int h = 0; h < 2; ++h) reinterpret_cast<u32x4*>(tile)[h * 64 + lane] = u32x4{r.o[4 * h], r.o[4 * h + 1], r.o[4 * h + 2], r.o[4 * h + 3]};
  }
  __device__ static inline void from_tile(Out& r, const uint32_t* tile, int lane) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u32x4 v = reinterpret_cast<const u32x4*>(tile)[h * 64 + lane];
      r.o[4 * h] = v.x; r.o[4 * h + 1] = v.y; r.o[4 * h + 2] = v.z; r.o[4 * h + 3] = v.w;
    }
  }
  __device__ static inline bool patch_tile(uint32_t* tile, uint32_t pos, uint32_t val) {
    uint16_t* t = reinterpret_cast<uint16_t*>(tile) + pos;
    *t = (uint16_t)((*t & ~0x7f80u) | (val << 7));
    return true;
  }
};
struct DE5m2 {
  static constexpr int ES = 1;
  static constexpr int kPlanesAhead = 1;
  struct Out { uint32_t o[4]; };
  __device__ static inline uint32_t table(int cb, const u32x4& dec) { return (dec16_at(dec, cb & 15) << 2) | (dec16_at(dec, cb >> 4) << 10); }
  __device__ static inline uint32_t table(int cb, const uint8_t* dec) { return ((uint32_t)dec[cb & 15] << 2) | ((uint32_t)dec[cb >> 4] << 10); }
  // E5M2 reads the entries with vector loads (a 32 MiB tensor: 14.7 us; 16.1 us with the entries in scalar registers)
  static constexpr bool kScalarDec = false;
  __device__ static inline bool full(const DecompressArgs& a, uint64_t cbase) { return cbase + kChunk < a.n; }
  typedef PlanesE5m2 In;
  template <bool FULL>
  __device__ static inline void load(const DecompressArgs& a, uint64_t cbase, int lane, In& in) { load_planes_e5m2<FULL>(a, cbase, lane, in); }
  __device__ static inline void decode(const In& in, const uint32_t* tbl, int lane, Out& r) { decode_chunk_e5m2(in, tbl, lane, r.o); }
  __device__ static inline void arrived(In& in) { asm volatile("" : "+v"(in.sm.x), "+v"(in.sm.y), "+v"(in.cd.x), "+v"(in.cd.y)); }
  template <bool FULL>
  __device__ static inline void store(const DecompressArgs& a, uint8_t* cptr, uint64_t cbase, int lane, const Out& r) { store_chunk_e5m2<FULL>(a, cptr, cbase, lane, r.o); }
  __device__ static inline bool patch_reg(Out& r, int lane, uint32_t pos, uint32_t val) {
    if (val > 31u) return false;
    const uint32_t e = pos & 15u, sh = 8u * (e & 3u);
    patch_regs<4>(r.o, e >> 2, (uint32_t)lane == (pos >> 4), 0x7cu << sh, val << (2u + sh));
    return true;
  }
  static constexpr uint32_t kTileDwords = 256;
  __device__ static inline void to_tile(const Out& r, uint32_t* tile, int lane) {
    reinterpret_cast<u32x4*>(tile)[lane] = u32x4{r.o[0], r.o[1], r.o[2], r.o[3]};
  }
  __device__ static inline void from_tile(Out& r, const uint32_t* tile, int lane) {
    const u32x4 v = reinterpret_cast<const u32x4*>(tile)[lane];
    r.o[0] = v.x; r.o[1] = v.y; r.o[2] = v.z; r.o[3] = v.w;
  }
  __device__ static inline bool patch_tile(uint32_t* tile, uint32_t pos, uint32_t val) {
    if (val > 31u) return false;
    uint8_t* t = reinterpret_cast<uint8_t*>(tile) + pos;
    *t = (uint8_t)((*t & ~0x7cu) | (val << 2));
    return true;
  }
};

constexpr uint32_t kRegPatchDefault = 4;   // escapes of a chunk that are still applied in registers

// a wave's LDS accesses are carried out in program order; this keeps the compiler from reordering accesses it
// takes for unrelated because they go through different types
__device__ inline void lds_settle() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// one workgroup: tile `tile` of the tensor described by a (4 waves x cpw chunks); lds_chunk: kTileDwords per wave
template <typename F>
__device__ inline void decompress_tile(const DecompressArgs& a, const u32x4& dec, const uint8_t* dec_ptr, uint32_t tile, uint32_t* tbl,
                                       uint32_t* lds_chunk) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t* tab = reinterpret_cast<const uint32_t*>(a.comp + a.off_tab);
  const uint32_t cpw = a.cpw;
  const uint32_t wave_chunk0 = (tile * kWaves + wave) * cpw;
  // first of all the loads everything else waits for: this wave's slice of the offset table (lane c
  // <-> its chunk c, one entry more for the end) and M as the table states it
  const uint32_t my_tab = (uint32_t)lane <= cpw && wave_chunk0 + lane <= a.n_chunks ? tab[wave_chunk0 + lane] : 0u;
  uint32_t M = tab[a.n_chunks];
  // paged tensor: the pool pages of the wave's chunks, lane c <-> its chunk c
  uint32_t my_pages = 0;
  if (a.w.table && (uint32_t)lane < cpw && wave_chunk0 + lane < a.n_chunks) my_pages = page_of_chunk(a.w, wave_chunk0 + lane);

  // The wave's chunks; only the tensor's last chunk can be ragged, and it is the last of its wave.
  const uint32_t mine = wave_chunk0 < a.n_chunks ? (a.n_chunks - wave_chunk0 < cpw ? a.n_chunks - wave_chunk0 : cpw) : 0u;
  const bool last_ragged = mine > 0 && !F::full(a, (uint64_t)(wave_chunk0 + mine - 1) * kChunk);
  const uint32_t fast = mine - (last_ragged ? 1u : 0u);
  // everything chunk c needs from memory: its planes and the first 64 of its records, one lane each
  struct Fetched {
    typename F::In in;
    uint32_t pos, val;
  };
  Fetched cur, nxt;
  // The planes of the wave's first chunk depend on nothing that is loaded: they are asked for right behind the
  // table entries, and the decode table is built while both are on their way (the barrier below is for LDS only).
  if (fast > 0) F::template load<true>(a, (uint64_t)wave_chunk0 * kChunk, lane, cur.in);
  if (F::kPlanesAhead == 2 && fast > 1) F::template load<true>(a, (uint64_t)(wave_chunk0 + 1) * kChunk, lane, nxt.in);   // and those of its second
  tbl[tid] = F::kScalarDec ? F::table(tid, dec) : F::table(tid, dec_ptr);

  // escapes are only trusted if their sections lie inside the stream
  const uint64_t off_val = a.off_pos + a256(2ull * M);
  const bool esc_ok = M <= a.n && off_val + M <= a.comp_bytes;
  if (tile == 0 && tid == 0) {
    u32x4 d = dec;
    if (!F::kScalarDec) {
      const uint32_t* dp = reinterpret_cast<const uint32_t*>(dec_ptr);   // 4-byte aligned wherever the entries lie
      d = u32x4{dp[0], dp[1], dp[2], dp[3]};
    }
    decompress_check_header(a, d, M);
    if (!esc_ok) flag_bad(a);
  }
  if (!esc_ok) M = 0;
  const uint16_t* pos_arr = reinterpret_cast<const uint16_t*>(a.comp + a.off_pos);
  const uint8_t* val_arr = a.comp + off_val;
  lds_barrier();

  // escape records of the wave's c-th chunk: first record and count, from the offset table (0 records if the entries are inconsistent)
  auto records = [&](uint32_t c, uint32_t& lo, bool& valid) -> uint32_t {
    const uint64_t cbase = (uint64_t)(wave_chunk0 + c) * kChunk;
    const uint32_t hi = __builtin_amdgcn_readlane(my_tab, c + 1);
    lo = __builtin_amdgcn_readlane(my_tab, c);
    const uint32_t clen = (uint32_t)(a.n - cbase < kChunk ? a.n - cbase : kChunk);
    valid = hi >= lo && hi - lo <= clen && hi <= M;
    return valid ? hi - lo : 0u;
  };
  auto fetch_records = [&](uint32_t c, Fetched& f) {
    uint32_t lo;
    bool valid;
    const uint32_t cnt = records(c, lo, valid);
    f.pos = 0; f.val = 0;
    if ((uint32_t)lane < cnt) {
      f.pos = pos_arr[lo + lane];
      f.val = val_arr[lo + lane];
    }
  };
  auto fetch = [&](uint32_t c, Fetched& f, auto complete) {
    fetch_records(c, f);
    F::template load<decltype(complete)::value>(a, (uint64_t)(wave_chunk0 + c) * kChunk, lane, f.in);
  };
  // A few escapes, the usual case, are applied to the decoded words in registers, one after the other; more
  // of them are applied in parallel, one lane each, to the chunk laid out in LDS.  Either way every word is
  // stored once.
  auto chunk = [&](uint32_t c, const Fetched& f, auto complete) {
    constexpr bool FULL = decltype(complete)::value;
    const uint64_t cbase = (uint64_t)(wave_chunk0 + c) * kChunk;
    uint32_t lo;
    bool esc_valid;
    const uint32_t cnt = records(c, lo, esc_valid);
    const uint32_t clen = (uint32_t)(a.n - cbase < kChunk ? a.n - cbase : kChunk);
    if (!esc_valid && lane == 0) flag_bad(a);
    typename F::Out r;
    F::decode(f.in, tbl, lane, r);
    if (cnt > 0 && cnt <= a.reg_patch_max) {
      uint32_t floor = 0;   // a chunk's positions ascend: each must lie above the one before it
      for (uint32_t j = 0; j < cnt; ++j) {
        const uint32_t p = __builtin_amdgcn_readlane(f.pos, j), v = __builtin_amdgcn_readlane(f.val, j);
        if (p >= clen || p < floor || !F::patch_reg(r, lane, p, v)) {
          if (lane == 0) flag_bad(a);
        }
        floor = p + 1;
      }
    }
    if (cnt > a.reg_patch_max) {
      uint32_t* t = lds_chunk + (uint32_t)wave * F::kTileDwords;
      F::to_tile(r, t, lane);
      lds_settle();
      for (uint32_t j = lane; j < cnt; j += 64) {
        uint32_t p = f.pos, v = f.val;
        if (j >= 64) {
          p = pos_arr[lo + j];
          v = val_arr[lo + j];
        }
        // a chunk's positions ascend: the record before this one (the lane below holds it, or memory does)
        uint32_t before = (uint32_t)__shfl_up((int)p, 1);
        if (lane == 0 && j > 0) before = pos_arr[lo + j - 1];
        if (p >= clen || (j > 0 && p <= before) || !F::patch_tile(t, p, v)) flag_bad(a);
      }
      lds_settle();
      F::from_tile(r, t, lane);
      lds_settle();   // the tile is written again for the wave's next chunk
    }
    uint8_t* cptr = chunk_at<F::ES>(a.w, cbase, __builtin_amdgcn_readlane(my_pages, c));
    F::template store<FULL>(a, cptr, cbase, lane, r);
  };
  // BF16: planes are asked for two chunks ahead and records one chunk ahead (they need the table entries, the
  // planes need nothing); E5M2, whose kernel is short of instruction slots rather than of bytes in flight: both
  // one chunk ahead (two ahead: 0.65 instead of 0.70 of the HBM peak).  The first chunk is awaited before the loop, and the ragged chunk stays out of it altogether,
  // its loads included: the compiler's wait at the bottom of an iteration then covers the next chunk's loads but
  // not the store issued after them, and no wait stands in front of the loads.
  if (fast > 0) {
    fetch_records(0, cur);
    F::arrived(cur.in);
    asm volatile("" : "+v"(cur.pos), "+v"(cur.val));
  }
  for (uint32_t c = 0; c < fast; ++c) {
    if (F::kPlanesAhead == 2) {
      if (c + 1 < fast) fetch_records(c + 1, nxt);
    } else {
      if (c + 1 < fast) fetch(c + 1, nxt, std::true_type{});
    }
    chunk(c, cur, std::true_type{});
    cur = nxt;
    if (F::kPlanesAhead == 2 && c + 2 < fast) F::template load<true>(a, (uint64_t)(wave_chunk0 + c + 2) * kChunk, lane, nxt.in);
  }
  if (last_ragged) {
    fetch(mine - 1, cur, std::false_type{});
    chunk(mine - 1, cur, std::false_type{});
  }
}

template <typename F>
__global__ __launch_bounds__(kThreads) void decompress_kernel(const DecompressArgs a) {
  __shared__ uint32_t tbl[256];
  __shared__ __attribute__((aligned(16))) uint32_t lds_chunk[kWaves * F::kTileDwords];
  u32x4 dec16 = u32x4{0u, 0u, 0u, 0u};
  if (F::kScalarDec) dec16 = a.d_dec ? load_dec16(a.d_dec) : dec16_from(a.dec);
  decompress_tile<F>(a, dec16, a.d_dec ? a.d_dec : a.dec, blockIdx.x, tbl, lds_chunk);
}

// several streams in one launch: blockIdx.y picks the stream, blockIdx.x the tile
struct DBatchItem {
  const uint8_t* comp;
  uint8_t* out;
  uint64_t n, comp_bytes;
};
struct DecompressBatchArgs {
  DBatchItem item[kBatchMax];
  splitzip_sizes* sizes;   // nullable; one record, status bits sticky
  uint32_t cpw, dtype, reg_patch_max;
  Words paging;            // as in CompressBatchArgs
  uint8_t dec[kBatchMax][16];   // every stream's codebook
  const splitzip_codebook* d_cbs;   // nullable: n_items codebooks in device memory, used instead of dec
  uint32_t own_dec;        // 1: every stream is decoded with the 16 decode entries of its own header
};

template <typename F>
__global__ __launch_bounds__(kThreads) void decompress_batch_kernel(const DecompressBatchArgs b) {
  __shared__ uint32_t tbl[256];
  __shared__ __attribute__((aligned(16))) uint32_t lds_chunk[kWaves * F::kTileDwords];
  const DBatchItem it = b.item[blockIdx.y];
  const Layout L = make_layout(it.n, (int)b.dtype);
  const uint32_t n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * b.cpw - 1) / (kWaves * b.cpw));
  if (blockIdx.x >= (n_tiles ? n_tiles : 1u)) return;
  DecompressArgs a;
  a.comp = it.comp;
  a.w = item_words(b.paging, it.out);
  a.n = it.n;
  a.comp_bytes = it.comp_bytes;
  a.sizes = b.sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = n_tiles;
  a.cpw = b.cpw;
  a.dtype = b.dtype;
  a.reg_patch_max = b.reg_patch_max;
  u32x4 dec16 = u32x4{0u, 0u, 0u, 0u};
  if (F::kScalarDec) dec16 = b.own_dec ? load_dec16(it.comp + kHeaderDecOffset) : b.d_cbs ? load_dec16(b.d_cbs[blockIdx.y].dec) : dec16_from(b.dec[blockIdx.y]);
  decompress_tile<F>(a, dec16, b.own_dec ? it.comp + kHeaderDecOffset : b.d_cbs ? b.d_cbs[blockIdx.y].dec : b.dec[blockIdx.y], blockIdx.x, tbl, lds_chunk);   // a.dec stays unset: the table comes from the kernel arguments
}

#endif  // SPLITZIP_DECOMPRESS_HPP
