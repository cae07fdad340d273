// SplitZip codec for MI355X (gfx950): HIP kernels and the C ABI of include/splitzip.h.
//
// One compress call is ONE kernel launch (tensors of up to 64 Mi elements or
// so; larger ones take one launch per segment and a small finishing launch).
// The dense transform (paper section 3.2 eq. (1), encode table, nibble pack,
// sign+mantissa plane) is fused with escape detection, per-chunk counting and
// the position-ordered compaction of the escape stream (appendix A fuses only
// the counting).  The input is read exactly once: escapes are staged in LDS
// while their words are in registers.  The launch is a persistent grid that
// fits the chip; every workgroup owns one contiguous range of chunks, and the
// one cross-workgroup step is a flat exchange of the per-range escape counts
// through one word per workgroup: each workgroup publishes its count, reads
// everybody's, and then knows both its own offset (counts of the ranges before
// it) and M, so positions, values and the offset table go straight to their
// final place.  No atomic read-modify-write is used: on this chip every
// device-wide atomic on one address costs about 12 ns, serialised.
// One decompress call is ONE kernel launch as well: nibble unpack, decode
// table, eq. (2), and the sparse overwrite done by the wave that owns the
// chunk once its own dense stores have completed.
//
// Work decomposition (wavefront = 64 lanes):
//   chunk = 1024 elements (the escape-position granule), owned by one wave and
//           processed as two half-chunks of 512 elements; in a half-chunk lane
//           l owns elements [8 l, 8 l + 8): every global access of a wave is
//           one fully coalesced run (16, 8 or 4 bytes per lane).
//   compress: the chunks of a workgroup's range are dealt round-robin to its
//           waves, so a workgroup reads one moving window.
//   decompress: one workgroup per tile of 4 waves x cpw chunks.
// All plane traffic uses non-temporal loads / stores: nothing is re-used.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "splitzip.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kChunk = 1024;
constexpr uint32_t kHalf = 512;
constexpr uint32_t kHeaderBytes = 64;
constexpr int kThreads = 256;                             // decompress / helper kernels
constexpr int kWaves = kThreads / 64;
constexpr uint32_t kMaxCpw = 16;                          // decompress: chunks per wave per tile, at most
constexpr uint32_t kMaxRange = 256;                       // compress: chunks per workgroup per launch, at most
constexpr uint32_t kMaxWorkgroups = 4096;                 // compress: words of exchange state in the workspace
constexpr uint32_t kWsTableBytes = 8 * kMaxWorkgroups;
constexpr uint32_t kStageCap = 512;                       // escapes a wave can stage in LDS
constexpr uint32_t kWsHeaderBytes = 64;                   // epoch, running escape count, error flags
constexpr uint32_t kSegFirst = 1u, kSegLast = 2u;         // CompressArgs.flags
constexpr uint64_t kSpinTicks = 200000000ull;             // 2 s of the 100 MHz wall clock

__host__ __device__ inline uint64_t a256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

struct Layout {
  uint64_t n, n_chunks, sm_bytes, code_bytes;
  uint64_t off_tab, off_sm, off_code, off_pos;  // the value section starts at off_pos + a256(2M)
};

__host__ __device__ inline Layout make_layout(uint64_t n, int dtype) {
  Layout L;
  L.n = n;
  L.n_chunks = (n + kChunk - 1) / kChunk;
  L.sm_bytes = dtype == SPLITZIP_BF16 ? n : (3 * n + 7) / 8;
  L.code_bytes = (n + 1) / 2;
  L.off_tab = kHeaderBytes;
  L.off_sm = a256(L.off_tab + 4 * (L.n_chunks + 1));
  L.off_code = L.off_sm + a256(L.sm_bytes);
  L.off_pos = L.off_code + a256(L.code_bytes);
  return L;
}

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------

template <typename T>
__device__ inline T ld_stream(const T* p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ inline void st_stream(T* p, T v) { __builtin_nontemporal_store(v, p); }

// v_perm_b32: result byte i = byte sel[i] of the 8-byte pool {hi:4..7, lo:0..3}; 0x0c gives 0x00.
__device__ inline uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
  return __builtin_amdgcn_perm(hi, lo, sel);
}

// inclusive prefix sum over the 64 lanes with DPP moves: Kogge-Stone inside rows of 16 lanes,
// then the row totals are carried over with the two row-broadcast steps
__device__ inline uint32_t wave_incl_scan(uint32_t v) {
  v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
  return v;
}

__device__ inline uint32_t wave_last(uint32_t v) { return __builtin_amdgcn_readlane(v, 63); }

// agent-scope relaxed accesses: performed at the device-wide coherence point, no fences
template <typename T>
__device__ inline void st_agent(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ inline T ld_agent(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// ---------------------------------------------------------------------------
// compress
// ---------------------------------------------------------------------------

// what the dense pass and the trailer need to know of one tensor and its stream
struct Planes {
  const uint8_t* in;
  uint8_t* out;
  uint64_t n, capacity;
  uint64_t off_tab, off_sm, off_code, off_pos, sm_bytes, code_bytes;
  uint32_t n_chunks, dtype;
};

__host__ __device__ inline Planes make_planes(const void* in, void* out, uint64_t n, uint64_t capacity, int dtype) {
  const Layout L = make_layout(n, dtype);
  Planes p;
  p.in = static_cast<const uint8_t*>(in);
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
  uint8_t dec[16];
  uint16_t lut[256];     // exponent -> code | (non-member ? 0x100 : 0)   (the "marked" table of appendix A)
};

// where a chunk's escape records go: LDS staging (first pass) or their final place
struct LdsSink {
  uint16_t* pos;
  uint8_t* val;
  uint32_t tag;   // OR-ed into the position: which of the wave's chunks the record belongs to
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < kStageCap) {
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
__device__ inline void load_chunk_bf16(const Planes& a, uint64_t cbase, int lane, uint32_t (&w)[2][4]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;   // first element of this lane's group
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL) {
      // chunk pointer (wave-uniform) + a 32-bit lane offset: no 64-bit vector arithmetic
      const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(a.in + 2 * cbase) + (uint32_t)(h * 64 + lane));
      w[h][0] = v.x; w[h][1] = v.y; w[h][2] = v.z; w[h][3] = v.w;
    } else if (nvalid == 8) {
      const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(a.in + 2 * g0));
      w[h][0] = v.x; w[h][1] = v.y; w[h][2] = v.z; w[h][3] = v.w;
    } else {
      const uint16_t* p = reinterpret_cast<const uint16_t*>(a.in) + g0;
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
  const uint32_t u = (t | (t >> 5)) & 0x003f003fu;
  return (u | (u >> 10)) & 0xfffu;
}
// inverse: 12 bits -> the sign and mantissa bits of four bytes, exponent field zero
__device__ inline uint32_t unpack3_e5m2(uint32_t r) {
  const uint32_t u = (r | (r << 10)) & 0x003f003fu;
  const uint32_t t = (u | (u << 5)) & 0x07070707u;
  return ((t & 0x04040404u) << 5) | (t & 0x03030303u);
}

template <bool FULL>
__device__ inline void load_chunk_e5m2(const Planes& a, uint64_t cbase, int lane, uint32_t (&w)[4]) {
  const uint64_t g0 = cbase + lane * 16;
  uint32_t nvalid = 16;
  if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 16 ? a.n - g0 : 16);
  if (FULL) {
    const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(a.in + cbase) + (uint32_t)lane);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if (nvalid == 16) {
    const u32x4 v = ld_stream(reinterpret_cast<const u32x4*>(a.in + g0));
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else {
    const uint8_t* p = a.in + g0;
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
    const uint32_t e0 = (w[d] >> 2) & 31u, e1 = (w[d] >> 10) & 31u, e2 = (w[d] >> 18) & 31u, e3 = (w[d] >> 26) & 31u;
    // low byte: code pair; high byte: flag pair in the same nibble layout
    u[2 * d] = (uint32_t)lut[e0] + ((uint32_t)lut[e1] << 4);
    u[2 * d + 1] = (uint32_t)lut[e2] + ((uint32_t)lut[e3] << 4);
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
    const uint32_t lo_up = __builtin_amdgcn_update_dpp(0u, lo, 0xF5, 0xf, 0xf, false);   // quad_perm [1,1,3,3]: the odd neighbour's lo
    const uint64_t sm_off = (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12;
    uint8_t* sm_dst = a.out + a.off_sm + (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12;   // uniform pointer + lane offset
    uint32_t d0, d1;
    if (lane & 1) {
      d0 = (lo >> 16) | (hi << 16);
      d1 = 0;
    } else {
      d0 = lo;
      d1 = (hi & 0xffffu) | (lo_up << 16);
    }
    if (FULL) {
      if (lane & 1) st_stream(reinterpret_cast<uint32_t*>(sm_dst + 8), d0);
      else st_stream(reinterpret_cast<u32x2*>(sm_dst), u32x2{d0, d1});
      st_stream(reinterpret_cast<u32x2*>(a.out + a.off_code + (cbase >> 1)) + (uint32_t)lane, u32x2{code[0], code[1]});
    } else {
      // dword by dword up to the padded end of each plane; the pad can reach 128 bytes past the
      // chunk's own 384 plane bytes
      const uint64_t sm_end = a256(a.sm_bytes);
      if (lane & 1) {
        if (sm_off + 8 < sm_end) *reinterpret_cast<uint32_t*>(sm_dst + 8) = d0;
      } else {
        if (sm_off < sm_end) *reinterpret_cast<uint32_t*>(sm_dst) = d0;
        if (sm_off + 4 < sm_end) *reinterpret_cast<uint32_t*>(sm_dst + 4) = d1;
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
  struct Regs { uint32_t w[2][4]; };
  // a chunk goes the fast way if it is complete (then nothing of a pad is its business: N is a multiple of 1024 there)
  __device__ static inline bool full(const Planes& a, uint64_t cbase) { return cbase + kChunk <= a.n; }
  template <bool FULL>
  __device__ static inline void load(const Planes& a, uint64_t cbase, int lane, Regs& r) { load_chunk_bf16<FULL>(a, cbase, lane, r.w); }
  template <bool FULL, bool STORE, typename Sink>
  __device__ static inline uint32_t process(const Planes& a, const uint16_t* lut, uint32_t* park, uint64_t cbase,
                                            int lane, const Regs& r, uint32_t base, const Sink& sink) {
    return process_chunk_bf16<FULL, STORE>(a, lut, park, cbase, lane, r.w, base, sink);
  }
};
struct E5m2 {
  struct Regs { uint32_t w[4]; };
  // the tensor's last chunk always goes the careful way: 384 plane bytes per chunk leave a pad behind an odd chunk count
  __device__ static inline bool full(const Planes& a, uint64_t cbase) { return cbase + kChunk < a.n; }
  template <bool FULL>
  __device__ static inline void load(const Planes& a, uint64_t cbase, int lane, Regs& r) { load_chunk_e5m2<FULL>(a, cbase, lane, r.w); }
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
  uint16_t* stage_pk;    // this wave's kStageCap entries
  uint8_t* stage_val;
  uint32_t* s_off;       // kMaxRange + 1
  uint16_t* s_wstart;    // kMaxRange
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

// dense pass of one wave over its chunks of the range; the next chunk's loads are issued before
// this chunk is worked on.  `mid` is called once, half way through (not at all by a wave without
// chunks).  Returns the wave's escape count.
template <int NW, typename F, typename Hook>
__device__ inline uint32_t dense_pass(const Planes& P, const uint16_t* lut, uint32_t* park, const RangeLds& L,
                                      uint32_t r0, uint32_t nb, int wave, int lane, Hook& mid) {
  uint32_t wave_count = 0;
  const uint32_t mid_it = nb > (uint32_t)wave ? ((nb - wave + NW - 1) / NW) / 2 : 0u;
  typename F::Regs w, nx;
  if ((uint32_t)wave < nb) {
    const uint64_t cbase = (uint64_t)(r0 + wave) * kChunk;
    if (F::full(P, cbase)) F::template load<true>(P, cbase, lane, w);
    else F::template load<false>(P, cbase, lane, w);
  }
  for (uint32_t k = wave, it = 0; k < nb; k += NW, ++it) {
    const uint64_t cbase = (uint64_t)(r0 + k) * kChunk;
    if (k + NW < nb) {
      const uint64_t nbase = cbase + (uint64_t)NW * kChunk;
      if (F::full(P, nbase)) F::template load<true>(P, nbase, lane, nx);
      else F::template load<false>(P, nbase, lane, nx);
    }
    if (it == mid_it) mid();
    const LdsSink lds{L.stage_pk, L.stage_val, it << 10};
    const uint32_t cnt = F::full(P, cbase) ? F::template process<true, true>(P, lut, park, cbase, lane, w, wave_count, lds)
                                           : F::template process<false, true>(P, lut, park, cbase, lane, w, wave_count, lds);
    if (lane == 0) {
      L.s_off[k] = cnt;
      L.s_wstart[k] = (uint16_t)(wave_count < 0xffffu ? wave_count : 0xffffu);
    }
    wave_count += cnt;
    w = nx;
  }
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
  if (wave_count <= kStageCap) {
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
      if (F::full(P, cbase)) {
        F::template load<true>(P, cbase, lane, w);
        F::template process<true, false>(P, lut, park, cbase, lane, w, r, g);
      } else {
        F::template load<false>(P, cbase, lane, w);
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
__global__ __launch_bounds__(T) void compress_kernel(const CompressArgs a) {
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
  const RangeLds L{stage_pk[wave], stage_val[wave], s_off, s_wstart};

  if (tid < 256) lut[tid] = a.lut[tid];
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
      if (single) compress_write_trailer(a.p, a.dec, a.sizes, base + al, err, lane);
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
constexpr uint32_t kBatchLuts = 2;     // codebooks per launch
constexpr uint32_t kRing = 4;          // exchange slots: a workgroup can be two tensors ahead of the slowest
constexpr uint32_t kRingWgs = 1024;    // words per slot

struct BatchItem {
  const uint8_t* in;
  uint8_t* out;
  uint64_t n, capacity;
};
struct CompressBatchArgs {
  BatchItem item[kBatchMax];
  uint8_t lut_of[kBatchMax];
  splitzip_sizes* sizes;     // n_items records
  uint32_t* ws_hdr;          // [0] epoch, [2] sticky error flags, [3] groups that are through
  uint64_t* state;           // per group kRing slots of group_wgs words: (epoch + item) << 32 | escapes in the range
  uint64_t spin_ticks;
  uint32_t n_items, dtype;
  uint32_t group_wgs;        // workgroups that share one tensor; the grid is n_groups * group_wgs
  uint32_t await_extra;      // error-path tests: words awaited beyond the group's
  uint8_t dec[kBatchLuts][16];
  uint16_t lut[kBatchLuts][256];
};

// wave 0, half way through a dense pass: the loads of the previous tensor's exchange words, so that
// their latency is hidden.  Up to 256 workgroups per group (four words per lane).
struct ExchangePrefetch {
  const uint64_t* slot;
  uint32_t wgs;
  int lane;
  bool enabled, issued;
  uint64_t v[4];
  __device__ inline void operator()() {
    if (!enabled) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t i = lane + 64 * j;
      v[j] = i < wgs ? ld_agent(&slot[i]) : 0ull;
    }
    issued = true;
  }
};

// The same persistent grid works through the tensors one after the other, and the exchange of
// tensor i is taken out of the critical path: a workgroup publishes its count for tensor i, then
// completes tensor i - 1 (whose counts every workgroup published a whole dense pass ago; the words
// are even fetched half way through the dense pass of tensor i, so the read costs nothing) and
// goes on to tensor i + 1.  Staging in LDS is double buffered.  What a single launch pays per
// tensor -- the wait for the slowest workgroup, the exchange, the write-out and the launch itself
// -- is paid once per batch here.  Small tensors are shared by a group of workgroups only; the
// groups work on different tensors at the same time (tensor i belongs to group i mod n_groups).
template <int T, typename F>
__global__ __launch_bounds__(T) void compress_batch_kernel(const CompressBatchArgs a) {
  constexpr int NW = T / 64;
  __shared__ uint16_t lut[kBatchLuts][256];
  __shared__ uint16_t stage_pk[2][NW][kStageCap];
  __shared__ uint8_t stage_val[2][NW][kStageCap];
  __shared__ uint32_t s_off[2][kMaxRange + 1];
  __shared__ uint16_t s_wstart[2][kMaxRange];
  __shared__ u32x4 s_park[T];
  __shared__ uint32_t s_red[16];
  __shared__ uint32_t s_misc[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t G = a.group_wgs, n_groups = gridDim.x / G;
  const uint32_t grp = blockIdx.x / G, b = blockIdx.x % G;
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);

  for (int i = tid; i < (int)(kBatchLuts * 256); i += T) lut[i >> 8][i & 255] = a.lut[i >> 8][i & 255];
  const uint32_t epoch = ld_agent(&a.ws_hdr[0]);
  const uint32_t err_before = b == 0 ? ld_agent(&a.ws_hdr[2]) : 0u;
  if (tid == 0) s_misc[3] = 0;   // set once an exchange was given up: later ones are not waited for
  __syncthreads();

  uint64_t* const ring = a.state + (uint64_t)grp * kRing * G;   // this group's slots
  Planes Pprev = make_planes(nullptr, nullptr, 0, 0, (int)a.dtype);
  uint32_t prev_count = 0, prev_r0 = 0, prev_nb = 0, prev_item = 0;
  // this group's tensors: grp, grp + n_groups, ...; seq counts them
  for (uint32_t seq = 0;; ++seq) {
    const uint32_t i = grp + seq * n_groups;
    const bool have = i < a.n_items;
    if (!have && seq == 0) break;   // a group without tensors
    const uint32_t set = seq & 1u;
    const RangeLds L{stage_pk[set][wave], stage_val[set][wave], s_off[set], s_wstart[set]};
    Planes P = Pprev;
    uint32_t r0 = 0, nb = 0, wave_count = 0;
    ExchangePrefetch pf;
    pf.slot = ring + ((seq + kRing - 1) % kRing) * G;
    pf.wgs = G;
    pf.lane = lane;
    pf.enabled = wave == 0 && seq > 0 && G <= 256 && a.await_extra == 0;
    pf.issued = false;
    if (have) {
      P = make_planes(a.item[i].in, a.item[i].out, a.item[i].n, a.item[i].capacity, (int)a.dtype);
      my_range(0, P.n_chunks, G, b, r0, nb);
      wave_count = dense_pass<NW, F>(P, lut[a.lut_of[i]], park, L, r0, nb, wave, lane, pf);
      if (lane == 0) s_red[wave] = wave_count;
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
          int ready = 1;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t q = lane + 64 * j;
            if (q < G) {
              if ((uint32_t)(pf.v[j] >> 32) != tag) ready = 0;
              al += (uint32_t)pf.v[j];
              lo += q < b ? (uint32_t)pf.v[j] : 0u;
            }
          }
          if (__ballot(ready) == ~0ull) {
            lo = wave_last(wave_incl_scan(lo));
            al = wave_last(wave_incl_scan(al));
            done = true;
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
          compress_write_trailer(Pprev, a.dec[a.lut_of[prev_item]], a.sizes + prev_item, al, err, lane);
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
    }
    __syncthreads();
    if (seq > 0 && s_misc[2] == 0) {
      const uint32_t pset = set ^ 1u;
      const RangeLds Lp{stage_pk[pset][wave], stage_val[pset][wave], s_off[pset], s_wstart[pset]};
      write_out<NW, F>(Pprev, lut[a.lut_of[prev_item]], park, Lp, prev_r0, prev_nb, prev_count, s_misc[0],
                       final_sink(Pprev, s_misc[1]), tid, wave, lane);
    }
    if (!have) break;
    __syncthreads();   // the previous tensor's LDS set is free again, s_misc may be rewritten
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
    compress_write_trailer(a.p, a.dec, a.sizes, M, err, threadIdx.x);
  }
}

// ---------------------------------------------------------------------------
// decompress
// ---------------------------------------------------------------------------

struct DecompressArgs {
  const uint8_t* comp;
  uint8_t* out;
  uint64_t n, comp_bytes;
  splitzip_sizes* sizes;   // nullable
  uint64_t off_tab, off_sm, off_code, off_pos, sm_bytes, code_bytes;
  uint32_t n_chunks, n_tiles, cpw, dtype;
  uint8_t dec[16];
};

__device__ inline void flag_bad(const DecompressArgs& a) {
  if (a.sizes) atomicOr(&a.sizes->status, SPLITZIP_STATUS_BAD_STREAM);
}

// header checks: one thread of workgroup 0
__device__ void decompress_check_header(const DecompressArgs& a, const uint8_t* dec, uint32_t M) {
  const uint32_t* h = reinterpret_cast<const uint32_t*>(a.comp);
  const uint64_t n = h[4] | ((uint64_t)h[5] << 32), m = h[6] | ((uint64_t)h[7] << 32);
  const uint64_t total = h[8] | ((uint64_t)h[9] << 32);
  bool ok = h[0] == 0x31505a53u && h[1] == (1u | (a.dtype << 16) | (4u << 24)) && h[2] == kChunk &&
            h[3] == 0 && n == a.n && m == M && total == a.off_pos + a256(2 * m) + m &&
            total <= a.comp_bytes && h[14] == 0 && h[15] == 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    ok = ok && h[10 + i] == (dec[4 * i] | (dec[4 * i + 1] << 8) | (dec[4 * i + 2] << 16) |
                             ((uint32_t)dec[4 * i + 3] << 24));
  if (!ok) flag_bad(a);
  if (a.sizes) {
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = m;
  }
}

// BF16 dense decode of one chunk by one wave into registers: two half-chunks, 8 elements per lane
// each; o[4 h + d] holds elements 2 d and 2 d + 1 of the lane's group in half h
template <bool FULL>
__device__ inline void decode_chunk_bf16(const DecompressArgs& a, const uint32_t* tbl, uint64_t cbase, int lane, uint32_t (&o)[8]) {
  u32x2 sm[2];
  uint32_t cd[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    sm[h] = u32x2{0u, 0u};
    cd[h] = 0;
    if (FULL || g0 < a256(a.sm_bytes)) sm[h] = ld_stream(reinterpret_cast<const u32x2*>(a.comp + a.off_sm + g0));
    if (FULL || (g0 >> 1) < a256(a.code_bytes))
      cd[h] = ld_stream(reinterpret_cast<const uint32_t*>(a.comp + a.off_code + (g0 >> 1)));
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t smw[2] = {sm[h].x, sm[h].y};
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      // code byte b -> both exponents already in place (bits 7..14 and 23..30)
      const uint32_t cb = (cd[h] >> (8 * b)) & 0xffu;
      // [a0, a0, a1, a1], then keep mantissa in the low and sign in the high byte of each half-word (eq. (2))
      const uint32_t p = byte_perm(0u, smw[b >> 1], (b & 1) ? 0x03030202u : 0x01010000u);
      o[4 * h + b] = (p & 0x807f807fu) | tbl[cb];
    }
  }
}

template <bool FULL>
__device__ inline void store_chunk_bf16(const DecompressArgs& a, uint64_t cbase, int lane, const uint32_t (&o)[8]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL || nvalid == 8) {
      st_stream(reinterpret_cast<u32x4*>(a.out + 2 * g0), u32x4{o[4 * h], o[4 * h + 1], o[4 * h + 2], o[4 * h + 3]});
    } else {
      uint16_t* q = reinterpret_cast<uint16_t*>(a.out) + g0;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if ((uint32_t)(2 * d) < nvalid) q[2 * d] = (uint16_t)o[4 * h + d];
        if ((uint32_t)(2 * d + 1) < nvalid) q[2 * d + 1] = (uint16_t)(o[4 * h + d] >> 16);
      }
    }
  }
}

// E5M2 dense decode of one chunk by one wave into registers: 16 elements per lane, o[d] holds
// elements 4 d .. 4 d + 3.  Lanes 2p and 2p+1 share 12 plane bytes: the even lane loads the first
// 8, the odd lane the last 4.
template <bool FULL>
__device__ inline void decode_chunk_e5m2(const DecompressArgs& a, const uint32_t* tbl, uint64_t cbase, int lane, uint32_t (&o)[4]) {
  const uint64_t g0 = cbase + lane * 16;
  const uint64_t sm_off = (cbase / 8) * 3 + (uint32_t)(lane >> 1) * 12;
  const uint8_t* sm_src = a.comp + a.off_sm + sm_off;
  const uint64_t sm_end = a256(a.sm_bytes);
  uint32_t d0 = 0, d1 = 0;
  u32x2 cd = u32x2{0u, 0u};
  if (lane & 1) {
    if (FULL || sm_off + 8 < sm_end) d0 = ld_stream(reinterpret_cast<const uint32_t*>(sm_src + 8));
  } else if (FULL || sm_off + 4 < sm_end) {
    const u32x2 v = ld_stream(reinterpret_cast<const u32x2*>(sm_src));   // 8 bytes below a multiple of 256: both in the stream
    d0 = v.x;
    d1 = v.y;
  } else if (sm_off < sm_end) {
    d0 = ld_stream(reinterpret_cast<const uint32_t*>(sm_src));
  }
  if (FULL || (g0 >> 1) < a256(a.code_bytes)) cd = ld_stream(reinterpret_cast<const u32x2*>(a.comp + a.off_code + (g0 >> 1)));
  const uint32_t d1_dn = __builtin_amdgcn_update_dpp(0u, d1, 0xA0, 0xf, 0xf, false);   // quad_perm [0,0,2,2]: the even neighbour's second dword
  // the lane's 48 plane bits
  const uint32_t lo = (lane & 1) ? (d1_dn >> 16) | (d0 << 16) : d0;
  const uint32_t hi = (lane & 1) ? d0 >> 16 : d1 & 0xffffu;
  const uint32_t r[4] = {lo & 0xfffu, (lo >> 12) & 0xfffu, (lo >> 24) | ((hi & 0xfu) << 8), (hi >> 4) & 0xfffu};
  const uint32_t cdw[2] = {cd.x, cd.y};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    // two code bytes -> four exponents already in place (bits 2..6 of each byte)
    const uint32_t c01 = (cdw[d >> 1] >> (16 * (d & 1))) & 0xffu, c23 = (cdw[d >> 1] >> (16 * (d & 1) + 8)) & 0xffu;
    o[d] = unpack3_e5m2(r[d]) | tbl[c01] | (tbl[c23] << 16);
  }
}

template <bool FULL>
__device__ inline void store_chunk_e5m2(const DecompressArgs& a, uint64_t cbase, int lane, const uint32_t (&o)[4]) {
  const uint64_t g0 = cbase + lane * 16;
  uint32_t nvalid = 16;
  if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 16 ? a.n - g0 : 16);
  if (FULL || nvalid == 16) {
    st_stream(reinterpret_cast<u32x4*>(a.out + g0), u32x4{o[0], o[1], o[2], o[3]});
  } else {
    uint8_t* q = a.out + g0;
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
  struct Out { uint32_t o[8]; };
  // table entry for a code byte: both exponents in place for one dword of output
  __device__ static inline uint32_t table(int cb, const uint8_t* dec) { return ((uint32_t)dec[cb & 15] << 7) | ((uint32_t)dec[cb >> 4] << 23); }
  __device__ static inline bool full(const DecompressArgs& a, uint64_t cbase) { return cbase + kChunk <= a.n; }
  template <bool FULL>
  __device__ static inline void decode(const DecompressArgs& a, const uint32_t* tbl, uint64_t cbase, int lane, Out& r) { decode_chunk_bf16<FULL>(a, tbl, cbase, lane, r.o); }
  template <bool FULL>
  __device__ static inline void store(const DecompressArgs& a, uint64_t cbase, int lane, const Out& r) { store_chunk_bf16<FULL>(a, cbase, lane, r.o); }
  // the scatter correction of the element at chunk position pos (wave-uniform), in the registers of the lane that holds it
  __device__ static inline bool patch_reg(Out& r, int lane, uint32_t pos, uint32_t val) {
    const uint32_t q = pos & 511u, e = q & 7u, sh = 16u * (e & 1u);
    patch_regs<8>(r.o, 4u * (pos >> 9) + (e >> 1), (uint32_t)lane == (q >> 3), 0x7f80u << sh, val << (7u + sh));
    return true;
  }
  // the same on the tensor in memory: exponent field := val, sign and mantissa from the stream
  __device__ static inline bool patch(const DecompressArgs& a, uint64_t i, uint32_t val) {
    const uint32_t sa = a.comp[a.off_sm + i];
    reinterpret_cast<uint16_t*>(a.out)[i] = (uint16_t)(((sa & 0x80u) << 8) | (val << 7) | (sa & 0x7fu));
    return true;
  }
};
struct DE5m2 {
  struct Out { uint32_t o[4]; };
  __device__ static inline uint32_t table(int cb, const uint8_t* dec) { return ((uint32_t)dec[cb & 15] << 2) | ((uint32_t)dec[cb >> 4] << 10); }
  __device__ static inline bool full(const DecompressArgs& a, uint64_t cbase) { return cbase + kChunk < a.n; }
  template <bool FULL>
  __device__ static inline void decode(const DecompressArgs& a, const uint32_t* tbl, uint64_t cbase, int lane, Out& r) { decode_chunk_e5m2<FULL>(a, tbl, cbase, lane, r.o); }
  template <bool FULL>
  __device__ static inline void store(const DecompressArgs& a, uint64_t cbase, int lane, const Out& r) { store_chunk_e5m2<FULL>(a, cbase, lane, r.o); }
  __device__ static inline bool patch_reg(Out& r, int lane, uint32_t pos, uint32_t val) {
    if (val > 31u) return false;
    const uint32_t e = pos & 15u, sh = 8u * (e & 3u);
    patch_regs<4>(r.o, e >> 2, (uint32_t)lane == (pos >> 4), 0x7cu << sh, val << (2u + sh));
    return true;
  }
  __device__ static inline bool patch(const DecompressArgs& a, uint64_t i, uint32_t val) {
    if (val > 31u) return false;
    const uint64_t bit = 3 * i;
    const uint8_t* p = a.comp + a.off_sm + (bit >> 3);
    uint32_t two = p[0];
    if ((bit & 7) > 5) two |= (uint32_t)p[1] << 8;   // the field straddles a byte; the next byte is inside the plane
    const uint32_t sa = (two >> (bit & 7)) & 7u;
    a.out[i] = (uint8_t)(((sa & 4u) << 5) | (val << 2) | (sa & 3u));
    return true;
  }
};

constexpr uint32_t kRegPatchMax = 32;   // escapes of a chunk that are applied in registers, before the store

// one workgroup: tile `tile` of the tensor described by a (4 waves x cpw chunks)
template <typename F>
__device__ inline void decompress_tile(const DecompressArgs& a, const uint8_t* dec, uint32_t tile, uint32_t* tbl) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t* tab = reinterpret_cast<const uint32_t*>(a.comp + a.off_tab);
  const uint32_t cpw = a.cpw;
  const uint32_t wave_chunk0 = (tile * kWaves + wave) * cpw;
  // first of all the loads everything else waits for: this wave's slice of the offset table (lane c
  // <-> its chunk c, one entry more for the end) and M as the table states it
  const uint32_t my_tab = (uint32_t)lane <= cpw && wave_chunk0 + lane <= a.n_chunks ? tab[wave_chunk0 + lane] : 0u;
  uint32_t M = tab[a.n_chunks];
  tbl[tid] = F::table(tid, dec);

  // escapes are only trusted if their sections lie inside the stream
  const uint64_t off_val = a.off_pos + a256(2ull * M);
  const bool esc_ok = M <= a.n && off_val + M <= a.comp_bytes;
  if (tile == 0 && tid == 0) {
    decompress_check_header(a, dec, M);
    if (!esc_ok) flag_bad(a);
  }
  if (!esc_ok) M = 0;
  const uint16_t* pos_arr = reinterpret_cast<const uint16_t*>(a.comp + a.off_pos);
  const uint8_t* val_arr = a.comp + off_val;
  __syncthreads();

  for (uint32_t c = 0; c < cpw; ++c) {
    const uint32_t chunk = wave_chunk0 + c;
    if (chunk >= a.n_chunks) break;
    const uint64_t cbase = (uint64_t)chunk * kChunk;
    const uint32_t lo = __builtin_amdgcn_readlane(my_tab, c), hi = __builtin_amdgcn_readlane(my_tab, c + 1);
    const uint32_t clen = (uint32_t)(a.n - cbase < kChunk ? a.n - cbase : kChunk);
    const bool esc_valid = hi >= lo && hi - lo <= clen && hi <= M;
    const uint32_t cnt = esc_valid ? hi - lo : 0u;
    if (!esc_valid && lane == 0) flag_bad(a);
    // a few escapes (the usual case): their records are fetched while the planes are on their way,
    // and applied to the decoded words in registers before the one store
    const bool in_regs = cnt > 0 && cnt <= kRegPatchMax;
    uint32_t pos = 0, val = 0;
    if (in_regs && (uint32_t)lane < cnt) {
      pos = pos_arr[lo + lane];
      val = val_arr[lo + lane];
    }
    typename F::Out r;
    const bool full = F::full(a, cbase);
    if (full) F::template decode<true>(a, tbl, cbase, lane, r);
    else F::template decode<false>(a, tbl, cbase, lane, r);
    if (in_regs) {
      for (uint32_t j = 0; j < cnt; ++j) {
        const uint32_t p = __builtin_amdgcn_readlane(pos, j), v = __builtin_amdgcn_readlane(val, j);
        if (p >= clen || !F::patch_reg(r, lane, p, v)) {
          if (lane == 0) flag_bad(a);
        }
      }
    }
    if (full) F::template store<true>(a, cbase, lane, r);
    else F::template store<false>(a, cbase, lane, r);
    if (cnt > kRegPatchMax) {
      // many escapes: sparse overwrite of the tensor in memory by the wave that wrote the chunk,
      // once its dense stores have completed
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      for (uint32_t j = lo + lane; j < hi; j += 64) {
        const uint32_t p = pos_arr[j];
        const uint32_t v = val_arr[j];
        if (p >= clen || !F::patch(a, cbase + p, v)) flag_bad(a);
      }
    }
  }
}

template <typename F>
__global__ __launch_bounds__(kThreads) void decompress_kernel(const DecompressArgs a) {
  __shared__ uint32_t tbl[256];
  decompress_tile<F>(a, a.dec, blockIdx.x, tbl);
}

// several streams in one launch: blockIdx.y picks the stream, blockIdx.x the tile
struct DBatchItem {
  const uint8_t* comp;
  uint8_t* out;
  uint64_t n, comp_bytes;
};
struct DecompressBatchArgs {
  DBatchItem item[kBatchMax];
  uint8_t dec_of[kBatchMax];
  splitzip_sizes* sizes;   // nullable; one record, status bits sticky
  uint32_t cpw, dtype;
  uint8_t dec[kBatchLuts][16];
};

template <typename F>
__global__ __launch_bounds__(kThreads) void decompress_batch_kernel(const DecompressBatchArgs b) {
  __shared__ uint32_t tbl[256];
  const DBatchItem it = b.item[blockIdx.y];
  const Layout L = make_layout(it.n, (int)b.dtype);
  const uint32_t n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * b.cpw - 1) / (kWaves * b.cpw));
  if (blockIdx.x >= (n_tiles ? n_tiles : 1u)) return;
  DecompressArgs a;
  a.comp = it.comp;
  a.out = it.out;
  a.n = it.n;
  a.comp_bytes = it.comp_bytes;
  a.sizes = b.sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = n_tiles;
  a.cpw = b.cpw;
  a.dtype = b.dtype;
  decompress_tile<F>(a, b.dec[b.dec_of[blockIdx.y]], blockIdx.x, tbl);   // a.dec stays unset: the table comes from the kernel arguments
}

// ---------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------

// Calibration histogram (section 3.3) of a device sample: exponent counts, added to hist[256].
// Every workgroup counts into eight copies of the bins in LDS -- lane l uses copy l mod 8, which
// keeps the lanes that meet on one of the few common exponents apart -- and adds its non-zero
// totals to the global bins at the end.
template <bool BF16>
__global__ __launch_bounds__(1024) void histogram_kernel(const uint8_t* in, uint64_t n, uint64_t* hist) {
  __shared__ uint32_t bins[8][256];
  const int tid = threadIdx.x;
  for (int i = tid; i < 8 * 256; i += 1024) (&bins[0][0])[i] = 0;
  __syncthreads();
  uint32_t* mine = bins[tid & 7];
  const uint64_t bytes = n * (BF16 ? 2 : 1), nvec = bytes / 16;
  const u32x4* v = reinterpret_cast<const u32x4*>(in);
  for (uint64_t i = blockIdx.x * 1024ull + tid; i < nvec; i += (uint64_t)gridDim.x * 1024) {
    const u32x4 q = ld_stream(v + i);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      if (BF16) {
        atomicAdd(&mine[(w[d] >> 7) & 0xffu], 1u);
        atomicAdd(&mine[(w[d] >> 23) & 0xffu], 1u);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) atomicAdd(&mine[(w[d] >> (8 * j + 2)) & 31u], 1u);
      }
    }
  }
  // the words behind the last whole vector, by workgroup 0
  if (blockIdx.x == 0) {
    for (uint64_t i = nvec * 16 + (uint64_t)tid * (BF16 ? 2 : 1); i < bytes; i += 1024 * (BF16 ? 2 : 1)) {
      const uint32_t e = BF16 ? ((uint32_t)(in[i] | (in[i + 1] << 8)) >> 7) & 0xffu : ((uint32_t)in[i] >> 2) & 31u;
      atomicAdd(&mine[e], 1u);
    }
  }
  __syncthreads();
  if (tid < 256) {
    uint64_t c = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) c += bins[r][tid];
    if (c) atomicAdd(reinterpret_cast<unsigned long long*>(&hist[tid]), (unsigned long long)c);
  }
}

__global__ void workspace_init_kernel(uint32_t* p, uint32_t nwords) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += gridDim.x * blockDim.x) p[i] = i == 0 ? 1u : 0u;
}

// Per step a workgroup reads four coalesced 4 KB runs and writes three: the codec's 4:3 traffic
// without its arithmetic.
__global__ __launch_bounds__(kThreads) void traffic_probe_kernel(const u32x4* src, uint64_t nread,
                                                                  u32x4* dst, uint64_t nwrite) {
  const uint64_t steps = (nread + 4 * kThreads - 1) / (4 * kThreads);
  for (uint64_t s = blockIdx.x; s < steps; s += gridDim.x) {
    u32x4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint64_t idx = (4 * s + i) * kThreads + threadIdx.x;
      v[i] = idx < nread ? ld_stream(src + idx) : u32x4{0u, 0u, 0u, 0u};
    }
    v[0].x ^= v[3].x; v[1].y ^= v[3].y; v[2].z ^= v[3].z; v[0].w ^= v[3].w;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const uint64_t idx = (3 * s + i) * kThreads + threadIdx.x;
      if (idx < nwrite) st_stream(dst + idx, v[i]);
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

bool dtype_ok(int dtype) { return dtype == SPLITZIP_BF16 || dtype == SPLITZIP_FP8_E5M2; }
unsigned exp_values(int dtype) { return dtype == SPLITZIP_BF16 ? 256u : 32u; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int env_int(const char* name, int dflt) {
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  const int v = atoi(s);
  return v > 0 ? v : dflt;
}

int cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (!cached[dev]) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// chunks per wave: the largest power of two (up to `most`) that still leaves `want` tiles per CU
uint32_t pick_cpw(uint64_t n_chunks, uint32_t most, uint32_t want_tiles_per_cu) {
  const uint64_t want = (uint64_t)cu_count() * want_tiles_per_cu;
  uint32_t cpw = most;
  while (cpw > 1 && (n_chunks + (uint64_t)kWaves * cpw - 1) / (kWaves * cpw) < want) cpw >>= 1;
  return cpw;
}

// Chunks per wave of a decompress launch over n_chunks chunks in all.  Measured on 64 MiB BF16 /
// 32 MiB E5M2 tensors: BF16 wants one chunk per wave for a single tensor (32 768 chunks) and two for
// a whole cache in one launch; E5M2 wants four and eight.
uint32_t pick_decompress_cpw(uint64_t n_chunks, int dtype, int tiles_per_cu_env) {
  const uint32_t most = dtype == SPLITZIP_BF16 ? 2 : 8;
  const uint32_t want = tiles_per_cu_env ? (uint32_t)tiles_per_cu_env : (dtype == SPLITZIP_BF16 ? 32u : 8u);
  return pick_cpw(n_chunks, most, want);
}

// tables must describe one bijection between 16 codes and 16 distinct exponents
bool codebook_ok(const splitzip_codebook* cb, int dtype) {
  if (!cb || cb->dtype != (uint32_t)dtype) return false;
  unsigned members = 0;
  for (unsigned v = 0; v < 256; ++v) {
    if (cb->member[v] > 1) return false;
    if (cb->member[v]) {
      if (v >= exp_values(dtype) || cb->enc[v] > 15 || cb->dec[cb->enc[v]] != v) return false;
      ++members;
    } else if (cb->enc[v] != 0) {
      return false;
    }
  }
  return members == 16;
}

template <int T>
void launch_compress(unsigned grid, hipStream_t stream, const CompressArgs& a) {
  if (a.p.dtype == SPLITZIP_BF16) hipLaunchKernelGGL((compress_kernel<T, Bf16>), dim3(grid), dim3(T), 0, stream, a);
  else hipLaunchKernelGGL((compress_kernel<T, E5m2>), dim3(grid), dim3(T), 0, stream, a);
}

// workgroups of T threads that can be resident on the current device at the same time
template <int T>
uint32_t resident_workgroups() {
  static uint32_t cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (!cached[dev]) {
    int per_cu = 0;
    // both formats' kernels use the same LDS; the BF16 one needs more registers
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, compress_kernel<T, Bf16>, T, 0) != hipSuccess || per_cu <= 0)
      return 0;
    cached[dev] = (uint32_t)per_cu * (uint32_t)cu_count();
  }
  return cached[dev];
}

// the same for the batch kernel (more LDS)
uint32_t resident_workgroups_batch() {
  static uint32_t cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (!cached[dev]) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, compress_batch_kernel<1024, Bf16>, 1024, 0) != hipSuccess || per_cu <= 0)
      return 0;
    cached[dev] = (uint32_t)per_cu * (uint32_t)cu_count();
  }
  return cached[dev];
}

}  // namespace

extern "C" {

int splitzip_version(void) { return 1; }

const char* splitzip_strerror(int err) {
  switch (err) {
    case SPLITZIP_OK: return "ok";
    case SPLITZIP_ERR_INVALID_ARG: return "invalid argument";
    case SPLITZIP_ERR_UNSUPPORTED: return "unsupported size or format";
    case SPLITZIP_ERR_CAPACITY: return "buffer too small";
    case SPLITZIP_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

int splitzip_codebook_from_dec(const uint8_t dec[16], int dtype, splitzip_codebook* out) {
  if (!dec || !out || !dtype_ok(dtype)) return SPLITZIP_ERR_INVALID_ARG;
  splitzip_codebook cb;
  memset(&cb, 0, sizeof cb);
  cb.dtype = (uint32_t)dtype;
  for (unsigned k = 0; k < 16; ++k) {
    const unsigned v = dec[k];
    if (v >= exp_values(dtype) || cb.member[v]) return SPLITZIP_ERR_INVALID_ARG;
    cb.dec[k] = (uint8_t)v;
    cb.enc[v] = (uint8_t)k;
    cb.member[v] = 1;
  }
  *out = cb;
  return SPLITZIP_OK;
}

int splitzip_calibrate(const void* h_sample, uint64_t n_elems, int dtype, splitzip_codebook* out,
                       uint64_t* hist_out) {
  if (!out || !dtype_ok(dtype) || (n_elems && !h_sample)) return SPLITZIP_ERR_INVALID_ARG;
  uint64_t hist[256] = {0};
  if (dtype == SPLITZIP_BF16) {
    const uint16_t* p = static_cast<const uint16_t*>(h_sample);
    for (uint64_t i = 0; i < n_elems; ++i) hist[(p[i] >> 7) & 0xff]++;
  } else {
    const uint8_t* p = static_cast<const uint8_t*>(h_sample);
    for (uint64_t i = 0; i < n_elems; ++i) hist[(p[i] >> 2) & 0x1f]++;
  }
  if (hist_out) memcpy(hist_out, hist, sizeof hist);
  return splitzip_codebook_from_hist(hist, dtype, out);
}

int splitzip_codebook_from_hist(const uint64_t hist[256], int dtype, splitzip_codebook* out) {
  if (!hist || !out || !dtype_ok(dtype)) return SPLITZIP_ERR_INVALID_ARG;
  // rank exponents by (count descending, value ascending): insertion into a sorted top-16 list
  const unsigned nv = exp_values(dtype);
  uint8_t top[16];
  unsigned filled = 0;
  for (unsigned v = 0; v < nv; ++v) {
    unsigned at = filled;
    while (at > 0 && hist[top[at - 1]] < hist[v]) --at;   // strict: equal counts keep the smaller value first
    if (at >= 16) continue;
    const unsigned last = filled < 16 ? filled : 15;
    for (unsigned i = last; i > at; --i) top[i] = top[i - 1];
    top[at] = (uint8_t)v;
    if (filled < 16) ++filled;
  }
  return splitzip_codebook_from_dec(top, dtype, out);
}

int splitzip_histogram(const void* d_sample, uint64_t n_elems, int dtype, uint64_t* d_hist, void* stream) {
  if (!dtype_ok(dtype) || !d_hist || (n_elems && !d_sample) || !aligned16(d_sample) ||
      (reinterpret_cast<uintptr_t>(d_hist) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (n_elems == 0) return SPLITZIP_OK;
  const uint64_t nvec = (n_elems * (dtype == SPLITZIP_BF16 ? 2 : 1) + 15) / 16;
  uint64_t grid = (nvec + 4 * 1024 - 1) / (4 * 1024);   // at least four vectors per thread
  const uint64_t most = (uint64_t)cu_count() * 2;
  if (grid > most) grid = most;
  if (grid < 1) grid = 1;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == SPLITZIP_BF16)
    hipLaunchKernelGGL(histogram_kernel<true>, dim3((unsigned)grid), dim3(1024), 0, st, static_cast<const uint8_t*>(d_sample), n_elems, d_hist);
  else
    hipLaunchKernelGGL(histogram_kernel<false>, dim3((unsigned)grid), dim3(1024), 0, st, static_cast<const uint8_t*>(d_sample), n_elems, d_hist);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

size_t splitzip_total_bytes(uint64_t n_elems, uint64_t n_escapes, int dtype) {
  if (!dtype_ok(dtype) || n_elems >> 32) return 0;
  const Layout L = make_layout(n_elems, dtype);
  return (size_t)(L.off_pos + a256(2 * n_escapes) + n_escapes);
}
size_t splitzip_fixed_bytes(uint64_t n_elems, int dtype) { return splitzip_total_bytes(n_elems, 0, dtype); }
size_t splitzip_compress_bound(uint64_t n_elems, int dtype) { return splitzip_total_bytes(n_elems, n_elems, dtype); }

size_t splitzip_workspace_bytes(uint64_t n_elems, int dtype) {
  if (!dtype_ok(dtype) || n_elems >> 32) return 0;
  return (size_t)(kWsHeaderBytes + kWsTableBytes + a256(n_elems));
}

int splitzip_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!d_workspace || !aligned16(d_workspace) || workspace_bytes < kWsHeaderBytes + kWsTableBytes)
    return SPLITZIP_ERR_INVALID_ARG;
  // header and exchange words; the epoch starts at 1 so that a cleared word never looks published
  hipLaunchKernelGGL(workspace_init_kernel, dim3(8), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint32_t*>(d_workspace), (uint32_t)((kWsHeaderBytes + kWsTableBytes) / 4));
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_compress(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                      void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                      splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || !d_out || !d_workspace || !d_sizes || (n_elems && !d_in)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_workspace) ||
      (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (!codebook_ok(cb, dtype)) return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (out_capacity < splitzip_fixed_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
  if (workspace_bytes < splitzip_workspace_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;

  const Layout L = make_layout(n_elems, dtype);
  CompressArgs a;
  memset(&a, 0, sizeof a);
  a.p = make_planes(d_in, d_out, n_elems, out_capacity, dtype);
  uint8_t* ws = static_cast<uint8_t*>(d_workspace);
  a.ws_hdr = reinterpret_cast<uint32_t*>(ws);
  a.state = reinterpret_cast<uint64_t*>(ws + kWsHeaderBytes);
  a.val_stage = ws + kWsHeaderBytes + kWsTableBytes;
  a.sizes = d_sizes;
  memcpy(a.dec, cb->dec, 16);
  for (unsigned v = 0; v < 256; ++v) a.lut[v] = cb->member[v] ? cb->enc[v] : 0x100u;   // indexed by the exponent
  static const int spin_env = env_int("SPLITZIP_SPIN_TICKS", 0);
  a.spin_ticks = spin_env ? (uint64_t)spin_env : kSpinTicks;

  // the grid: every workgroup resident at once, not more workgroups than tiles
  static const int threads = env_int("SPLITZIP_COMPRESS_THREADS", 1024);
  static const int wgs_per_cu = env_int("SPLITZIP_COMPRESS_WGS_PER_CU", 1);
  const int T = threads == 256 || threads == 512 ? threads : 1024;
  const uint32_t nw = (uint32_t)T / 64;
  uint32_t resident = T == 256 ? resident_workgroups<256>() : T == 512 ? resident_workgroups<512>() : resident_workgroups<1024>();
  if (!resident) return SPLITZIP_ERR_HIP;
  uint32_t w_max = (uint32_t)cu_count() * (uint32_t)wgs_per_cu;
  if (w_max > resident) w_max = resident;
  static const int max_wgs = env_int("SPLITZIP_COMPRESS_MAX_WGS", 0);   // small grids, to exercise calls of several launches
  if (max_wgs && w_max > (uint32_t)max_wgs) w_max = (uint32_t)max_wgs;
  if (w_max > kMaxWorkgroups) w_max = kMaxWorkgroups;
  const uint64_t seg_cap = (uint64_t)w_max * kMaxRange;   // chunks one launch can take
  const hipStream_t st = static_cast<hipStream_t>(stream);
  static const int missing = env_int("SPLITZIP_TEST_AWAIT_EXTRA_WGS", 0);   // error-path tests only

  uint64_t done = 0;
  const bool several = L.n_chunks > seg_cap;
  do {
    const uint64_t left = L.n_chunks - done;
    const uint32_t seg = (uint32_t)(left < seg_cap ? left : seg_cap);
    a.seg_chunk0 = (uint32_t)done;
    a.seg_chunks = seg;
    a.flags = (done == 0 ? kSegFirst : 0u) | (done + seg == L.n_chunks ? kSegLast : 0u);
    uint32_t grid = (seg + nw - 1) / nw;    // at least one chunk per wave where the tensor allows
    if (grid > w_max) grid = w_max;
    if (grid < 1) grid = 1;
    a.expect_wgs = grid + (uint32_t)missing;
    if (a.expect_wgs > kMaxWorkgroups) return SPLITZIP_ERR_INVALID_ARG;
    if (T == 256) launch_compress<256>(grid, st, a);
    else if (T == 512) launch_compress<512>(grid, st, a);
    else launch_compress<1024>(grid, st, a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
    done += seg;
  } while (done < L.n_chunks);
  if (several) {
    hipLaunchKernelGGL(compress_finish_kernel, dim3(64), dim3(kThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
  }
  return SPLITZIP_OK;
}

int splitzip_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                        const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || !d_comp || (n_elems && !d_out)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_comp) || !aligned16(d_out) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (!codebook_ok(cb, dtype)) return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (comp_bytes < splitzip_fixed_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;

  const Layout L = make_layout(n_elems, dtype);
  DecompressArgs a;
  memset(&a, 0, sizeof a);
  a.comp = static_cast<const uint8_t*>(d_comp);
  a.out = static_cast<uint8_t*>(d_out);
  a.n = n_elems;
  a.comp_bytes = comp_bytes;
  a.sizes = d_sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  static const int cpw_env = env_int("SPLITZIP_DECOMPRESS_CPW", 0);
  static const int tiles_per_cu = env_int("SPLITZIP_DECOMPRESS_TILES_PER_CU", 0);
  a.cpw = cpw_env ? (uint32_t)cpw_env : pick_decompress_cpw(L.n_chunks, dtype, tiles_per_cu);
  if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * a.cpw - 1) / (kWaves * a.cpw));
  a.dtype = (uint32_t)dtype;
  memcpy(a.dec, cb->dec, 16);

  const unsigned grid = a.n_tiles ? a.n_tiles : 1u;
  if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL(decompress_kernel<DBf16>, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  else hipLaunchKernelGGL(decompress_kernel<DE5m2>, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_compress_batch(const splitzip_item* items, uint32_t n_items, int dtype, void* d_workspace,
                            size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || (n_items && (!items || !d_sizes)) || !d_workspace || !aligned16(d_workspace) ||
      (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  uint64_t n_max = 0;
  for (uint32_t i = 0; i < n_items; ++i) {
    const splitzip_item& it = items[i];
    if (!it.d_out || (it.n_elems && !it.d_in) || !aligned16(it.d_in) || !aligned16(it.d_out) || !codebook_ok(it.cb, dtype))
      return SPLITZIP_ERR_INVALID_ARG;
    if (it.n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
    if (it.out_capacity < splitzip_fixed_bytes(it.n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
    if (it.n_elems > n_max) n_max = it.n_elems;
  }
  if (workspace_bytes < splitzip_workspace_bytes(n_max, dtype)) return SPLITZIP_ERR_CAPACITY;
  if (n_items == 0) return SPLITZIP_OK;

  static const int wgs_per_cu = env_int("SPLITZIP_COMPRESS_WGS_PER_CU", 1);
  const uint32_t resident = resident_workgroups_batch();
  if (!resident) return SPLITZIP_ERR_HIP;
  uint32_t W = (uint32_t)cu_count() * (uint32_t)wgs_per_cu;
  if (W > resident) W = resident;
  if (W > kRingWgs) W = kRingWgs;
  static const int max_wgs = env_int("SPLITZIP_COMPRESS_MAX_WGS", 0);
  if (max_wgs && W > (uint32_t)max_wgs) W = (uint32_t)max_wgs;
  const uint64_t chunk_cap = (uint64_t)W * kMaxRange;   // chunks of one tensor the batch kernel can take
  static const int spin_env = env_int("SPLITZIP_SPIN_TICKS", 0);
  static const int missing = env_int("SPLITZIP_TEST_AWAIT_EXTRA_WGS", 0);   // error-path tests only
  const hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(d_workspace);

  uint32_t i = 0;
  while (i < n_items) {
    // a tensor beyond the batch kernel's reach goes through the single call, in its place in the order
    if ((items[i].n_elems + kChunk - 1) / kChunk > chunk_cap) {
      const int rc = splitzip_compress(items[i].d_in, items[i].n_elems, dtype, items[i].cb, items[i].d_out,
                                       items[i].out_capacity, d_workspace, workspace_bytes, d_sizes + i, stream);
      if (rc != SPLITZIP_OK) return rc;
      ++i;
      continue;
    }
    // one launch: up to kBatchMax tensors that share at most kBatchLuts codebooks
    CompressBatchArgs a;
    memset(&a, 0, sizeof a);
    uint32_t k = 0, n_luts = 0;
    for (; i + k < n_items && k < kBatchMax; ++k) {
      const splitzip_item& it = items[i + k];
      if ((it.n_elems + kChunk - 1) / kChunk > chunk_cap) break;
      uint32_t id = 0;
      while (id < n_luts && memcmp(a.dec[id], it.cb->dec, 16) != 0) ++id;
      if (id == n_luts) {
        if (n_luts == kBatchLuts) break;
        memcpy(a.dec[id], it.cb->dec, 16);
        for (unsigned v = 0; v < 256; ++v) a.lut[id][v] = it.cb->member[v] ? it.cb->enc[v] : 0x100u;
        ++n_luts;
      }
      a.item[k].in = static_cast<const uint8_t*>(it.d_in);
      a.item[k].out = static_cast<uint8_t*>(it.d_out);
      a.item[k].n = it.n_elems;
      a.item[k].capacity = it.out_capacity;
      a.lut_of[k] = (uint8_t)id;
    }
    a.sizes = d_sizes + i;
    a.ws_hdr = reinterpret_cast<uint32_t*>(ws);
    a.state = reinterpret_cast<uint64_t*>(ws + kWsHeaderBytes);
    a.spin_ticks = spin_env ? (uint64_t)spin_env : kSpinTicks;
    a.n_items = k;
    a.dtype = (uint32_t)dtype;
    // Workgroups per tensor: all of them for large tensors; for small ones a power-of-two share that
    // leaves each workgroup about 64 chunks, the groups working on different tensors side by side.
    uint64_t chunks_max = 0;
    for (uint32_t q = 0; q < k; ++q) {
      const uint64_t c = (a.item[q].n + kChunk - 1) / kChunk;
      if (c > chunks_max) chunks_max = c;
    }
    uint32_t G = W;
    while (G > 8 && G % 2 == 0 && (uint64_t)(G / 2) * 64 >= chunks_max && W / (G / 2) <= k) G /= 2;   // never more groups than tensors
    while ((uint64_t)G * kMaxRange < chunks_max) G *= 2;   // never beyond W: chunks_max <= chunk_cap
    if (G > W) G = W;
    a.group_wgs = G;
    a.await_extra = (uint32_t)missing;
    const uint32_t grid = (W / G) * G;
    if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL((compress_batch_kernel<1024, Bf16>), dim3(grid), dim3(1024), 0, st, a);
    else hipLaunchKernelGGL((compress_batch_kernel<1024, E5m2>), dim3(grid), dim3(1024), 0, st, a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
    i += k;
  }
  return SPLITZIP_OK;
}

int splitzip_decompress_batch(const splitzip_ditem* items, uint32_t n_items, int dtype, splitzip_sizes* d_sizes,
                              void* stream) {
  if (!dtype_ok(dtype) || (n_items && !items) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u)) return SPLITZIP_ERR_INVALID_ARG;
  for (uint32_t i = 0; i < n_items; ++i) {
    const splitzip_ditem& it = items[i];
    if (!it.d_comp || (it.n_elems && !it.d_out) || !aligned16(it.d_comp) || !aligned16(it.d_out) || !codebook_ok(it.cb, dtype))
      return SPLITZIP_ERR_INVALID_ARG;
    if (it.n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
    if (it.comp_bytes < splitzip_fixed_bytes(it.n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
  }
  static const int cpw_env = env_int("SPLITZIP_DECOMPRESS_CPW", 0);
  static const int tiles_per_cu = env_int("SPLITZIP_DECOMPRESS_TILES_PER_CU", 0);
  uint32_t i = 0;
  while (i < n_items) {
    DecompressBatchArgs a;
    memset(&a, 0, sizeof a);
    uint32_t k = 0, n_decs = 0;
    uint64_t chunks_all = 0, chunks_max = 0;
    for (; i + k < n_items && k < kBatchMax; ++k) {
      const splitzip_ditem& it = items[i + k];
      uint32_t id = 0;
      while (id < n_decs && memcmp(a.dec[id], it.cb->dec, 16) != 0) ++id;
      if (id == n_decs) {
        if (n_decs == kBatchLuts) break;
        memcpy(a.dec[id], it.cb->dec, 16);
        ++n_decs;
      }
      a.item[k].comp = static_cast<const uint8_t*>(it.d_comp);
      a.item[k].out = static_cast<uint8_t*>(it.d_out);
      a.item[k].n = it.n_elems;
      a.item[k].comp_bytes = it.comp_bytes;
      a.dec_of[k] = (uint8_t)id;
      const uint64_t c = (it.n_elems + kChunk - 1) / kChunk;
      chunks_all += c;
      if (c > chunks_max) chunks_max = c;
    }
    a.sizes = d_sizes;
    a.dtype = (uint32_t)dtype;
    a.cpw = cpw_env ? (uint32_t)cpw_env : pick_decompress_cpw(chunks_all, dtype, tiles_per_cu);
    if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
    uint64_t gx = (chunks_max + (uint64_t)kWaves * a.cpw - 1) / (kWaves * a.cpw);
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, k);
    if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL(decompress_batch_kernel<DBf16>, grid, dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
    else hipLaunchKernelGGL(decompress_batch_kernel<DE5m2>, grid, dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
    i += k;
  }
  return SPLITZIP_OK;
}

int splitzip_traffic_probe(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes, void* stream) {
  if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || write_bytes > read_bytes)
    return SPLITZIP_ERR_INVALID_ARG;
  const uint64_t nread = read_bytes / 16, nwrite = write_bytes / 16;
  if (!nread) return SPLITZIP_OK;
  static const int wgs_per_cu = env_int("SPLITZIP_PROBE_WGS_PER_CU", 8);
  uint64_t grid = (uint64_t)cu_count() * wgs_per_cu;
  const uint64_t need = (nread + 4 * kThreads - 1) / (4 * kThreads);
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(traffic_probe_kernel, dim3((unsigned)grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(d_src), nread, static_cast<u32x4*>(d_dst), nwrite);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

}  // extern "C"
