// SplitZip codec for MI355X (gfx950): HIP kernels and the C ABI of include/splitzip.h.
//
// One compress call is ONE kernel launch.  The dense transform (paper section
// 3.2 eq. (1), encode table, nibble pack, sign+mantissa plane) is fused with
// escape detection, per-chunk counting and the position-ordered compaction of
// the escape stream (appendix A fuses only the counting).  The input is read
// exactly once: escapes are staged in LDS while their words are in registers,
// and the cross-workgroup offsets come from a decoupled look-back scan over
// per-tile escape counts, so the output does not depend on scheduling.
// One decompress call is ONE kernel launch as well: nibble unpack, decode
// table, eq. (2), and the sparse overwrite done by the wave that owns the
// chunk once its own dense stores have completed.
//
// Work decomposition (wavefront = 64 lanes, workgroup = 4 waves):
//   chunk = 1024 elements (the escape-position granule), owned by one wave and
//           processed as two half-chunks of 512 elements; in a half-chunk lane
//           l owns elements [8 l, 8 l + 8): every global access of a wave is
//           one fully coalesced run (16, 8 or 4 bytes per lane).
//   tile  = 4 waves x cpw consecutive chunks each, one tile per workgroup;
//           cpw (1..16) is chosen per call so that the grid fills the chip.
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
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr uint32_t kMaxCpw = 16;                          // chunks per wave per tile, at most
constexpr uint32_t kMinTileChunks = kWaves;               // smallest tile (cpw = 1)
constexpr uint32_t kStageCap = 512;                       // escapes a wave can stage in LDS
constexpr uint32_t kWsHeaderBytes = 64;                   // ticket, done, flags
constexpr uint32_t kSpinLimit = 1u << 22;                 // look-back polls before giving up

__host__ __device__ inline uint64_t a16(uint64_t x) { return (x + 15u) & ~(uint64_t)15u; }
__host__ __device__ inline uint64_t a256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

struct Layout {
  uint64_t n, n_chunks, sm_bytes, code_bytes;
  uint64_t off_tab, off_sm, off_code, off_pos;  // the value section starts at off_pos + a16(2M)
};

__host__ __device__ inline Layout make_layout(uint64_t n, int dtype) {
  Layout L;
  L.n = n;
  L.n_chunks = (n + kChunk - 1) / kChunk;
  L.sm_bytes = dtype == SPLITZIP_BF16 ? n : (3 * n + 7) / 8;
  L.code_bytes = (n + 1) / 2;
  L.off_tab = kHeaderBytes;
  L.off_sm = L.off_tab + a16(4 * (L.n_chunks + 1));
  L.off_code = L.off_sm + a16(L.sm_bytes);
  L.off_pos = L.off_code + a16(L.code_bytes);
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

// tile state of the decoupled look-back scan: flag in the two top bits, count below
constexpr uint64_t kFlagAgg = 1ull << 62;   // value = escapes of this tile only
constexpr uint64_t kFlagInc = 2ull << 62;   // value = escapes of all tiles up to and including this one

// Run by one whole wave.  Publishes this tile's escape count, sums the counts
// of all earlier tiles (64 predecessors per poll) and publishes the inclusive
// total.  Flag and count share one 64-bit word, so relaxed accesses suffice.
// Tiles are handed out by a ticket counter: every tile a wave waits for belongs
// to a workgroup that is already running and that publishes its count without
// waiting for anyone, so the wait always ends; the poll limit only guards
// against a workspace that was never initialised.
__device__ inline uint32_t lookback(uint64_t* state, uint32_t tile, uint32_t agg, int lane,
                                    uint32_t* ws_flags) {
  if (tile == 0) {
    if (lane == 0) st_agent(&state[0], kFlagInc | (uint64_t)agg);
    return 0;
  }
  if (lane == 0) st_agent(&state[tile], kFlagAgg | (uint64_t)agg);
  uint32_t prefix = 0;
  int64_t base = (int64_t)tile - 1;
  uint32_t spins = 0;
  for (;;) {
    const int64_t idx = base - lane;
    const uint64_t s = idx >= 0 ? ld_agent(&state[idx]) : kFlagInc;  // before tile 0: inclusive 0
    const uint32_t flag = (uint32_t)(s >> 62);
    const uint64_t inc_mask = __ballot(flag == 2u);
    const uint64_t empty_mask = __ballot(flag == 0u);
    const int first_inc = inc_mask ? (__ffsll((unsigned long long)inc_mask) - 1) : 64;
    const uint64_t need = first_inc >= 63 ? ~0ull : ((2ull << first_inc) - 1ull);
    if (empty_mask & need) {
      if (++spins > kSpinLimit) {
        if (lane == 0) atomicOr(ws_flags, SPLITZIP_STATUS_INTERNAL);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
      continue;
    }
    prefix += wave_last(wave_incl_scan(lane <= first_inc ? (uint32_t)s : 0u));
    if (first_inc < 64) break;
    base -= 64;
  }
  if (lane == 0) st_agent(&state[tile], kFlagInc | (uint64_t)(prefix + agg));
  return prefix;
}

// ---------------------------------------------------------------------------
// compress
// ---------------------------------------------------------------------------

struct CompressArgs {
  const uint8_t* in;
  uint8_t* out;
  uint64_t n, capacity;
  uint32_t* ws_hdr;      // [0] ticket, [1] done, [2] flags
  uint64_t* state;       // n_tiles look-back words
  uint8_t* val_stage;    // n bytes: escape values until M is known
  splitzip_sizes* sizes;
  uint64_t off_tab, off_sm, off_code, off_pos, sm_bytes, code_bytes;
  uint32_t n_chunks, n_tiles, cpw, dtype;
  uint8_t dec[16];
  uint16_t lut[256];     // exponent -> code | (non-member ? 0x100 : 0)   (the "marked" table of appendix A)
};

// where a chunk's escape records go: LDS staging (first pass) or their final place (second pass)
struct LdsSink {
  uint16_t* pos;
  uint8_t* val;
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (r < kStageCap) {
      pos[r] = (uint16_t)p;
      val[r] = (uint8_t)e;
    }
  }
};
struct GlobalSink {
  const CompressArgs* a;
  __device__ inline void put(uint32_t r, uint32_t p, uint32_t e) const {
    if (a->off_pos + 2ull * (r + 1) <= a->capacity) reinterpret_cast<uint16_t*>(a->out + a->off_pos)[r] = (uint16_t)p;
    st_agent(a->val_stage + r, (uint8_t)e);
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

// One chunk by one wave: load, dense transform, (optionally) plane stores, escape
// ranks inside the chunk, escape records into `sink` starting at rank `base`.
// Returns the chunk's escape count (wave-uniform).
template <bool FULL, bool STORE, typename Sink>
__device__ inline uint32_t compress_chunk_bf16(const CompressArgs& a, const uint16_t* lut, uint32_t* park,
                                               uint64_t cbase, int lane, uint32_t base, const Sink& sink) {
  uint32_t w[2][4], F[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;   // first element of this lane's group
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL || nvalid == 8) {
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
      // Sections are padded to 16 bytes and a lane's group never straddles the padded end, so
      // whole-group stores also write the zero padding.
      if (FULL || g0 < a16(a.sm_bytes)) st_stream(reinterpret_cast<u32x2*>(a.out + a.off_sm + g0), sm);
      if (FULL || (g0 >> 1) < a16(a.code_bytes))
        st_stream(reinterpret_cast<uint32_t*>(a.out + a.off_code + (g0 >> 1)), code);
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

// Last workgroup to finish: M is known now.  Moves the staged escape values
// behind the position array, writes pads, header and sizes, and leaves the
// workspace zeroed for the next call.  The staged values were written with
// agent-scope stores that had completed before their workgroup signalled, and
// are read with agent-scope loads.
__device__ void compress_finalize(const CompressArgs& a, int tid) {
  const uint32_t M = a.n_tiles ? (uint32_t)ld_agent(&a.state[a.n_tiles - 1]) : 0u;
  const uint64_t off_val = a.off_pos + a16(2ull * M);
  const uint64_t total = off_val + M;
  const uint64_t nvec = M / 8;
  const uint64_t* src = reinterpret_cast<const uint64_t*>(a.val_stage);
  uint64_t* dst = reinterpret_cast<uint64_t*>(a.out + off_val);
  for (uint64_t i = tid; i < nvec; i += kThreads)
    if (off_val + 8 * (i + 1) <= a.capacity) dst[i] = ld_agent(src + i);
  for (uint64_t i = nvec * 8 + tid; i < M; i += kThreads)
    if (off_val + i < a.capacity) a.out[off_val + i] = ld_agent(a.val_stage + i);
  for (uint64_t i = 2ull * M + tid; i < a16(2ull * M); i += kThreads)
    if (a.off_pos + i < a.capacity) a.out[a.off_pos + i] = 0;
  if (a.n_tiles == 0 && tid < 4) reinterpret_cast<uint32_t*>(a.out + a.off_tab)[tid] = 0;  // chunk_off[0] + pad
  for (uint32_t i = tid; i < a.n_tiles; i += kThreads) st_agent(&a.state[i], (uint64_t)0);
  if (tid == 0) {
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
      h[10 + i] = a.dec[4 * i] | (a.dec[4 * i + 1] << 8) | (a.dec[4 * i + 2] << 16) | ((uint32_t)a.dec[4 * i + 3] << 24);
    uint4* ho = reinterpret_cast<uint4*>(a.out);
#pragma unroll
    for (int i = 0; i < 4; ++i) ho[i] = make_uint4(h[4 * i], h[4 * i + 1], h[4 * i + 2], h[4 * i + 3]);
    const uint32_t flags = ld_agent(&a.ws_hdr[2]);
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = M;
    a.sizes->status = (total > a.capacity ? SPLITZIP_STATUS_OVERFLOW : 0u) | flags;
    a.sizes->reserved = 0;
    st_agent(&a.ws_hdr[0], 0u);
    st_agent(&a.ws_hdr[1], 0u);
    st_agent(&a.ws_hdr[2], 0u);
  }
}

__global__ __launch_bounds__(kThreads) void compress_bf16_kernel(const CompressArgs a) {
  __shared__ uint16_t lut[256];
  __shared__ uint16_t stage_pos[kWaves][kStageCap];
  __shared__ uint8_t stage_val[kWaves][kStageCap];
  __shared__ uint32_t s_cnt[kWaves * kMaxCpw];
  __shared__ u32x4 s_park[kThreads];
  __shared__ uint32_t s_tile, s_prefix, s_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* park = reinterpret_cast<uint32_t*>(&s_park[tid]);

  lut[tid] = a.lut[tid];
  if (tid < (int)(kWaves * kMaxCpw)) s_cnt[tid] = 0;
  if (tid == 0) s_tile = a.n_tiles ? __hip_atomic_fetch_add(&a.ws_hdr[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
  __syncthreads();
  const uint32_t tile = s_tile;

  if (tile < a.n_tiles) {
    const uint32_t cpw = a.cpw;
    const uint32_t tile_chunk0 = tile * kWaves * cpw;
    const uint32_t wave_chunk0 = tile_chunk0 + wave * cpw;
    const LdsSink lds{stage_pos[wave], stage_val[wave]};
    uint32_t wave_count = 0;
    for (uint32_t c = 0; c < cpw; ++c) {
      const uint32_t chunk = wave_chunk0 + c;
      if (chunk >= a.n_chunks) break;
      const uint64_t cbase = (uint64_t)chunk * kChunk;
      const uint32_t cnt = cbase + kChunk <= a.n
                               ? compress_chunk_bf16<true, true>(a, lut, park, cbase, lane, wave_count, lds)
                               : compress_chunk_bf16<false, true>(a, lut, park, cbase, lane, wave_count, lds);
      if (lane == 0) s_cnt[wave * cpw + c] = cnt;
      wave_count += cnt;
    }
    __syncthreads();

    // exclusive offsets of the tile's chunks (lane q <-> chunk q of the tile) and the tile total
    const uint32_t my = lane < (int)(kWaves * cpw) ? s_cnt[lane] : 0u;
    const uint32_t incl = wave_incl_scan(my);
    const uint32_t tile_tot = wave_last(incl);
    const uint32_t chunk_excl = incl - my;
    if (wave == 0) {
      const uint32_t p = lookback(a.state, tile, tile_tot, lane, &a.ws_hdr[2]);
      if (lane == 0) s_prefix = p;
    }
    __syncthreads();
    const uint32_t tile_prefix = s_prefix;

    if (wave == 0) {
      uint32_t* tab = reinterpret_cast<uint32_t*>(a.out + a.off_tab);
      if (lane < (int)(kWaves * cpw) && tile_chunk0 + lane < a.n_chunks) tab[tile_chunk0 + lane] = tile_prefix + chunk_excl;
      if (tile == a.n_tiles - 1 && lane == 0) {
        // chunk_off[C] = M, then zero padding up to the 16-byte boundary
        tab[a.n_chunks] = tile_prefix + tile_tot;
        for (uint64_t i = a.n_chunks + 1; 4 * i < a16(4ull * (a.n_chunks + 1)); ++i) tab[i] = 0;
      }
    }

    // this wave's escape records go to their final rank
    const uint32_t wave_base = tile_prefix + __shfl(chunk_excl, wave * cpw, 64);
    if (wave_count <= kStageCap) {
      const GlobalSink g{&a};
      for (uint32_t i = lane; i < wave_count; i += 64) g.put(wave_base + i, stage_pos[wave][i], stage_val[wave][i]);
    } else {
      // more escapes than the staging holds: go over this wave's chunks again (their lines are
      // still in cache) and write the records straight to their place
      const GlobalSink g{&a};
      uint32_t r = wave_base;
      for (uint32_t c = 0; c < cpw; ++c) {
        const uint32_t chunk = wave_chunk0 + c;
        if (chunk >= a.n_chunks) break;
        const uint64_t cbase = (uint64_t)chunk * kChunk;
        r += cbase + kChunk <= a.n ? compress_chunk_bf16<true, false>(a, lut, park, cbase, lane, r, g)
                                   : compress_chunk_bf16<false, false>(a, lut, park, cbase, lane, r, g);
      }
    }
  }

  // the last workgroup to get here finishes the stream; every store of escape values has
  // completed (vmcnt) before its workgroup is counted
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0)
    s_last = __hip_atomic_fetch_add(&a.ws_hdr[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1 ? 1u : 0u;
  __syncthreads();
  if (s_last) compress_finalize(a, tid);
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
__device__ void decompress_check_header(const DecompressArgs& a, uint32_t M) {
  const uint32_t* h = reinterpret_cast<const uint32_t*>(a.comp);
  const uint64_t n = h[4] | ((uint64_t)h[5] << 32), m = h[6] | ((uint64_t)h[7] << 32);
  const uint64_t total = h[8] | ((uint64_t)h[9] << 32);
  bool ok = h[0] == 0x31505a53u && h[1] == (1u | (a.dtype << 16) | (4u << 24)) && h[2] == kChunk &&
            h[3] == 0 && n == a.n && m == M && total == a.off_pos + a16(2 * m) + m &&
            total <= a.comp_bytes && h[14] == 0 && h[15] == 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    ok = ok && h[10 + i] == (a.dec[4 * i] | (a.dec[4 * i + 1] << 8) | (a.dec[4 * i + 2] << 16) |
                             ((uint32_t)a.dec[4 * i + 3] << 24));
  if (!ok) flag_bad(a);
  if (a.sizes) {
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = m;
  }
}

// dense decode of one chunk by one wave: two half-chunks, 8 elements per lane each
template <bool FULL>
__device__ inline void decompress_chunk_bf16(const DecompressArgs& a, const uint32_t* tbl, uint64_t cbase, int lane) {
  u32x2 sm[2];
  uint32_t cd[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    sm[h] = u32x2{0u, 0u};
    cd[h] = 0;
    if (FULL || g0 < a16(a.sm_bytes)) sm[h] = ld_stream(reinterpret_cast<const u32x2*>(a.comp + a.off_sm + g0));
    if (FULL || (g0 >> 1) < a16(a.code_bytes))
      cd[h] = ld_stream(reinterpret_cast<const uint32_t*>(a.comp + a.off_code + (g0 >> 1)));
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t g0 = cbase + h * kHalf + lane * 8;
    const uint32_t smw[2] = {sm[h].x, sm[h].y};
    uint32_t o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      // code byte b -> both exponents already in place (bits 7..14 and 23..30)
      const uint32_t cb = (cd[h] >> (8 * b)) & 0xffu;
      // [a0, a0, a1, a1], then keep mantissa in the low and sign in the high byte of each half-word (eq. (2))
      const uint32_t p = byte_perm(0u, smw[b >> 1], (b & 1) ? 0x03030202u : 0x01010000u);
      o[b] = (p & 0x807f807fu) | tbl[cb];
    }
    uint32_t nvalid = 8;
    if (!FULL) nvalid = g0 >= a.n ? 0u : (uint32_t)(a.n - g0 < 8 ? a.n - g0 : 8);
    if (FULL || nvalid == 8) {
      st_stream(reinterpret_cast<u32x4*>(a.out + 2 * g0), u32x4{o[0], o[1], o[2], o[3]});
    } else {
      uint16_t* q = reinterpret_cast<uint16_t*>(a.out) + g0;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if ((uint32_t)(2 * d) < nvalid) q[2 * d] = (uint16_t)o[d];
        if ((uint32_t)(2 * d + 1) < nvalid) q[2 * d + 1] = (uint16_t)(o[d] >> 16);
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void decompress_bf16_kernel(const DecompressArgs a) {
  __shared__ uint32_t tbl[256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  tbl[tid] = ((uint32_t)a.dec[tid & 15] << 7) | ((uint32_t)a.dec[tid >> 4] << 23);

  const uint32_t* tab = reinterpret_cast<const uint32_t*>(a.comp + a.off_tab);
  // M as the offset table states it; escapes are only trusted if their sections lie inside the stream
  uint32_t M = tab[a.n_chunks];
  const uint64_t off_val = a.off_pos + a16(2ull * M);
  const bool esc_ok = M <= a.n && off_val + M <= a.comp_bytes;
  if (blockIdx.x == 0 && tid == 0) {
    decompress_check_header(a, M);
    if (!esc_ok) flag_bad(a);
  }
  if (!esc_ok) M = 0;
  const uint16_t* pos_arr = reinterpret_cast<const uint16_t*>(a.comp + a.off_pos);
  const uint8_t* val_arr = a.comp + off_val;
  __syncthreads();

  const uint32_t cpw = a.cpw;
  const uint32_t wave_chunk0 = (blockIdx.x * kWaves + wave) * cpw;
  for (uint32_t c = 0; c < cpw; ++c) {
    const uint32_t chunk = wave_chunk0 + c;
    if (chunk >= a.n_chunks) break;
    const uint64_t cbase = (uint64_t)chunk * kChunk;
    const uint32_t lo = tab[chunk], hi = tab[chunk + 1];
    if (cbase + kChunk <= a.n)
      decompress_chunk_bf16<true>(a, tbl, cbase, lane);
    else
      decompress_chunk_bf16<false>(a, tbl, cbase, lane);
    // sparse overwrite (the exponent field of x at every recorded position), by the wave that
    // wrote the chunk, once its dense stores have completed
    if (hi == lo) continue;
    const uint32_t clen = (uint32_t)(a.n - cbase < kChunk ? a.n - cbase : kChunk);
    if (hi < lo || hi - lo > clen || hi > M) {
      if (lane == 0) flag_bad(a);
      continue;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (uint32_t j = lo + lane; j < hi; j += 64) {
      const uint32_t pos = pos_arr[j];
      const uint32_t val = val_arr[j];
      if (pos >= clen) {
        flag_bad(a);
        continue;
      }
      const uint32_t sa = a.comp[a.off_sm + cbase + pos];
      reinterpret_cast<uint16_t*>(a.out)[cbase + pos] =
          (uint16_t)(((sa & 0x80u) << 8) | (val << 7) | (sa & 0x7fu));
    }
  }
}

// ---------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------

__global__ void workspace_init_kernel(uint4* p, uint64_t nvec) {
  for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < nvec; i += (uint64_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
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

// most tiles a call of n elements can have (cpw = 1); sizes the look-back state in the workspace
uint64_t max_tiles(uint64_t n) {
  const uint64_t chunks = (n + kChunk - 1) / kChunk;
  return (chunks + kMinTileChunks - 1) / kMinTileChunks;
}

// chunks per wave: the largest power of two (up to `most`) that still leaves `want` tiles per CU
uint32_t pick_cpw(uint64_t n_chunks, uint32_t most, uint32_t want_tiles_per_cu) {
  const uint64_t want = (uint64_t)cu_count() * want_tiles_per_cu;
  uint32_t cpw = most;
  while (cpw > 1 && (n_chunks + (uint64_t)kWaves * cpw - 1) / (kWaves * cpw) < want) cpw >>= 1;
  return cpw;
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
  if (hist_out) memcpy(hist_out, hist, sizeof hist);
  return splitzip_codebook_from_dec(top, dtype, out);
}

size_t splitzip_total_bytes(uint64_t n_elems, uint64_t n_escapes, int dtype) {
  if (!dtype_ok(dtype) || n_elems >> 32) return 0;
  const Layout L = make_layout(n_elems, dtype);
  return (size_t)(L.off_pos + a16(2 * n_escapes) + n_escapes);
}
size_t splitzip_fixed_bytes(uint64_t n_elems, int dtype) { return splitzip_total_bytes(n_elems, 0, dtype); }
size_t splitzip_compress_bound(uint64_t n_elems, int dtype) { return splitzip_total_bytes(n_elems, n_elems, dtype); }

size_t splitzip_workspace_bytes(uint64_t n_elems, int dtype) {
  if (!dtype_ok(dtype) || n_elems >> 32) return 0;
  return (size_t)(kWsHeaderBytes + a256(8 * max_tiles(n_elems)) + a256(n_elems));
}

int splitzip_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!d_workspace || !aligned16(d_workspace) || workspace_bytes < kWsHeaderBytes) return SPLITZIP_ERR_INVALID_ARG;
  // the escape-value staging at the end needs no clearing, but one pass over everything is simplest
  const uint64_t nvec = workspace_bytes / 16;
  const unsigned blocks = (unsigned)((nvec + 255) / 256 < 1024 ? (nvec + 255) / 256 : 1024);
  hipLaunchKernelGGL(workspace_init_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint4*>(d_workspace), nvec);
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
  if (dtype != SPLITZIP_BF16) return SPLITZIP_ERR_UNSUPPORTED;
  if (out_capacity < splitzip_fixed_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
  if (workspace_bytes < splitzip_workspace_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;

  const Layout L = make_layout(n_elems, dtype);
  CompressArgs a;
  memset(&a, 0, sizeof a);
  a.in = static_cast<const uint8_t*>(d_in);
  a.out = static_cast<uint8_t*>(d_out);
  a.n = n_elems;
  a.capacity = out_capacity;
  uint8_t* ws = static_cast<uint8_t*>(d_workspace);
  a.ws_hdr = reinterpret_cast<uint32_t*>(ws);
  a.state = reinterpret_cast<uint64_t*>(ws + kWsHeaderBytes);
  a.val_stage = ws + kWsHeaderBytes + a256(8 * max_tiles(n_elems));
  a.sizes = d_sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  static const int cpw_env = env_int("SPLITZIP_COMPRESS_CPW", 0);
  static const int tiles_per_cu = env_int("SPLITZIP_COMPRESS_TILES_PER_CU", 4);
  a.cpw = cpw_env ? (uint32_t)cpw_env : pick_cpw(L.n_chunks, 8, (uint32_t)tiles_per_cu);
  if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * a.cpw - 1) / (kWaves * a.cpw));
  a.dtype = (uint32_t)dtype;
  memcpy(a.dec, cb->dec, 16);
  for (unsigned v = 0; v < 256; ++v) a.lut[v] = cb->member[v] ? cb->enc[v] : 0x100u;

  const unsigned grid = a.n_tiles ? a.n_tiles : 1u;
  hipLaunchKernelGGL(compress_bf16_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                        const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || !d_comp || (n_elems && !d_out)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_comp) || !aligned16(d_out) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (!codebook_ok(cb, dtype)) return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (dtype != SPLITZIP_BF16) return SPLITZIP_ERR_UNSUPPORTED;
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
  static const int tiles_per_cu = env_int("SPLITZIP_DECOMPRESS_TILES_PER_CU", 8);
  a.cpw = cpw_env ? (uint32_t)cpw_env : pick_cpw(L.n_chunks, 4, (uint32_t)tiles_per_cu);
  if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * a.cpw - 1) / (kWaves * a.cpw));
  a.dtype = (uint32_t)dtype;
  memcpy(a.dec, cb->dec, 16);

  const unsigned grid = a.n_tiles ? a.n_tiles : 1u;
  hipLaunchKernelGGL(decompress_bf16_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
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
