// SplitZip codec for MI355X (gfx950): HIP kernels and the C ABI of include/splitzip.h.
//
// One compress call is ONE kernel launch: the dense transform (paper section
// 3.2 eq. (1), encode table, nibble pack, sign+mantissa plane) is fused with
// escape detection, per-chunk counting and the position-ordered compaction of
// the escape stream.  The cross-workgroup offsets of the compaction come from
// a decoupled look-back scan over per-tile escape counts, so the input is read
// exactly once and the output does not depend on scheduling.
// One decompress call is ONE kernel launch as well: nibble unpack, decode
// table, eq. (2), and the sparse overwrite done by the wave that owns the
// chunk, after its own dense stores.
//
// Work decomposition (wavefront = 64 lanes, workgroup = 4 waves):
//   tile  = 8 chunks = 8192 elements, one per workgroup iteration
//   chunk = 1024 elements, owned by one wave; lane l owns elements
//           [16 l, 16 l + 16) of the chunk: two 128-bit loads, one 128-bit
//           sign+mantissa store and one 64-bit code store per lane and chunk.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "splitzip.h"

namespace {

constexpr uint32_t kChunk = 1024;
constexpr uint32_t kHeaderBytes = 64;
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kCPW = 2;                                   // chunks per wave per tile
constexpr uint32_t kTileChunks = kWaves * kCPW;           // 8
constexpr uint32_t kTileElems = kTileChunks * kChunk;     // 8192
constexpr uint32_t kLaneElems = 16;                       // elements per lane per chunk (BF16)
constexpr uint32_t kWsHeaderBytes = 64;                   // ticket, done, flags
constexpr uint32_t kSpinLimit = 1u << 22;                 // look-back polls before giving up

__host__ __device__ inline uint64_t a16(uint64_t x) { return (x + 15u) & ~(uint64_t)15u; }
__host__ __device__ inline uint64_t a256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

struct Layout {
  uint64_t n, n_chunks, n_tiles, sm_bytes, code_bytes;
  uint64_t off_tab, off_sm, off_code, off_pos;  // the value section starts at off_pos + a16(2M)
};

__host__ __device__ inline Layout make_layout(uint64_t n, int dtype) {
  Layout L;
  L.n = n;
  L.n_chunks = (n + kChunk - 1) / kChunk;
  L.n_tiles = (n + kTileElems - 1) / kTileElems;
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

// v_perm_b32: result byte i = byte sel[i] of the 8-byte pool {hi:4..7, lo:0..3}; 0x0c gives 0x00.
__device__ inline uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
  return __builtin_amdgcn_perm(hi, lo, sel);
}

__device__ inline uint32_t wave_incl_scan(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

__device__ inline uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// tile state of the decoupled look-back scan: flag in the two top bits, count below
constexpr uint64_t kFlagAgg = 1ull << 62;   // value = escapes of this tile only
constexpr uint64_t kFlagInc = 2ull << 62;   // value = escapes of all tiles up to and including this one

__device__ inline void st_state(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint64_t ld_state(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Run by one whole wave.  Publishes this tile's escape count, sums the counts
// of all earlier tiles (64 predecessors per poll) and publishes the inclusive
// total.  Flag and count share one 64-bit word, so relaxed accesses suffice.
// Every tile a wave waits for was handed out earlier by the ticket counter and
// publishes its count without waiting for anyone, so the wait always ends; the
// poll limit only guards against a workspace that was never initialised.
__device__ inline uint32_t lookback(uint64_t* state, uint32_t tile, uint32_t agg, int lane,
                                    uint32_t* ws_flags) {
  if (tile == 0) {
    if (lane == 0) st_state(&state[0], kFlagInc | agg);
    return 0;
  }
  if (lane == 0) st_state(&state[tile], kFlagAgg | agg);
  uint32_t prefix = 0;
  int64_t base = (int64_t)tile - 1;
  uint32_t spins = 0;
  for (;;) {
    const int64_t idx = base - lane;
    const uint64_t s = idx >= 0 ? ld_state(&state[idx]) : kFlagInc;  // before tile 0: inclusive 0
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
      __builtin_amdgcn_s_sleep(2);
      continue;
    }
    prefix += wave_sum(lane <= first_inc ? (uint32_t)s : 0u);
    if (first_inc < 64) break;
    base -= 64;
  }
  if (lane == 0) st_state(&state[tile], kFlagInc | (uint64_t)(prefix + agg));
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
  uint32_t n_chunks, n_tiles, dtype, pad;
  uint8_t dec[16];
  uint16_t lut[256];     // exponent -> code | (non-member ? 0x100 : 0)   (the "marked" table of appendix A)
};

// Dense transform of one lane's 16 BF16 elements (eight dwords w).
//   sm   : 16 sign+mantissa bytes, a = ((x >> 8) & 0x80) | (x & 0x7f)        (eq. (1))
//   code : 16 nibbles, element j in nibble j
//   F    : 16 nibbles, nibble j = 1 if element j is an escape
__device__ inline void encode16_bf16(const uint32_t (&w)[8], const uint16_t* lut, uint4& sm,
                                     uint2& code, uint2& F) {
  uint32_t t[8], u[8];
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    // bytes 0 and 2 of t hold a of the low / high half-word
    t[d] = (w[d] & 0x007f007fu) | ((w[d] >> 8) & 0x00800080u);
    const uint32_t e0 = (w[d] >> 7) & 0xffu, e1 = (w[d] >> 23) & 0xffu;
    // low byte: code pair; high byte: flag pair in the same nibble layout
    u[d] = (uint32_t)lut[e0] + ((uint32_t)lut[e1] << 4);
  }
  sm.x = byte_perm(t[1], t[0], 0x06040200u);
  sm.y = byte_perm(t[3], t[2], 0x06040200u);
  sm.z = byte_perm(t[5], t[4], 0x06040200u);
  sm.w = byte_perm(t[7], t[6], 0x06040200u);
  // x = [code(u_lo), code(u_hi), flag(u_lo), flag(u_hi)]
  const uint32_t x01 = byte_perm(u[1], u[0], 0x05010400u), x23 = byte_perm(u[3], u[2], 0x05010400u);
  const uint32_t x45 = byte_perm(u[5], u[4], 0x05010400u), x67 = byte_perm(u[7], u[6], 0x05010400u);
  code.x = byte_perm(x23, x01, 0x05040100u);
  code.y = byte_perm(x67, x45, 0x05040100u);
  F.x = byte_perm(x23, x01, 0x07060302u);
  F.y = byte_perm(x67, x45, 0x07060302u);
}

template <bool FULL>
__device__ inline void compress_lane_chunk_bf16(const CompressArgs& a, const uint16_t* lut,
                                                uint64_t e0, uint2& F) {
  uint32_t w[8];
  uint32_t nvalid = kLaneElems;
  if (!FULL) nvalid = e0 >= a.n ? 0u : (uint32_t)(a.n - e0 < kLaneElems ? a.n - e0 : kLaneElems);
  if (FULL || nvalid == kLaneElems) {
    const uint4* p = reinterpret_cast<const uint4*>(a.in + 2 * e0);
    const uint4 v0 = p[0], v1 = p[1];
    w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w;
    w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
  } else {
    const uint16_t* p = reinterpret_cast<const uint16_t*>(a.in) + e0;
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      const uint32_t lo = (uint32_t)(2 * d) < nvalid ? p[2 * d] : 0u;
      const uint32_t hi = (uint32_t)(2 * d + 1) < nvalid ? p[2 * d + 1] : 0u;
      w[d] = lo | (hi << 16);
    }
  }
  uint4 sm;
  uint2 code;
  encode16_bf16(w, lut, sm, code, F);
  if (!FULL && nvalid < kLaneElems) {
    // elements past N contribute zero nibbles (their sm bytes are already 0)
    const uint64_t keep = nvalid ? (~0ull >> (64 - 4 * nvalid)) : 0ull;
    code.x &= (uint32_t)keep; code.y &= (uint32_t)(keep >> 32);
    F.x &= (uint32_t)keep; F.y &= (uint32_t)(keep >> 32);
  }
  // Sections are padded to 16 bytes and a lane's group never straddles the
  // padded end, so whole-vector stores also write the zero padding.
  if (FULL || e0 < a16(a.sm_bytes)) *reinterpret_cast<uint4*>(a.out + a.off_sm + e0) = sm;
  if (FULL || (e0 >> 1) < a16(a.code_bytes)) *reinterpret_cast<uint2*>(a.out + a.off_code + (e0 >> 1)) = code;
}

// Last workgroup to finish: M is known now.  Moves the staged escape values
// behind the position array, writes pads, header and sizes, and leaves the
// workspace zeroed for the next call.
__device__ void compress_finalize(const CompressArgs& a, int tid) {
  const uint32_t M = a.n_tiles ? (uint32_t)ld_state(&a.state[a.n_tiles - 1]) : 0u;
  const uint64_t off_val = a.off_pos + a16(2ull * M);
  const uint64_t total = off_val + M;
  const uint64_t nvec = M / 16;
  const uint4* src = reinterpret_cast<const uint4*>(a.val_stage);
  uint4* dst = reinterpret_cast<uint4*>(a.out + off_val);
  for (uint64_t i = tid; i < nvec; i += kThreads)
    if (off_val + 16 * (i + 1) <= a.capacity) dst[i] = src[i];
  for (uint64_t i = nvec * 16 + tid; i < M; i += kThreads)
    if (off_val + i < a.capacity) a.out[off_val + i] = a.val_stage[i];
  for (uint64_t i = 2ull * M + tid; i < a16(2ull * M); i += kThreads)
    if (a.off_pos + i < a.capacity) a.out[a.off_pos + i] = 0;
  if (a.n_tiles == 0 && tid < 4) reinterpret_cast<uint32_t*>(a.out + a.off_tab)[tid] = 0;  // chunk_off[0] + pad
  for (uint32_t i = tid; i < a.n_tiles; i += kThreads) st_state(&a.state[i], 0);
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
    const uint32_t flags = a.ws_hdr[2];
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = M;
    a.sizes->status = (total > a.capacity ? SPLITZIP_STATUS_OVERFLOW : 0u) | flags;
    a.sizes->reserved = 0;
    a.ws_hdr[0] = 0;
    a.ws_hdr[1] = 0;
    a.ws_hdr[2] = 0;
  }
}

__global__ __launch_bounds__(kThreads) void compress_bf16_kernel(const CompressArgs a) {
  __shared__ uint16_t lut[256];
  __shared__ uint32_t s_cnt[kTileChunks];
  __shared__ uint32_t s_next, s_prefix, s_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  lut[tid] = a.lut[tid];
  if (tid == 0) s_next = atomicAdd(&a.ws_hdr[0], 1u);
  __syncthreads();
  uint32_t tile = s_next;

  while (tile < a.n_tiles) {
    // ticket of the next tile: asked for now, needed at the end of this iteration
    uint32_t ticket = 0;
    if (tid == 0) ticket = atomicAdd(&a.ws_hdr[0], 1u);

    const uint64_t tile_e0 = (uint64_t)tile * kTileElems;
    const uint32_t chunk0 = tile * kTileChunks + wave * kCPW;   // first chunk of this wave
    const bool full = tile_e0 + kTileElems <= a.n;
    uint2 F[kCPW];
    if (full) {
#pragma unroll
      for (int k = 0; k < kCPW; ++k)
        compress_lane_chunk_bf16<true>(a, lut, (uint64_t)(chunk0 + k) * kChunk + lane * kLaneElems, F[k]);
    } else {
#pragma unroll
      for (int k = 0; k < kCPW; ++k)
        compress_lane_chunk_bf16<false>(a, lut, (uint64_t)(chunk0 + k) * kChunk + lane * kLaneElems, F[k]);
    }

    // escapes per lane and chunk, both chunks scanned at once (16 bits each: a chunk has <= 1024)
    uint32_t cnt[kCPW], packed = 0;
#pragma unroll
    for (int k = 0; k < kCPW; ++k) {
      cnt[k] = __popc(F[k].x) + __popc(F[k].y);
      packed |= cnt[k] << (16 * k);
    }
    const uint32_t incl = wave_incl_scan(packed, lane);
    const uint32_t wave_tot = __shfl(incl, 63, 64);
    const uint32_t excl = incl - packed;
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < kCPW; ++k) s_cnt[wave * kCPW + k] = (wave_tot >> (16 * k)) & 0xffffu;
    }
    __syncthreads();

    // escapes of the chunks before this wave's first chunk, and of the whole tile
    uint32_t before = 0, tile_tot = 0;
#pragma unroll
    for (int q = 0; q < (int)kTileChunks; ++q) {
      const uint32_t c = s_cnt[q];
      if (q < wave * kCPW) before += c;
      tile_tot += c;
    }
    if (wave == 0) {
      const uint32_t p = lookback(a.state, tile, tile_tot, lane, &a.ws_hdr[2]);
      if (lane == 0) {
        s_prefix = p;
        s_next = ticket;
      }
    }
    __syncthreads();
    const uint32_t tile_prefix = s_prefix;
    const uint32_t next_tile = s_next;

    // chunk offsets
    uint32_t* tab = reinterpret_cast<uint32_t*>(a.out + a.off_tab);
    uint32_t chunk_prefix[kCPW];
    {
      uint32_t run = tile_prefix + before;
#pragma unroll
      for (int k = 0; k < kCPW; ++k) {
        chunk_prefix[k] = run;
        if (lane == 0 && chunk0 + k < a.n_chunks) tab[chunk0 + k] = run;
        run += (wave_tot >> (16 * k)) & 0xffffu;
      }
    }
    if (tile == a.n_tiles - 1 && tid == 0) {
      // chunk_off[C] = M, then zero padding up to the 16-byte boundary
      tab[a.n_chunks] = tile_prefix + tile_tot;
      for (uint64_t i = a.n_chunks + 1; 4 * i < a16(4ull * (a.n_chunks + 1)); ++i) tab[i] = 0;
    }

    // escape records, in element order: lanes ascending, elements ascending inside a lane
    uint16_t* pos_arr = reinterpret_cast<uint16_t*>(a.out + a.off_pos);
#pragma unroll
    for (int k = 0; k < kCPW; ++k) {
      if (cnt[k]) {
        uint64_t m = (uint64_t)F[k].x | ((uint64_t)F[k].y << 32);
        uint32_t rank = chunk_prefix[k] + ((excl >> (16 * k)) & 0xffffu);
        const uint64_t cbase = (uint64_t)(chunk0 + k) * kChunk;
        while (m) {
          const uint32_t j = (uint32_t)(__ffsll((unsigned long long)m) - 1) >> 2;
          m &= m - 1;
          const uint32_t pos = lane * kLaneElems + j;
          const uint32_t x = reinterpret_cast<const uint16_t*>(a.in)[cbase + pos];
          if (a.off_pos + 2ull * (rank + 1) <= a.capacity) pos_arr[rank] = (uint16_t)pos;
          a.val_stage[rank] = (uint8_t)((x >> 7) & 0xffu);
          ++rank;
        }
      }
    }
    tile = next_tile;
  }

  // the last workgroup to get here finishes the stream
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    s_last = atomicAdd(&a.ws_hdr[1], 1u) == gridDim.x - 1 ? 1u : 0u;
  }
  __syncthreads();
  if (s_last) {
    __threadfence();
    compress_finalize(a, tid);
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
  uint32_t n_chunks, n_tiles, dtype, pad;
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

template <bool FULL>
__device__ inline void decompress_lane_chunk_bf16(const DecompressArgs& a, const uint32_t* tbl,
                                                  uint64_t e0) {
  uint4 sm = make_uint4(0, 0, 0, 0);
  uint2 cd = make_uint2(0, 0);
  if (FULL || e0 < a16(a.sm_bytes)) sm = *reinterpret_cast<const uint4*>(a.comp + a.off_sm + e0);
  if (FULL || (e0 >> 1) < a16(a.code_bytes)) cd = *reinterpret_cast<const uint2*>(a.comp + a.off_code + (e0 >> 1));
  const uint32_t smw[4] = {sm.x, sm.y, sm.z, sm.w};
  const uint32_t cw[2] = {cd.x, cd.y};
  uint32_t o[8];
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    // code byte b -> both exponents already in place (bits 7..14 and 23..30)
    const uint32_t cb = (cw[b >> 2] >> (8 * (b & 3))) & 0xffu;
    // [a0, a0, a1, a1], then keep mantissa in the low and sign in the high byte of each half-word (eq. (2))
    const uint32_t p = byte_perm(0u, smw[b >> 1], (b & 1) ? 0x03030202u : 0x01010000u);
    o[b] = (p & 0x807f807fu) | tbl[cb];
  }
  uint32_t nvalid = kLaneElems;
  if (!FULL) nvalid = e0 >= a.n ? 0u : (uint32_t)(a.n - e0 < kLaneElems ? a.n - e0 : kLaneElems);
  if (FULL || nvalid == kLaneElems) {
    uint4* q = reinterpret_cast<uint4*>(a.out + 2 * e0);
    q[0] = make_uint4(o[0], o[1], o[2], o[3]);
    q[1] = make_uint4(o[4], o[5], o[6], o[7]);
  } else {
    uint16_t* q = reinterpret_cast<uint16_t*>(a.out) + e0;
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      if ((uint32_t)(2 * d) < nvalid) q[2 * d] = (uint16_t)o[d];
      if ((uint32_t)(2 * d + 1) < nvalid) q[2 * d + 1] = (uint16_t)(o[d] >> 16);
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

  for (uint32_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
    const uint64_t tile_e0 = (uint64_t)tile * kTileElems;
    const uint32_t chunk0 = tile * kTileChunks + wave * kCPW;
    const bool full = tile_e0 + kTileElems <= a.n;
    uint32_t lo[kCPW], hi[kCPW];
#pragma unroll
    for (int k = 0; k < kCPW; ++k) {
      lo[k] = hi[k] = 0;
      if (chunk0 + k < a.n_chunks) {
        lo[k] = tab[chunk0 + k];
        hi[k] = tab[chunk0 + k + 1];
      }
    }
    if (full) {
#pragma unroll
      for (int k = 0; k < kCPW; ++k)
        decompress_lane_chunk_bf16<true>(a, tbl, (uint64_t)(chunk0 + k) * kChunk + lane * kLaneElems);
    } else {
#pragma unroll
      for (int k = 0; k < kCPW; ++k)
        decompress_lane_chunk_bf16<false>(a, tbl, (uint64_t)(chunk0 + k) * kChunk + lane * kLaneElems);
    }
    // sparse overwrite (the exponent field of x at every recorded position), by the wave that
    // wrote the chunk, once its dense stores have completed
#pragma unroll
    for (int k = 0; k < kCPW; ++k) {
      if (hi[k] == lo[k]) continue;
      const uint64_t cbase = (uint64_t)(chunk0 + k) * kChunk;
      const uint32_t clen = (uint32_t)(a.n - cbase < kChunk ? a.n - cbase : kChunk);
      if (hi[k] < lo[k] || hi[k] - lo[k] > clen || hi[k] > M) {
        if (lane == 0) flag_bad(a);
        continue;
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      for (uint32_t j = lo[k] + lane; j < hi[k]; j += 64) {
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
}

// ---------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------

__global__ void workspace_init_kernel(uint4* p, uint64_t nvec) {
  for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < nvec; i += (uint64_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}

// reads 64 bytes, writes 48 bytes per thread and step when the sizes are in the codec's 4:3 ratio
__global__ __launch_bounds__(kThreads) void traffic_probe_kernel(const uint4* src, uint64_t nread,
                                                                  uint4* dst, uint64_t nwrite) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  const uint64_t groups = (nread + 3) / 4;
  for (uint64_t g = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; g < groups; g += stride) {
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = 4 * g + i < nread ? src[4 * g + i] : make_uint4(0, 0, 0, 0);
    v[0].x ^= v[3].x; v[1].y ^= v[3].y; v[2].z ^= v[3].z; v[0].w ^= v[3].w;
#pragma unroll
    for (int i = 0; i < 3; ++i)
      if (3 * g + i < nwrite) dst[3 * g + i] = v[i];
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
  const Layout L = make_layout(n_elems, dtype);
  return (size_t)(kWsHeaderBytes + a256(8 * L.n_tiles) + a256(n_elems));
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
  a.val_stage = ws + kWsHeaderBytes + a256(8 * L.n_tiles);
  a.sizes = d_sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  a.n_chunks = (uint32_t)L.n_chunks; a.n_tiles = (uint32_t)L.n_tiles; a.dtype = (uint32_t)dtype;
  memcpy(a.dec, cb->dec, 16);
  for (unsigned v = 0; v < 256; ++v) a.lut[v] = cb->member[v] ? cb->enc[v] : 0x100u;

  static const int wgs_per_cu = env_int("SPLITZIP_COMPRESS_WGS_PER_CU", 4);
  uint64_t grid = (uint64_t)cu_count() * wgs_per_cu;
  if (grid > L.n_tiles) grid = L.n_tiles;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(compress_bf16_kernel, dim3((unsigned)grid), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), a);
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
  a.n_chunks = (uint32_t)L.n_chunks; a.n_tiles = (uint32_t)L.n_tiles; a.dtype = (uint32_t)dtype;
  memcpy(a.dec, cb->dec, 16);

  static const int wgs_per_cu = env_int("SPLITZIP_DECOMPRESS_WGS_PER_CU", 8);
  uint64_t grid = (uint64_t)cu_count() * wgs_per_cu;
  if (grid > L.n_tiles) grid = L.n_tiles;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(decompress_bf16_kernel, dim3((unsigned)grid), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_traffic_probe(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes, void* stream) {
  if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || write_bytes > read_bytes)
    return SPLITZIP_ERR_INVALID_ARG;
  const uint64_t nread = read_bytes / 16, nwrite = write_bytes / 16;
  if (!nread) return SPLITZIP_OK;
  static const int wgs_per_cu = env_int("SPLITZIP_PROBE_WGS_PER_CU", 8);
  uint64_t grid = (uint64_t)cu_count() * wgs_per_cu;
  const uint64_t need = (nread / 4 + kThreads - 1) / kThreads;
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(traffic_probe_kernel, dim3((unsigned)grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(d_src), nread, static_cast<uint4*>(d_dst), nwrite);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

}  // extern "C"
