// SplitZip for MI355X: the format variants of the paper's ablations (sections "Ablation on Top-k
// Exponent Coding" and "Ablation on Escape-Position Metadata", appendices "Ablation on Chunk Size"
// and "SplitZip on FP8") through one generic set of kernels.  Part of the single translation unit
// splitzip.hip (included inside its anonymous namespace).
//
// These kernels follow the structure of the tuned path: a dense pass that also counts the escapes of every chunk
// and stages the escape records of every block of 1024 elements in a slot of the workspace, sums of the counts,
// and a short finishing pass that ranks the records and moves them to their final place (the paper's own
// structure, appendix "Quad64 Vectorized Encoding", counts in the dense pass and reads the input a second time
// to write the records; the first version of these kernels did that).  They are deliberately plain --
// a block of 1024 elements per wave, eight elements per lane and step, both planes packed as
// LSB-first bit streams of any width and staged through LDS so that global accesses stay whole
// dwords -- because their job is to compare the formats with one another on equal terms, the main
// format included.  The tuned path for the main format is compress.hpp / decompress.hpp.
#ifndef SPLITZIP_VARIANTS_HPP
#define SPLITZIP_VARIANTS_HPP

constexpr uint32_t kVBlock = 1024;   // elements a wave handles at a time
constexpr uint32_t kVStep = 512;     // ... in two steps of 8 elements per lane
constexpr uint32_t kVSlotCap = 128;  // escape records a block's slot holds (one in eight elements: a block with more is encoded again by the finishing pass)

// per-format field arithmetic: e, a and the inverse (eq. (1) and (2); FP8 by analogy)
template <int DT>
struct VFmt;
template <>
struct VFmt<SPLITZIP_BF16> {
  static constexpr int ES = 2, SB = 8, EXPS = 256;
  __device__ static inline uint32_t exponent(uint32_t x) { return (x >> 7) & 0xffu; }
  __device__ static inline uint32_t signmant(uint32_t x) { return ((x >> 8) & 0x80u) | (x & 0x7fu); }
  __device__ static inline uint32_t combine(uint32_t a, uint32_t e) { return ((a & 0x80u) << 8) | (e << 7) | (a & 0x7fu); }
};
template <>
struct VFmt<SPLITZIP_FP8_E5M2> {
  static constexpr int ES = 1, SB = 3, EXPS = 32;
  __device__ static inline uint32_t exponent(uint32_t x) { return (x >> 2) & 0x1fu; }
  __device__ static inline uint32_t signmant(uint32_t x) { return ((x >> 5) & 0x4u) | (x & 0x3u); }
  __device__ static inline uint32_t combine(uint32_t a, uint32_t e) { return ((a & 0x4u) << 5) | (e << 2) | (a & 0x3u); }
};
template <>
struct VFmt<SPLITZIP_FP8_E4M3> {
  static constexpr int ES = 1, SB = 4, EXPS = 16;
  __device__ static inline uint32_t exponent(uint32_t x) { return (x >> 3) & 0xfu; }
  __device__ static inline uint32_t signmant(uint32_t x) { return ((x >> 4) & 0x8u) | (x & 0x7u); }
  __device__ static inline uint32_t combine(uint32_t a, uint32_t e) { return ((a & 0x8u) << 4) | (e << 3) | (a & 0x7u); }
};

__host__ __device__ inline uint32_t v_sm_bits(uint32_t dtype) { return dtype == SPLITZIP_BF16 ? 8u : dtype == SPLITZIP_FP8_E5M2 ? 3u : 4u; }
__host__ __device__ inline uint32_t v_exp_values(uint32_t dtype) { return dtype == SPLITZIP_BF16 ? 256u : dtype == SPLITZIP_FP8_E5M2 ? 32u : 16u; }
__host__ __device__ inline uint32_t v_exp_bits(uint32_t dtype) { return dtype == SPLITZIP_BF16 ? 8u : dtype == SPLITZIP_FP8_E5M2 ? 5u : 4u; }
// bytes of the value section for m escapes of vb bits each
__host__ __device__ inline uint64_t v_val_bytes(uint64_t m, uint32_t vb) { return (m * vb + 7) / 8; }
__host__ __device__ inline uint32_t v_pos_bytes(uint32_t mode, uint32_t chunk) {
  return mode == SPLITZIP_ESC_SENTINEL ? 0u : mode == SPLITZIP_ESC_ABS32 ? 4u : chunk > 256u ? 2u : 1u;
}

// what every variant kernel needs to know about a call
struct VArgs {
  const uint8_t* in;     // compress: the words; decompress: the stream
  uint8_t* out;          // compress: the stream; decompress: the words
  uint64_t capacity;     // bytes of the stream buffer (compress: room, decompress: what the caller holds)
  uint64_t n;
  uint32_t dtype, code_bits, k, mode;
  uint32_t chunk_shift;  // log2 of the chunk the counts are kept for (10 in the absolute mode: the wave's block)
  uint32_t pos_bytes;
  uint32_t val_bits;     // bits per escape value: 8, or the exponent field's own width
  uint8_t* val_stage;    // compress, val_bits < 8: workspace for the values as whole bytes, until v_pack_kernel packs them
  uint64_t n_chunks;     // of that chunk size
  uint64_t sm_bytes, code_bytes;
  uint64_t off_tab, off_sm, off_code, off_pos;
  uint32_t* counts;      // workspace: escapes per chunk
  uint32_t* offs;        // exclusive offsets, n_chunks + 1: in the stream, or in the workspace in the absolute mode
  uint32_t* tile_sums;   // workspace: escapes per tile of kVScanTile chunks
  uint32_t n_tiles;
  uint32_t* slots;       // workspace: per block of 1024 elements kVSlotCap records, position in the block | exponent << 16

  splitzip_sizes* sizes;
  uint32_t hdr[16];      // the header of a stream of this call, words 6..9 (M, total) left 0
  uint8_t dec[16];
  uint8_t lut[256];      // exponent -> code, | 0x80 for an escape
};

// eight elements of a lane: words beyond N read as zero
template <int DT>
__device__ inline void v_load8(const VArgs& a, uint64_t g0, uint32_t (&x)[8]) {
  using F = VFmt<DT>;
  if (g0 + 8 <= a.n) {
    if (F::ES == 2) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(a.in + 2 * g0);
      x[0] = v.x & 0xffffu; x[1] = v.x >> 16; x[2] = v.y & 0xffffu; x[3] = v.y >> 16;
      x[4] = v.z & 0xffffu; x[5] = v.z >> 16; x[6] = v.w & 0xffffu; x[7] = v.w >> 16;
    } else {
      const u32x2 v = *reinterpret_cast<const u32x2*>(a.in + g0);
#pragma unroll
      for (int j = 0; j < 4; ++j) { x[j] = (v.x >> (8 * j)) & 0xffu; x[4 + j] = (v.y >> (8 * j)) & 0xffu; }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      x[j] = 0;
      if (g0 + j < a.n) x[j] = F::ES == 2 ? reinterpret_cast<const uint16_t*>(a.in)[g0 + j] : a.in[g0 + j];
    }
  }
}

// A wave's LDS accesses are carried out in program order; this keeps the compiler from reordering
// accesses it takes for unrelated because they go through different types, and waits for the data.
__device__ inline void v_lds_settle() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// how many of the eight elements starting at g0 exist (the valid ones are always a prefix of the group)
__device__ inline uint32_t v_nvalid(const VArgs& a, uint64_t g0) {
  return g0 >= a.n ? 0u : (a.n - g0 < 8 ? (uint32_t)(a.n - g0) : 8u);
}

// NB bytes of v to / from a lane's slot in LDS (slot = lane * NB; 8 and 4 are aligned)
template <int NB>
__device__ inline void v_lds_put(uint8_t* p, uint64_t v) {
  if (NB == 8) *reinterpret_cast<uint64_t*>(p) = v;
  else if (NB == 4) *reinterpret_cast<uint32_t*>(p) = (uint32_t)v;
  else { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); }
}
template <int NB>
__device__ inline uint64_t v_lds_get(const uint8_t* p) {
  if (NB == 8) return *reinterpret_cast<const uint64_t*>(p);
  if (NB == 4) return *reinterpret_cast<const uint32_t*>(p);
  return (uint64_t)p[0] | ((uint64_t)p[1] << 8) | ((uint64_t)p[2] << 16);
}

// split + encode of a lane's eight elements: packed a, packed codes, escape mask (bit j = element j).  Words beyond
// N were loaded as zero; their codes and escape bits are masked off at the end (no per-element branches).
template <int DT, int CB>
__device__ inline void v_encode8(const VArgs& a, const uint8_t* lut, uint64_t g0, const uint32_t (&x)[8], uint64_t& smw,
                                 uint32_t& cw, uint32_t& esc) {
  using F = VFmt<DT>;
  smw = 0; cw = 0; esc = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t t = lut[F::exponent(x[j])];
    smw |= (uint64_t)F::signmant(x[j]) << (F::SB * j);   // zero for words beyond N
    cw |= (t & 0x7fu) << (CB * j);
    esc |= (t >> 7) << j;
  }
  const uint32_t nv = v_nvalid(a, g0);
  if (nv < 8) {
    cw &= (1u << (CB * nv)) - 1u;
    esc &= (1u << nv) - 1u;
  }
}

// compress pass 1: both planes and the escape count of every chunk
template <int DT, int CB>
__global__ __launch_bounds__(kThreads) void v_dense_kernel(const VArgs a) {
  using F = VFmt<DT>;
  __shared__ uint8_t lut[256];
  __shared__ __attribute__((aligned(16))) uint8_t s_sm[kWaves][64 * F::SB];
  __shared__ __attribute__((aligned(16))) uint8_t s_code[kWaves][64 * CB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  lut[tid] = a.lut[tid];
  __syncthreads();
  const uint64_t blk = (uint64_t)blockIdx.x * kWaves + wave;
  if (blk * kVBlock >= a.n) return;
  uint32_t carry = 0;   // escapes of step 0, for 1024-element chunks
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const uint64_t g = blk * kVBlock + s * kVStep, g0 = g + lane * 8;
    uint32_t x[8];
    v_load8<DT>(a, g0, x);
    uint64_t smw;
    uint32_t cw, esc;
    v_encode8<DT, CB>(a, lut, g0, x, smw, cw, esc);
    v_lds_put<F::SB>(&s_sm[wave][lane * F::SB], smw);
    v_lds_put<CB>(&s_code[wave][lane * CB], cw);
    v_lds_settle();
    // the step's plane bytes leave as whole dwords, up to the padded end of the section
    const uint64_t sm0 = g / 8 * F::SB, code0 = g / 8 * CB;
    for (uint32_t i = lane; i < 16u * F::SB; i += 64)
      if (sm0 + 4 * i < a256(a.sm_bytes))
        st_stream(reinterpret_cast<uint32_t*>(a.out + a.off_sm + sm0) + i, reinterpret_cast<const uint32_t*>(s_sm[wave])[i]);
    if ((uint32_t)lane < 16u * CB && code0 + 4 * lane < a256(a.code_bytes))
      st_stream(reinterpret_cast<uint32_t*>(a.out + a.off_code + code0) + lane, reinterpret_cast<const uint32_t*>(s_code[wave])[lane]);
    v_lds_settle();   // the staging is written again in the next step
    const uint32_t incl = wave_incl_scan(__popc(esc));
    const uint32_t t31 = __builtin_amdgcn_readlane(incl, 31), t63 = __builtin_amdgcn_readlane(incl, 63);
    // the block's escape records, in element order, into its slot
    if (esc) {
      uint32_t r = (s == 0 ? 0u : carry) + incl - __popc(esc);
      uint32_t* slot = a.slots + blk * kVSlotCap;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!((esc >> j) & 1u)) continue;
        if (r < kVSlotCap) slot[r] = (uint32_t)(s * kVStep + lane * 8 + j) | (F::exponent(x[j]) << 16);
        ++r;
      }
    }
    if (a.chunk_shift == 10) {
      if (s == 1 && lane == 0) a.counts[blk] = carry + t63;
    } else if (lane == 0) {   // two 256-element chunks per step
      const uint64_t c0 = g >> 8;
      if (c0 < a.n_chunks) a.counts[c0] = t31;
      if (c0 + 1 < a.n_chunks) a.counts[c0 + 1] = t63 - t31;
    }
    if (s == 0) carry = t63;
  }
}

constexpr uint32_t kVScanTile = 1024;   // counts per workgroup of the two scan kernels

// sum of 1024 values, one per thread, in every thread (two barriers)
__device__ inline uint32_t v_block_sum(uint32_t v, uint32_t* s_wave /*16*/, uint32_t& incl_out, uint32_t& before_out) {
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan(v);
  __syncthreads();   // s_wave may still be read from an earlier call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
  for (uint32_t w = 0; w < 16; ++w) {
    if (w < wave) before += s_wave[w];
    all += s_wave[w];
  }
  incl_out = incl;
  before_out = before;
  return all;
}

// compress pass 2a: the escapes of every tile of 1024 chunks
__global__ __launch_bounds__(1024) void v_tile_sum_kernel(const VArgs a) {
  __shared__ uint32_t s_wave[16];
  const uint64_t c = (uint64_t)blockIdx.x * kVScanTile + threadIdx.x;
  uint32_t incl, before;
  const uint32_t all = v_block_sum(c < a.n_chunks ? a.counts[c] : 0u, s_wave, incl, before);
  if (threadIdx.x == 0) a.tile_sums[blockIdx.x] = all;
}

constexpr uint32_t kVFinishBlocks = 64;   // blocks of 1024 elements per workgroup of the finishing pass

// where record `rank` of the stream goes: its position in the variant's width (none in the sentinel mode) and its
// exponent (as a byte of the stream, or of the workspace if values are narrower than a byte: v_pack_kernel)
__device__ inline void v_put_record(const VArgs& a, uint64_t off_val, uint32_t rank, uint64_t elem, uint32_t e) {
  if (a.mode == SPLITZIP_ESC_POS) {
    const uint32_t p = (uint32_t)elem & ((1u << a.chunk_shift) - 1u);
    const uint64_t at = a.off_pos + (uint64_t)a.pos_bytes * rank;
    if (at + a.pos_bytes <= a.capacity) {
      if (a.pos_bytes == 2) *reinterpret_cast<uint16_t*>(a.out + at) = (uint16_t)p;
      else a.out[at] = (uint8_t)p;
    }
  } else if (a.mode == SPLITZIP_ESC_ABS32) {
    const uint64_t at = a.off_pos + 4ull * rank;
    if (at + 4 <= a.capacity) *reinterpret_cast<uint32_t*>(a.out + at) = (uint32_t)elem;
  }
  if (a.val_bits != 8) a.val_stage[rank] = (uint8_t)e;
  else if (off_val + rank < a.capacity) a.out[off_val + rank] = (uint8_t)e;
}

// compress pass 3: one workgroup per kVFinishBlocks blocks.  It sums the counts (the whole tensor's: M; those before
// its blocks: its first rank), writes its chunks' entries of the offset table, and moves its blocks' records from
// their slots to their ranks; a block with more records than its slot holds is encoded once more from the words.
// Workgroup 0 also writes the header, the sizes record and the zero padding.
template <int DT>
__global__ __launch_bounds__(kThreads) void v_finish_kernel(const VArgs a) {
  using F = VFmt<DT>;
  __shared__ uint8_t lut[256];
  __shared__ uint32_t s_part[3][kWaves];
  __shared__ uint32_t s_bp[kVFinishBlocks + 1];   // escapes of the group's blocks before each block
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = blockIdx.x;
  const uint32_t cpb_shift = 10u - a.chunk_shift;   // log2 of the chunks per block: 0 or 2
  const uint64_t n_blocks = (a.n + kVBlock - 1) / kVBlock;
  const uint64_t blk0 = (uint64_t)g * kVFinishBlocks, c0 = blk0 << cpb_shift;
  lut[tid] = a.lut[tid];
  // escapes before the group's first chunk and in the whole tensor: whole scan tiles by their sums, the rest by chunk
  uint32_t before = 0, all = 0;
  const uint64_t whole = c0 / kVScanTile;
  for (uint32_t t = tid; t < a.n_tiles; t += kThreads) {
    const uint32_t v = a.tile_sums[t];
    all += v;
    before += t < whole ? v : 0u;
  }
  for (uint64_t c = whole * kVScanTile + tid; c < c0 && c < a.n_chunks; c += kThreads) before += a.counts[c];
  // the group's chunks, one per thread (64 or 256 of them)
  const uint64_t my_c = c0 + tid;
  const bool have = tid < (kVFinishBlocks << cpb_shift) && my_c < a.n_chunks;
  const uint32_t mine = have ? a.counts[my_c] : 0u;
  const uint32_t incl = wave_incl_scan(mine);
  before = wave_last(wave_incl_scan(before));
  all = wave_last(wave_incl_scan(all));
  if (lane == 63) {
    s_part[0][wave] = incl;
    s_part[1][wave] = before;
    s_part[2][wave] = all;
  }
  __syncthreads();
  uint32_t first = 0, M = 0, waves_before = 0, group_total = 0;
#pragma unroll
  for (uint32_t w = 0; w < kWaves; ++w) {
    waves_before += w < wave ? s_part[0][w] : 0u;
    group_total += s_part[0][w];
    first += s_part[1][w];
    M += s_part[2][w];
  }
  const uint32_t excl = waves_before + incl - mine;   // escapes of the group before this thread's chunk
  if (have && (tid & ((1u << cpb_shift) - 1u)) == 0) s_bp[tid >> cpb_shift] = excl;
  // blocks behind the tensor's last start where the group ends
  const uint64_t blocks_here = n_blocks > blk0 ? (n_blocks - blk0 < kVFinishBlocks ? n_blocks - blk0 : kVFinishBlocks) : 0;
  if (tid >= blocks_here && tid <= kVFinishBlocks) s_bp[tid] = group_total;
  __syncthreads();
  if (have && a.mode != SPLITZIP_ESC_ABS32) a.offs[my_c] = first + excl;
  const uint64_t off_val = a.off_pos + a256((uint64_t)a.pos_bytes * M);

  // records that wait in their blocks' slots: rank r of the group belongs to the last block that starts at or before r
  for (uint32_t r = tid; r < group_total; r += kThreads) {
    uint32_t b = 0;
#pragma unroll
    for (uint32_t step = kVFinishBlocks / 2; step; step >>= 1)
      if (s_bp[b + step] <= r) b += step;
    if (s_bp[b + 1] - s_bp[b] > kVSlotCap) continue;
    const uint32_t rec = a.slots[(blk0 + b) * kVSlotCap + (r - s_bp[b])];
    v_put_record(a, off_val, first + r, (blk0 + b) * kVBlock + (rec & 0xffffu), rec >> 16);
  }
  // blocks whose records did not fit their slots, a wave each
  for (uint32_t b = wave; b < blocks_here; b += kWaves) {
    if (s_bp[b + 1] - s_bp[b] <= kVSlotCap) continue;
    uint32_t rank = first + s_bp[b];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint64_t g0 = (blk0 + b) * kVBlock + s * kVStep + lane * 8;
      uint32_t x[8];
      v_load8<DT>(a, g0, x);
      uint32_t esc = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) esc |= (uint32_t)(lut[F::exponent(x[j])] >> 7) << j;
      esc &= (1u << v_nvalid(a, g0)) - 1u;
      const uint32_t cnt = __popc(esc), sc = wave_incl_scan(cnt);
      uint32_t r = rank + sc - cnt;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!((esc >> j) & 1u)) continue;
        v_put_record(a, off_val, r, g0 + j, F::exponent(x[j]));
        ++r;
      }
      rank += __builtin_amdgcn_readlane(sc, 63);
    }
  }
  if (g != 0) return;

  if (tid == 0) a.offs[a.n_chunks] = M;   // the table's last entry; in the absolute mode a word of the workspace, for v_pack_kernel
  const uint64_t pos_sec = a256((uint64_t)a.pos_bytes * M), total = a.off_pos + pos_sec + v_val_bytes(M, a.val_bits);
  // zero padding: behind the table, behind what the dense pass covered of each plane, behind the positions
  const uint64_t tab_end = a.mode == SPLITZIP_ESC_ABS32 ? kHeaderBytes : a.off_tab + 4 * (a.n_chunks + 1);
  for (uint64_t i = tab_end + tid; i < a.off_sm; i += kThreads) a.out[i] = 0;
  const uint64_t sm_cov = n_blocks * (kVBlock / 8) * v_sm_bits(a.dtype), code_cov = n_blocks * (kVBlock / 8) * a.code_bits;
  for (uint64_t i = sm_cov + tid; i < a256(a.sm_bytes); i += kThreads) a.out[a.off_sm + i] = 0;
  for (uint64_t i = code_cov + tid; i < a256(a.code_bytes); i += kThreads) a.out[a.off_code + i] = 0;
  for (uint64_t i = (uint64_t)a.pos_bytes * M + tid; i < pos_sec; i += kThreads)
    if (a.off_pos + i < a.capacity) a.out[a.off_pos + i] = 0;
  if (tid < 16) {
    uint32_t w = a.hdr[tid];
    if (tid == 6) w = M;
    if (tid == 8) w = (uint32_t)total;
    if (tid == 9) w = (uint32_t)(total >> 32);
    reinterpret_cast<uint32_t*>(a.out)[tid] = w;
  }
  if (tid == 0) {
    a.sizes->total_bytes = total;
    a.sizes->n_escapes = M;
    a.sizes->status = total > a.capacity ? SPLITZIP_STATUS_OVERFLOW : 0u;
    a.sizes->reserved = 0;
  }
}

// compress pass 4, for values narrower than a byte: the value section as an LSB-first bit stream of val_bits per
// value, from the whole-byte values of the workspace.  Every thread makes whole bytes of the section from the
// values that overlap them, so no two threads write the same byte.
__global__ __launch_bounds__(kThreads) void v_pack_kernel(const VArgs a) {
  const uint32_t M = a.offs[a.n_chunks], vb = a.val_bits;
  const uint64_t off_val = a.off_pos + a256((uint64_t)a.pos_bytes * M), bytes = v_val_bytes(M, vb);
  for (uint64_t b = (uint64_t)blockIdx.x * kThreads + threadIdx.x; b < bytes; b += (uint64_t)gridDim.x * kThreads) {
    uint32_t byte = 0;
    for (uint64_t r = 8 * b / vb; r < M && r * vb < 8 * b + 8; ++r) {
      const int64_t shift = (int64_t)(r * vb) - (int64_t)(8 * b);   // where value r starts, relative to this byte
      const uint32_t v = a.val_stage[r];
      byte |= shift >= 0 ? v << shift : v >> -shift;
    }
    if (off_val + b < a.capacity) a.out[off_val + b] = (uint8_t)byte;
  }
}

// ---- decompress -----------------------------------------------------------------------------

// escape value idx of a stream whose value section starts at off_val (the section is known to lie inside the stream)
__device__ inline uint32_t v_value(const VArgs& a, uint64_t off_val, uint64_t idx) {
  if (a.val_bits == 8) return a.in[off_val + idx];
  const uint64_t bit = idx * a.val_bits;
  const uint32_t sh = (uint32_t)(bit & 7u);
  uint32_t v = a.in[off_val + (bit >> 3)] >> sh;
  if (sh + a.val_bits > 8) v |= (uint32_t)a.in[off_val + (bit >> 3) + 1] << (8 - sh);
  return v & ((1u << a.val_bits) - 1u);
}

// an inconsistent header or record: sticky bit in the caller's sizes record (nullable)
__device__ inline void v_flag_bad(const VArgs& a) {
  if (a.sizes) atomicOr(&a.sizes->status, SPLITZIP_STATUS_BAD_STREAM);
}

// The header as every wave reads it: lane i < 16 holds word i.  Words 6..9 (M, total) are checked against the
// layout, the others against what the call expects.  Wave-uniform result; M through m_out.
__device__ inline bool v_check_header(const VArgs& a, uint32_t hw, int lane, uint32_t* m_out) {
  const bool word_ok = lane >= 16 || (lane >= 6 && lane <= 9) || hw == a.hdr[lane & 15];
  const uint64_t M = __builtin_amdgcn_readlane(hw, 6) | ((uint64_t)__builtin_amdgcn_readlane(hw, 7) << 32);
  const uint64_t total = __builtin_amdgcn_readlane(hw, 8) | ((uint64_t)__builtin_amdgcn_readlane(hw, 9) << 32);
  *m_out = (uint32_t)M;
  return __builtin_amdgcn_ballot_w64(!word_ok) == 0 && M <= a.n &&
         total == a.off_pos + a256(a.pos_bytes * M) + v_val_bytes(M, a.val_bits) && total <= a.capacity;
}

// One block of 1024 elements per wave.  Everything that depends on nothing -- the header, the offsets of the
// block's chunks, the block's slices of both planes -- is fetched at once; the escape records of the chunks
// follow as soon as the offsets are known and travel while the planes are decoded into an LDS tile; the records
// are applied to the tile (in the sentinel mode the exponent of every sentinel is fetched while decoding
// instead), and the tile is stored.  In the absolute mode the correction is left to v_scatter_kernel.
template <int DT, int CB, int MODE, int CS>
__global__ __launch_bounds__(kThreads) void v_decode_kernel(const VArgs a) {
  using F = VFmt<DT>;
  // escape mode, chunk size and position width are compile-time here: none of the format's choices costs a branch
  constexpr uint32_t PB = MODE == SPLITZIP_ESC_POS ? (CS == 10 ? 2u : 1u) : MODE == SPLITZIP_ESC_ABS32 ? 4u : 0u;
  __shared__ uint8_t s_dec[16];
  __shared__ __attribute__((aligned(16))) uint8_t s_sm[kWaves][128 * F::SB];
  __shared__ __attribute__((aligned(16))) uint8_t s_code[kWaves][128 * CB];
  __shared__ __attribute__((aligned(16))) uint8_t s_tile[kWaves][kVBlock * F::ES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 16) s_dec[tid] = (uint32_t)tid < a.k ? a.dec[tid] : 0;
  const uint64_t blk = (uint64_t)blockIdx.x * kWaves + wave;
  const bool live = blk * kVBlock < a.n;
  const uint32_t per_blk = kVBlock >> CS, chunk = 1u << CS;
  const uint64_t c_first = blk * per_blk;

  const uint32_t hw = lane < 16 ? reinterpret_cast<const uint32_t*>(a.in)[lane] : 0u;
  uint32_t my_off = 0;   // lane q holds the offset of chunk c_first + q
  if (live && MODE != SPLITZIP_ESC_ABS32 && (uint32_t)lane <= per_blk && c_first + lane <= a.n_chunks)
    my_off = a.offs[c_first + lane];
  // The block's slices of both planes (whole dwords; the sections are padded, so nothing past them is read) are
  // asked for now and kept in registers: they go to LDS further down, once the escape records -- whose addresses
  // need the offsets and the header, asked for before the planes -- are on their way too.
  constexpr uint32_t SMD = (32u * F::SB + 63u) / 64u, CDD = (32u * CB + 63u) / 64u;   // dwords per lane
  uint32_t psm[SMD], pcd[CDD];
  {
    const uint64_t sm0 = blk * (kVBlock / 8) * F::SB, code0 = blk * (kVBlock / 8) * CB;
#pragma unroll
    for (uint32_t q = 0; q < SMD; ++q) {
      const uint32_t i = lane + 64 * q;
      psm[q] = live && i < 32u * F::SB && sm0 + 4 * i < a256(a.sm_bytes) ? ld_stream(reinterpret_cast<const uint32_t*>(a.in + a.off_sm + sm0) + i) : 0u;
    }
#pragma unroll
    for (uint32_t q = 0; q < CDD; ++q) {
      const uint32_t i = lane + 64 * q;
      pcd[q] = live && i < 32u * CB && code0 + 4 * i < a256(a.code_bytes) ? ld_stream(reinterpret_cast<const uint32_t*>(a.in + a.off_code + code0) + i) : 0u;
    }
  }
  uint32_t M;
  const bool ok = v_check_header(a, hw, lane, &M);
  if (blockIdx.x == 0 && tid == 0) {
    if (a.sizes) {
      a.sizes->total_bytes = __builtin_amdgcn_readlane(hw, 8) | ((uint64_t)__builtin_amdgcn_readlane(hw, 9) << 32);
      a.sizes->n_escapes = M;
    }
    if (!ok) v_flag_bad(a);
  }
  lds_barrier();            // s_dec (an LDS-only barrier: the planes stay on their way)
  if (!ok || !live) return;   // nothing of a stream with a bad header is followed
  const uint64_t off_val = a.off_pos + a256((uint64_t)PB * M);
  const uint32_t sentinel = (1u << CB) - 1u;
  // codes the codebook does not have can only occur if it leaves some unused (wave-uniform: no per-element work otherwise)
  const bool check_codes = a.k + (MODE == SPLITZIP_ESC_SENTINEL ? 1u : 0u) < (1u << CB);
  bool bad = false;

  // chunk-relative records: the first 64 of every chunk of the block are fetched now
  uint32_t rec_p[4] = {0, 0, 0, 0}, rec_e[4] = {0, 0, 0, 0}, rec_lo[4], rec_n[4] = {0, 0, 0, 0};
  if (MODE == SPLITZIP_ESC_POS) {
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      rec_lo[q] = 0;
      if (q >= per_blk || c_first + q >= a.n_chunks) continue;
      const uint32_t lo = __builtin_amdgcn_readlane(my_off, q), hi = __builtin_amdgcn_readlane(my_off, q + 1);
      const uint64_t first = (c_first + q) << CS, len = first + chunk <= a.n ? chunk : a.n - first;
      if (hi < lo || hi - lo > len || hi > M) { bad = true; continue; }
      rec_lo[q] = lo;
      rec_n[q] = hi - lo;
      if ((uint32_t)lane < hi - lo) {
        rec_p[q] = PB == 2 ? reinterpret_cast<const uint16_t*>(a.in + a.off_pos)[lo + lane] : a.in[a.off_pos + lo + lane];
        rec_e[q] = v_value(a, off_val, lo + lane);
      }
    }
  }

  // the planes into LDS now (every lane its dwords), so that each lane can pick its elements' bits
#pragma unroll
  for (uint32_t q = 0; q < SMD; ++q)
    if (lane + 64 * q < 32u * F::SB) reinterpret_cast<uint32_t*>(s_sm[wave])[lane + 64 * q] = psm[q];
#pragma unroll
  for (uint32_t q = 0; q < CDD; ++q)
    if (lane + 64 * q < 32u * CB) reinterpret_cast<uint32_t*>(s_code[wave])[lane + 64 * q] = pcd[q];
  v_lds_settle();
  uint32_t carry = 0;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const uint64_t g = blk * kVBlock + s * kVStep, g0 = g + lane * 8;
    const uint64_t smw = v_lds_get<F::SB>(&s_sm[wave][(s * 64 + lane) * F::SB]);
    const uint32_t cw = (uint32_t)v_lds_get<CB>(&s_code[wave][(s * 64 + lane) * CB]);
    const uint32_t vmask = (1u << v_nvalid(a, g0)) - 1u;   // bit j: element j exists
    uint32_t w[8], sent = 0, unknown = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t av = (uint32_t)(smw >> (F::SB * j)) & ((1u << F::SB) - 1u), code = (cw >> (CB * j)) & sentinel;
      sent |= (uint32_t)(code == sentinel) << j;
      if (check_codes) unknown |= (uint32_t)(code >= a.k) << j;
      w[j] = F::combine(av, s_dec[code & 15u]);
    }
    sent = MODE == SPLITZIP_ESC_SENTINEL ? sent & vmask : 0u;
    if (unknown & vmask & ~sent) bad = true;
    if (MODE == SPLITZIP_ESC_SENTINEL) {
      // rank of every sentinel inside its chunk, then its exponent from the value array
      const uint32_t cnt = __popc(sent), incl = wave_incl_scan(cnt);
      const uint32_t t31 = __builtin_amdgcn_readlane(incl, 31), t63 = __builtin_amdgcn_readlane(incl, 63);
      uint32_t r, r_end;
      if (CS == 10) {
        r = __builtin_amdgcn_readlane(my_off, 0) + carry + incl - cnt;
        r_end = __builtin_amdgcn_readlane(my_off, 1);
        carry = t63;
      } else {
        const uint32_t q = 2 * s + (lane >> 5);   // the chunk of this half-wave, inside the block
        const bool there = c_first + q < a.n_chunks;
        const uint32_t o0 = __builtin_amdgcn_readlane(my_off, 2 * s), o1 = __builtin_amdgcn_readlane(my_off, 2 * s + 1),
                       o2 = __builtin_amdgcn_readlane(my_off, 2 * s + 2);
        r = there ? (lane < 32 ? o0 : o1) + incl - cnt - (lane >= 32 ? t31 : 0u) : 0u;
        r_end = there ? (lane < 32 ? o1 : o2) : 0u;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!((sent >> j) & 1u)) continue;
        uint32_t e = 0;
        if (r < r_end && r < M) e = v_value(a, off_val, r);
        else bad = true;
        if (e >= (uint32_t)F::EXPS) { bad = true; e = 0; }
        const uint32_t av = (uint32_t)(smw >> (F::SB * j)) & ((1u << F::SB) - 1u);
        w[j] = F::combine(av, e);
        ++r;
      }
    }
    if (F::ES == 2)
      *reinterpret_cast<u32x4*>(&s_tile[wave][(s * kVStep + lane * 8) * 2]) =
          u32x4{w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16)};
    else
      *reinterpret_cast<u32x2*>(&s_tile[wave][s * kVStep + lane * 8]) =
          u32x2{w[0] | (w[1] << 8) | (w[2] << 16) | (w[3] << 24), w[4] | (w[5] << 8) | (w[6] << 16) | (w[7] << 24)};
  }

  v_lds_settle();
  if (MODE == SPLITZIP_ESC_POS) {
    // the records of the block's chunks, one lane each, straight into the tile
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
      if (q >= per_blk || rec_n[q] == 0) continue;
      const uint64_t first = (c_first + q) << CS, len = first + chunk <= a.n ? chunk : a.n - first;
      for (uint32_t i = lane; i < rec_n[q]; i += 64) {
        uint32_t p = rec_p[q], e = rec_e[q];
        if (i >= 64) {   // a chunk with more than 64 escapes: the rest is fetched here
          p = PB == 2 ? reinterpret_cast<const uint16_t*>(a.in + a.off_pos)[rec_lo[q] + i] : a.in[a.off_pos + rec_lo[q] + i];
          e = v_value(a, off_val, rec_lo[q] + i);
        }
        // a chunk's positions ascend: the record before this one (the lane below holds it, or memory does)
        uint32_t before = (uint32_t)__shfl_up((int)p, 1);
        if (lane == 0 && i > 0) before = PB == 2 ? reinterpret_cast<const uint16_t*>(a.in + a.off_pos)[rec_lo[q] + i - 1] : a.in[a.off_pos + rec_lo[q] + i - 1];
        if (p >= len || (i > 0 && p <= before) || e >= (uint32_t)F::EXPS) { bad = true; continue; }
        const uint32_t at = q * chunk + p;
        if (F::ES == 2) {
          uint16_t* t = reinterpret_cast<uint16_t*>(s_tile[wave]) + at;
          *t = (uint16_t)F::combine(F::signmant(*t), e);
        } else {
          uint8_t* t = s_tile[wave] + at;
          *t = (uint8_t)F::combine(F::signmant(*t), e);
        }
      }
    }
  }

  v_lds_settle();
  // the tile, 16 bytes per lane and step
  const uint64_t e0 = blk * kVBlock;
  const uint32_t bytes = F::ES * kVBlock;
  if (e0 + kVBlock <= a.n) {
    for (uint32_t i = lane; i < bytes / 16; i += 64)
      st_stream(reinterpret_cast<u32x4*>(a.out + e0 * F::ES) + i, reinterpret_cast<const u32x4*>(s_tile[wave])[i]);
  } else {
    for (uint32_t i = lane; e0 + i < a.n; i += 64) {
      if (F::ES == 2) reinterpret_cast<uint16_t*>(a.out)[e0 + i] = reinterpret_cast<const uint16_t*>(s_tile[wave])[i];
      else a.out[e0 + i] = s_tile[wave][i];
    }
  }
  if (bad) v_flag_bad(a);
}

// absolute mode: every record overwrites the exponent field of its element (runs after v_decode_kernel)
template <int DT>
__global__ __launch_bounds__(kThreads) void v_scatter_kernel(const VArgs a) {
  using F = VFmt<DT>;
  const int lane = threadIdx.x & 63;
  uint32_t M;
  if (!v_check_header(a, lane < 16 ? reinterpret_cast<const uint32_t*>(a.in)[lane] : 0u, lane, &M)) return;
  const uint64_t off_val = a.off_pos + a256(4ull * M);
  bool bad = false;
  for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < M; i += (uint64_t)gridDim.x * kThreads) {
    const uint64_t p = reinterpret_cast<const uint32_t*>(a.in + a.off_pos)[i];
    const uint32_t e = v_value(a, off_val, i);
    // the element indices ascend
    if (p >= a.n || e >= (uint32_t)F::EXPS || (i > 0 && p <= reinterpret_cast<const uint32_t*>(a.in + a.off_pos)[i - 1])) { bad = true; continue; }
    if (F::ES == 2) {
      uint16_t* t = reinterpret_cast<uint16_t*>(a.out) + p;
      *t = (uint16_t)F::combine(F::signmant(*t), e);
    } else {
      a.out[p] = (uint8_t)F::combine(F::signmant(a.out[p]), e);
    }
  }
  if (bad) v_flag_bad(a);
}

#endif  // SPLITZIP_VARIANTS_HPP
