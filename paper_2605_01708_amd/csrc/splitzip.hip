// SplitZip codec for MI355X (gfx950): the C ABI of include/splitzip.h and the host side of its
// kernels.  One translation unit; the kernels live in the headers included below:
//   common.hpp      stream layout, wave scan, agent-scope accesses
//   compress.hpp    dense transform (paper section 3.2 eq. (1), encode table, nibble pack, planes)
//                   fused with escape detection, counting and position-ordered compaction
//                   (appendix "Quad64 Vectorized Encoding" fuses only the counting); one launch
//                   per tensor, or one launch for a batch of tensors
//   decompress.hpp  nibble unpack, decode table, eq. (2), scatter correction in registers; one
//                   launch per tensor or per batch
//   aux_kernels.hpp calibration histogram (section 3.3), workspace initialisation, traffic probe
//   variants.hpp    the formats of the ablations (top-8 / 3-bit codes, top-15 + sentinel, chunk 256,
//                   absolute positions, E4M3) through one plain set of kernels
//
// Work decomposition (wavefront = 64 lanes): a chunk of 1024 elements (the escape-position
// granule) is owned by one wave; every global access of a wave is one fully coalesced run of 16,
// 8 or 4 bytes per lane; all plane traffic uses non-temporal loads and stores, nothing is re-used.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "splitzip.h"

namespace {

#include "common.hpp"
#include "compress.hpp"
#include "decompress.hpp"
#include "aux_kernels.hpp"
#include "variants.hpp"

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

bool dtype_ok(int dtype) { return dtype == SPLITZIP_BF16 || dtype == SPLITZIP_FP8_E5M2; }
unsigned exp_values(int dtype) { return dtype == SPLITZIP_BF16 ? 256u : 32u; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

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
// 32 MiB E5M2 tensors: BF16 wants two chunks per wave from 32 768 chunks in a launch on (with the planes of both
// asked for at once: 23.7 us per 64 MiB tensor against 24.1 us with one) and one below; E5M2 wants four for a
// single tensor and eight for a whole cache in one launch.
uint32_t pick_decompress_cpw(uint64_t n_chunks, int dtype) {
  const uint32_t most = dtype == SPLITZIP_BF16 ? 2 : 8;
  const uint32_t want = dtype == SPLITZIP_BF16 ? 16u : 8u;
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

// What the tests of the rarely taken paths turn: a staging area and a status area smaller than the workspace has
// (tiles whose records do not fit their slots; batches that take several launches), and the number of groups a
// workgroup of the finishing pass takes, which small launches would leave at one, and the bytes of tile counts the
// finishing pass may read directly before it is given sums instead.  Set through
// splitzip_internal_test_hooks (exported, not declared in splitzip.h); zero in normal use.
struct TestHooks {
  std::atomic<uint64_t> stage_bytes{0};
  std::atomic<uint64_t> status_bytes{0};
  std::atomic<uint32_t> finish_groups{0};
  std::atomic<uint64_t> direct_bytes{0};
};
TestHooks g_hooks;

// ---------------------------------------------------------------------------
// format variants: host side
// ---------------------------------------------------------------------------

bool variant_ok(const splitzip_variant* v) {
  if (!v || v->dtype > SPLITZIP_FP8_E4M3) return false;
  if (v->code_bits != 3 && v->code_bits != 4) return false;
  if (v->escape_mode > SPLITZIP_ESC_ABS32) return false;
  const uint32_t codes = 1u << v->code_bits;
  const uint32_t kmax = v->escape_mode == SPLITZIP_ESC_SENTINEL ? codes - 1 : codes;
  if (v->k < 1 || v->k > kmax || v->k > v_exp_values(v->dtype)) return false;
  if (v->escape_mode != SPLITZIP_ESC_ABS32 && v->chunk_elems != 256 && v->chunk_elems != 1024) return false;
  if (v->value_bits != 0 && v->value_bits != 8 && v->value_bits != v_exp_bits(v->dtype)) return false;
  return true;
}

// exactly the first k entries of dec are members, with codes 0 .. k-1
bool variant_codebook_ok(const splitzip_codebook* cb, const splitzip_variant* v) {
  if (!cb || cb->dtype != v->dtype) return false;
  unsigned members = 0;
  for (unsigned e = 0; e < 256; ++e) {
    if (cb->member[e] > 1) return false;
    if (cb->member[e]) {
      if (e >= v_exp_values(v->dtype) || cb->enc[e] >= v->k || cb->dec[cb->enc[e]] != e) return false;
      ++members;
    }
  }
  return members == v->k;
}

// the part of VArgs that follows from (n, variant): layout and chunking
void variant_layout(uint64_t n, const splitzip_variant* v, VArgs* a) {
  memset(a, 0, sizeof *a);
  const bool absolute = v->escape_mode == SPLITZIP_ESC_ABS32;
  a->n = n;
  a->dtype = v->dtype; a->code_bits = v->code_bits; a->k = v->k; a->mode = v->escape_mode;
  a->chunk_shift = absolute || v->chunk_elems == 1024 ? 10 : 8;
  a->pos_bytes = v_pos_bytes(v->escape_mode, v->chunk_elems);
  a->val_bits = v->value_bits ? v->value_bits : 8u;
  a->n_chunks = (n + (1ull << a->chunk_shift) - 1) >> a->chunk_shift;
  a->sm_bytes = (n * v_sm_bits(v->dtype) + 7) / 8;
  a->code_bytes = (n * v->code_bits + 7) / 8;
  a->off_tab = kHeaderBytes;
  a->off_sm = a256(kHeaderBytes + (absolute ? 0 : 4 * (a->n_chunks + 1)));
  a->off_code = a->off_sm + a256(a->sm_bytes);
  a->off_pos = a->off_code + a256(a->code_bytes);
  a->n_tiles = (uint32_t)((a->n_chunks + kVScanTile - 1) / kVScanTile);
  if (a->n_tiles == 0) a->n_tiles = 1;
}

// header words of a stream of this call (M and total, words 6..9, are the kernels' business) and the tables
void variant_tables(const splitzip_variant* v, const splitzip_codebook* cb, VArgs* a) {
  memcpy(a->dec, cb->dec, 16);
  for (uint32_t j = v->k; j < 16; ++j) a->dec[j] = 0;
  a->hdr[0] = 0x31505A53u;   // "SZP1"
  a->hdr[1] = 2u | (a->dtype << 16) | (a->code_bits << 24);
  a->hdr[2] = a->mode == SPLITZIP_ESC_ABS32 ? 0u : 1u << a->chunk_shift;
  a->hdr[3] = a->mode | (a->k << 8) | ((a->val_bits == 8 ? 0u : a->val_bits) << 16);
  a->hdr[4] = (uint32_t)a->n;
  a->hdr[5] = (uint32_t)(a->n >> 32);
  for (int i = 0; i < 4; ++i)
    a->hdr[10 + i] = a->dec[4 * i] | (a->dec[4 * i + 1] << 8) | (a->dec[4 * i + 2] << 16) | ((uint32_t)a->dec[4 * i + 3] << 24);
}

#define SPLITZIP_V_DISPATCH2(KERNEL, grid, block, st, args)                                                        \
  do {                                                                                                             \
    const int key_ = (int)(args).dtype * 2 + ((args).code_bits == 4 ? 1 : 0);                                      \
    switch (key_) {                                                                                                \
      case 0: hipLaunchKernelGGL((KERNEL<SPLITZIP_BF16, 3>), grid, block, 0, st, args); break;                     \
      case 1: hipLaunchKernelGGL((KERNEL<SPLITZIP_BF16, 4>), grid, block, 0, st, args); break;                     \
      case 2: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E5M2, 3>), grid, block, 0, st, args); break;                 \
      case 3: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E5M2, 4>), grid, block, 0, st, args); break;                 \
      case 4: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E4M3, 3>), grid, block, 0, st, args); break;                 \
      default: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E4M3, 4>), grid, block, 0, st, args); break;                \
    }                                                                                                              \
  } while (0)
#define SPLITZIP_V_DISPATCH1(KERNEL, grid, block, st, args)                                                        \
  do {                                                                                                             \
    switch ((args).dtype) {                                                                                        \
      case SPLITZIP_BF16: hipLaunchKernelGGL((KERNEL<SPLITZIP_BF16>), grid, block, 0, st, args); break;            \
      case SPLITZIP_FP8_E5M2: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E5M2>), grid, block, 0, st, args); break;    \
      default: hipLaunchKernelGGL((KERNEL<SPLITZIP_FP8_E4M3>), grid, block, 0, st, args); break;                   \
    }                                                                                                              \
  } while (0)

template <int DT, int CB>
void launch_v_decode(unsigned grid, hipStream_t st, const VArgs& a) {
  const dim3 g(grid), b(kThreads);
  if (a.mode == SPLITZIP_ESC_POS) {
    if (a.chunk_shift == 10) hipLaunchKernelGGL((v_decode_kernel<DT, CB, SPLITZIP_ESC_POS, 10>), g, b, 0, st, a);
    else hipLaunchKernelGGL((v_decode_kernel<DT, CB, SPLITZIP_ESC_POS, 8>), g, b, 0, st, a);
  } else if (a.mode == SPLITZIP_ESC_SENTINEL) {
    if (a.chunk_shift == 10) hipLaunchKernelGGL((v_decode_kernel<DT, CB, SPLITZIP_ESC_SENTINEL, 10>), g, b, 0, st, a);
    else hipLaunchKernelGGL((v_decode_kernel<DT, CB, SPLITZIP_ESC_SENTINEL, 8>), g, b, 0, st, a);
  } else {
    hipLaunchKernelGGL((v_decode_kernel<DT, CB, SPLITZIP_ESC_ABS32, 10>), g, b, 0, st, a);
  }
}

}  // namespace

extern "C" {

int splitzip_version(void) { return 1; }


// ---- format variants ---------------------------------------------------------

int splitzip_variant_supported(const splitzip_variant* v) { return variant_ok(v) ? 1 : 0; }

size_t splitzip_variant_total_bytes(uint64_t n_elems, uint64_t n_escapes, const splitzip_variant* v) {
  if (!variant_ok(v) || (n_elems >> 32)) return 0;
  VArgs a;
  variant_layout(n_elems, v, &a);
  return a.off_pos + a256(a.pos_bytes * n_escapes) + v_val_bytes(n_escapes, a.val_bits);
}

size_t splitzip_variant_compress_bound(uint64_t n_elems, const splitzip_variant* v) {
  return splitzip_variant_total_bytes(n_elems, n_elems, v);
}

size_t splitzip_variant_workspace_bytes(uint64_t n_elems, const splitzip_variant* v) {
  if (!variant_ok(v) || (n_elems >> 32)) return 0;
  VArgs a;
  variant_layout(n_elems, v, &a);
  const uint64_t n_blocks = (n_elems + kVBlock - 1) / kVBlock;
  return a256(4 * a.n_chunks + 4) + a256(4 * (a.n_chunks + 1)) + a256(4 * (uint64_t)a.n_tiles) +
         a256(4ull * kVSlotCap * n_blocks) +         // the blocks' slots of staged escape records
         (a.val_bits == 8 ? 0 : a256(n_elems));   // values narrower than a byte are packed from whole bytes kept here
}

int splitzip_variant_codebook_from_dec(const uint8_t* dec, const splitzip_variant* v, splitzip_codebook* out) {
  if (!dec || !out || !variant_ok(v)) return SPLITZIP_ERR_INVALID_ARG;
  memset(out, 0, sizeof *out);
  out->dtype = v->dtype;
  for (uint32_t j = 0; j < v->k; ++j) {
    if (dec[j] >= v_exp_values(v->dtype) || out->member[dec[j]]) return SPLITZIP_ERR_INVALID_ARG;
    out->dec[j] = dec[j];
    out->enc[dec[j]] = (uint8_t)j;
    out->member[dec[j]] = 1;
  }
  return SPLITZIP_OK;
}

int splitzip_variant_calibrate(const void* h_sample, uint64_t n_elems, const splitzip_variant* v,
                               splitzip_codebook* out, uint64_t* hist_out) {
  if (!out || !variant_ok(v) || (n_elems && !h_sample)) return SPLITZIP_ERR_INVALID_ARG;
  uint64_t hist[256] = {0};
  if (v->dtype == SPLITZIP_BF16) {
    const uint16_t* p = static_cast<const uint16_t*>(h_sample);
    for (uint64_t i = 0; i < n_elems; ++i) hist[(p[i] >> 7) & 0xff]++;
  } else {
    const uint8_t* p = static_cast<const uint8_t*>(h_sample);
    const unsigned shift = v->dtype == SPLITZIP_FP8_E5M2 ? 2 : 3, mask = v->dtype == SPLITZIP_FP8_E5M2 ? 0x1f : 0xf;
    for (uint64_t i = 0; i < n_elems; ++i) hist[(p[i] >> shift) & mask]++;
  }
  if (hist_out) memcpy(hist_out, hist, sizeof hist);
  // the ranking of splitzip_codebook_from_hist, cut at k
  const unsigned nv = v_exp_values(v->dtype);
  uint8_t top[16];
  unsigned filled = 0;
  for (unsigned e = 0; e < nv; ++e) {
    unsigned at = filled;
    while (at > 0 && hist[top[at - 1]] < hist[e]) --at;
    if (at >= 16) continue;
    const unsigned last = filled < 16 ? filled : 15;
    for (unsigned i = last; i > at; --i) top[i] = top[i - 1];
    top[at] = (uint8_t)e;
    if (filled < 16) ++filled;
  }
  return splitzip_variant_codebook_from_dec(top, v, out);
}

int splitzip_variant_compress(const void* d_in, uint64_t n_elems, const splitzip_variant* v,
                              const splitzip_codebook* cb, void* d_out, size_t out_capacity, void* d_workspace,
                              size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream) {
  if (!variant_ok(v) || !variant_codebook_ok(cb, v) || !d_out || !d_sizes || !d_workspace || (n_elems && !d_in))
    return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_workspace) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (out_capacity < splitzip_variant_total_bytes(n_elems, 0, v) ||
      workspace_bytes < splitzip_variant_workspace_bytes(n_elems, v))
    return SPLITZIP_ERR_CAPACITY;

  VArgs a;
  variant_layout(n_elems, v, &a);
  a.in = static_cast<const uint8_t*>(d_in);
  a.out = static_cast<uint8_t*>(d_out);
  a.capacity = out_capacity;
  a.sizes = d_sizes;
  a.counts = static_cast<uint32_t*>(d_workspace);
  uint8_t* ws = static_cast<uint8_t*>(d_workspace);
  a.offs = v->escape_mode == SPLITZIP_ESC_ABS32 ? reinterpret_cast<uint32_t*>(ws + a256(4 * a.n_chunks + 4))
                                                : reinterpret_cast<uint32_t*>(a.out + a.off_tab);
  a.tile_sums = reinterpret_cast<uint32_t*>(ws + a256(4 * a.n_chunks + 4) + a256(4 * (a.n_chunks + 1)));
  const uint64_t blocks = (n_elems + kVBlock - 1) / kVBlock;
  a.slots = reinterpret_cast<uint32_t*>(ws + a256(4 * a.n_chunks + 4) + a256(4 * (a.n_chunks + 1)) + a256(4 * (uint64_t)a.n_tiles));
  a.val_stage = reinterpret_cast<uint8_t*>(a.slots) + a256(4ull * kVSlotCap * blocks);
  variant_tables(v, cb, &a);
  const uint8_t escape = (uint8_t)(0x80u | (v->escape_mode == SPLITZIP_ESC_SENTINEL ? (1u << v->code_bits) - 1u : 0u));
  for (unsigned e = 0; e < 256; ++e) a.lut[e] = cb->member[e] ? cb->enc[e] : escape;

  const hipStream_t st = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)((blocks + kWaves - 1) / kWaves);
  if (grid) SPLITZIP_V_DISPATCH2(v_dense_kernel, dim3(grid), dim3(kThreads), st, a);
  hipLaunchKernelGGL(v_tile_sum_kernel, dim3(a.n_tiles), dim3(1024), 0, st, a);
  const unsigned fgrid = (unsigned)((blocks + kVFinishBlocks - 1) / kVFinishBlocks);
  SPLITZIP_V_DISPATCH1(v_finish_kernel, dim3(fgrid ? fgrid : 1u), dim3(kThreads), st, a);
  if (grid && a.val_bits != 8) {
    // M is known to the device only: a grid that strides over however many bytes the section has
    uint64_t g = (v_val_bytes(n_elems, a.val_bits) + kThreads - 1) / kThreads;
    const uint64_t cap = (uint64_t)cu_count() * 8;
    if (g > cap) g = cap;
    hipLaunchKernelGGL(v_pack_kernel, dim3((unsigned)g), dim3(kThreads), 0, st, a);
  }
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_variant_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, const splitzip_variant* v,
                                const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes, void* stream) {
  if (!variant_ok(v) || !variant_codebook_ok(cb, v) || !d_comp || (n_elems && !d_out)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_comp) || !aligned16(d_out) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (comp_bytes < splitzip_variant_total_bytes(n_elems, 0, v)) return SPLITZIP_ERR_CAPACITY;

  VArgs a;
  variant_layout(n_elems, v, &a);
  a.in = static_cast<const uint8_t*>(d_comp);
  a.out = static_cast<uint8_t*>(d_out);
  a.capacity = comp_bytes;
  a.sizes = d_sizes;
  a.offs = const_cast<uint32_t*>(reinterpret_cast<const uint32_t*>(a.in + a.off_tab));   // read only; unused in the absolute mode
  variant_tables(v, cb, &a);

  const hipStream_t st = static_cast<hipStream_t>(stream);
  const uint64_t blocks = (n_elems + kVBlock - 1) / kVBlock;
  const unsigned grid = blocks ? (unsigned)((blocks + kWaves - 1) / kWaves) : 1u;
  switch ((int)a.dtype * 2 + (a.code_bits == 4 ? 1 : 0)) {
    case 0: launch_v_decode<SPLITZIP_BF16, 3>(grid, st, a); break;
    case 1: launch_v_decode<SPLITZIP_BF16, 4>(grid, st, a); break;
    case 2: launch_v_decode<SPLITZIP_FP8_E5M2, 3>(grid, st, a); break;
    case 3: launch_v_decode<SPLITZIP_FP8_E5M2, 4>(grid, st, a); break;
    case 4: launch_v_decode<SPLITZIP_FP8_E4M3, 3>(grid, st, a); break;
    default: launch_v_decode<SPLITZIP_FP8_E4M3, 4>(grid, st, a); break;
  }
  if (v->escape_mode == SPLITZIP_ESC_ABS32 && n_elems) {
    // M is known to the device only: a grid that strides over whatever the header says
    const uint64_t most = (comp_bytes - a.off_pos) / 5;
    uint64_t g = (most + kThreads - 1) / kThreads;
    const uint64_t cap = (uint64_t)cu_count() * 8;
    if (g > cap) g = cap;
    if (g) SPLITZIP_V_DISPATCH1(v_scatter_kernel, dim3((unsigned)g), dim3(kThreads), st, a);
  }
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

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
  const uint64_t most = (uint64_t)cu_count();   // one workgroup per CU: with two, their 512 final adds per bin cost more than the extra waves bring
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
  return (size_t)(kWsHeaderBytes + kStatusBytes + kStageFloor + a256(n_elems));
}

int splitzip_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!d_workspace || !aligned16(d_workspace) || workspace_bytes < kWsHeaderBytes + kStatusBytes + kStageFloor)
    return SPLITZIP_ERR_INVALID_ARG;
  // No word of a workspace needs a defined value before a call; the header is cleared all the same, so that what
  // a later version of the library may keep there starts from zero.
  hipLaunchKernelGGL(workspace_init_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                     static_cast<uint32_t*>(d_workspace), (uint32_t)(kWsHeaderBytes / 4));
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

void splitzip_internal_test_hooks(uint64_t stage_bytes, uint64_t status_bytes, uint32_t finish_groups, uint64_t direct_bytes) {
  g_hooks.direct_bytes = direct_bytes;
  g_hooks.stage_bytes = stage_bytes;
  g_hooks.status_bytes = status_bytes;
  g_hooks.finish_groups = finish_groups == 1 || finish_groups == 2 || finish_groups == 4 ? finish_groups : 0;
}

}  // extern "C"

namespace {

// table and page geometry of a splitzip_paged as the kernels see them (base left null); false if unusable for
// words of dtype
bool paging_geometry(const splitzip_paged* pg, int dtype, Words* w) {
  if (!pg || !pg->d_block_table || (reinterpret_cast<uintptr_t>(pg->d_block_table) & 3u)) return false;
  const uint64_t es = dtype == SPLITZIP_BF16 ? 2 : 1;
  const uint32_t be = pg->block_elems;
  if (be < kChunk || (be & (be - 1u)) || pg->n_pool_blocks == 0) return false;
  if ((pg->page_stride_bytes & 15u) || (pg->offset_bytes & 15u)) return false;
  if (pg->offset_bytes + (uint64_t)be * es > pg->page_stride_bytes) return false;       // the tensor's part of a page fits the page
  w->base = nullptr;
  w->table = pg->d_block_table;
  w->page_stride = pg->page_stride_bytes;
  w->page_shift = (uint32_t)__builtin_ctz(be);
  w->n_pages = pg->n_pool_blocks;
  return true;
}

// a splitzip_paged as the kernels see it; false if the description is not usable for n_elems words of dtype
bool paged_words(const splitzip_paged* pg, uint64_t n_elems, int dtype, Words* w) {
  if (!paging_geometry(pg, dtype, w) || !pg->d_pool || !aligned16(pg->d_pool)) return false;
  if ((uint64_t)pg->n_blocks * pg->block_elems < n_elems) return false;                   // the table covers the tensor
  w->base = static_cast<uint8_t*>(pg->d_pool) + pg->offset_bytes;
  return true;
}

// ---- the workspace of splitzip_compress_noalloc: one copy per GPU, alive until the process ends ----
// Header, status area and staging area as in a caller's workspace, only smaller.
constexpr uint64_t kScratchStatusBytes = 256u << 10, kScratchStageBytes = 768u << 10;
static __device__ __align__(256) uint32_t scratch[(kWsHeaderBytes + kScratchStatusBytes + kScratchStageBytes) / 4];

// The array's address on the current device (each GPU holds its own copy at its own address), looked up once per
// device with that device current; null if the runtime refuses.  `scratch` itself is a host-side stand-in and is
// never handed to a kernel.
void* scratch_on_current_device() {
  static std::mutex lock;
  static void* ptr[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    ptr[dev] = p;
  }
  return ptr[dev];
}

// a workspace as the compress calls see it: header, then the status words, then the staging of escape values
struct WsView {
  uint8_t* base;
  uint64_t status_bytes, stage_bytes;
};

// the view of a workspace: a caller's (d_workspace non-null: sized by splitzip_workspace_bytes for its largest tensor,
// n_max elements) or the library's own array on the current device; an error code if it is too small or not to be had
int workspace_view(void* d_workspace, size_t workspace_bytes, uint64_t n_max, int dtype, WsView* v) {
  if (d_workspace) {
    if (workspace_bytes < splitzip_workspace_bytes(n_max, dtype)) return SPLITZIP_ERR_CAPACITY;
    v->base = static_cast<uint8_t*>(d_workspace);
    v->status_bytes = kStatusBytes;
    v->stage_bytes = (workspace_bytes - kWsHeaderBytes - kStatusBytes) & ~(uint64_t)255u;
  } else {
    v->base = static_cast<uint8_t*>(scratch_on_current_device());
    if (!v->base) return SPLITZIP_ERR_HIP;
    v->status_bytes = kScratchStatusBytes;
    v->stage_bytes = kScratchStageBytes;
  }
  // tests of the paths that small areas force
  const uint64_t hs = g_hooks.status_bytes, hg = g_hooks.stage_bytes;
  if (hs && hs < v->status_bytes) v->status_bytes = hs;
  if (hg && hg < v->stage_bytes) v->stage_bytes = hg;
  return SPLITZIP_OK;
}

uint64_t chunks_of(uint64_t n) { return (n + kChunk - 1) / kChunk; }
uint64_t tiles_of(uint64_t chunks, uint32_t cpt) { return (chunks + 4ull * cpt - 1) / (4ull * cpt); }
// bytes of the status area a tensor of `tiles` tiles takes: a count per tile, a sum per group of tiles
uint64_t status_need(uint64_t tiles) { return a256(4 * tiles + 4 * ((tiles + kSumGroup - 1) / kSumGroup)); }

// chunks per wave and tile for a tensor of `chunks` chunks: `at_least`, doubled until the tensor's counts fit
// `status_bytes`; 0 if nothing fits
uint32_t pick_cpt(uint64_t chunks, uint32_t at_least, uint64_t status_bytes) {
  for (uint32_t cpt = at_least; cpt <= kMaxRange / 4; cpt *= 2)
    if (status_need(tiles_of(chunks, cpt)) <= status_bytes) return cpt;
  return 0;
}

// The compress calls, all of them: n_items tensors (a host list), each under its own codebook -- the items' own (host)
// or d_cbs[k] (device memory).  paging: table and page geometry shared by all items, or contiguous tensors (table null).
// d_workspace: the caller's workspace, or null with own_scratch for the library's own array.
int compress_launch(const splitzip_item* items, uint32_t n_items, int dtype, const Words& paging, uint64_t paged_room,
                   const splitzip_codebook* d_cbs, void* d_workspace, size_t workspace_bytes, bool own_scratch,
                   splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || (n_items && (!items || !d_sizes)) || (own_scratch ? d_workspace != nullptr : !d_workspace) ||
      !aligned16(d_workspace) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u) || (reinterpret_cast<uintptr_t>(d_cbs) & 3u))
    return SPLITZIP_ERR_INVALID_ARG;
  uint64_t n_max = 0;
  for (uint32_t i = 0; i < n_items; ++i) {
    const splitzip_item& it = items[i];
    if (!it.d_out || (it.n_elems && !it.d_in) || !aligned16(it.d_in) || !aligned16(it.d_out) || (!d_cbs && !codebook_ok(it.cb, dtype)))
      return SPLITZIP_ERR_INVALID_ARG;
    if (it.n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
    if (paging.table && it.n_elems > paged_room) return SPLITZIP_ERR_INVALID_ARG;   // the table does not cover the tensor
    if (it.out_capacity < splitzip_fixed_bytes(it.n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
    if (it.n_elems > n_max) n_max = it.n_elems;
  }
  WsView ws;
  const int rc = workspace_view(d_workspace, workspace_bytes, n_max, dtype, &ws);
  if (rc != SPLITZIP_OK) return rc;
  if (n_items == 0) return SPLITZIP_OK;
  if (!pick_cpt(chunks_of(n_max), 1, ws.status_bytes)) return SPLITZIP_ERR_CAPACITY;
  const uint32_t base_cpt = dtype == SPLITZIP_BF16 ? Bf16::kCpt : E5m2::kCpt;
  const hipStream_t st = static_cast<hipStream_t>(stream);

  uint32_t i = 0;
  while (i < n_items) {
    // one pair of launches: as many of the next tensors (kBatchMax at most) as find room for their counts in the
    // status area; all of them share the tile size of the one that needs the largest
    uint32_t k = 0, cpt = base_cpt;
    for (; i + k < n_items && k < kBatchMax; ++k) {
      const uint32_t need = pick_cpt(chunks_of(items[i + k].n_elems), cpt, ws.status_bytes);
      uint64_t total = 0;
      for (uint32_t q = 0; q <= k && need; ++q) total += status_need(tiles_of(chunks_of(items[i + q].n_elems), need));
      if (!need || total > ws.status_bytes) break;
      cpt = need;
    }
    if (k == 0) return SPLITZIP_ERR_CAPACITY;   // cannot happen: every tensor fits alone
    TileArgs a;
    memset(&a, 0, sizeof a);
    uint64_t off = 0, tiles_max = 0;
    for (uint32_t q = 0; q < k; ++q) {
      const splitzip_item& it = items[i + q];
      if (!d_cbs) memcpy(a.dec[q], it.cb->dec, 16);   // codebook_ok has shown that dec and the encode table describe the same bijection
      a.item[q].in = static_cast<const uint8_t*>(it.d_in);
      a.item[q].out = static_cast<uint8_t*>(it.d_out);
      a.item[q].n = it.n_elems;
      a.item[q].capacity = it.out_capacity;
      const uint64_t tiles = tiles_of(chunks_of(it.n_elems), cpt);
      a.status_off[q] = (uint32_t)off;
      off += status_need(tiles);
      if (tiles > tiles_max) tiles_max = tiles;
    }
    a.sizes = d_sizes + i;
    a.d_cbs = d_cbs ? d_cbs + i : nullptr;
    a.status = ws.base + kWsHeaderBytes;
    a.stage = ws.base + kWsHeaderBytes + ws.status_bytes;
    a.stage_cap = (ws.stage_bytes / k) & ~(uint64_t)255u;
    a.n_items = k;
    a.dtype = (uint32_t)dtype;
    a.cpt = cpt;
    a.tile_shift = 2u + (uint32_t)__builtin_ctz(cpt);
    {
      const uint64_t per_tile = tiles_max ? a.stage_cap / 4 / tiles_max : 0;
      a.slot_cap = (uint32_t)(per_tile < kSlotCapMost ? per_tile : kSlotCapMost);
    }
    a.paging = paging;
    const unsigned groups_max = (unsigned)((tiles_max + kGroup - 1) / kGroup), sums_max = (unsigned)((tiles_max + kSumGroup - 1) / kSumGroup);
    // many groups in the launch: several per workgroup, as long as the chip still gets a few workgroups per CU
    a.finish_groups = 1;
    while (a.finish_groups < kFinishMost && (uint64_t)groups_max * k / (2 * a.finish_groups) >= (uint64_t)cu_count() * 8) a.finish_groups *= 2;
    if (const uint32_t forced = g_hooks.finish_groups.load()) a.finish_groups = forced;
    const unsigned fgroups = (groups_max + a.finish_groups - 1) / a.finish_groups;
    // A finishing workgroup that sums all tile counts of its tensor itself reads 4 bytes per tile: fine while all
    // workgroups of the launch together read no more than kDirectBytes that way, mostly from the L2 (one launch
    // fewer; 64 tensors of 64 MiB: 67 MB of counts read, 1259 us per call against 1262-1292 us with the sums);
    // beyond that they read sums of kSumGroup counts instead (tile_group_sum_kernel).
    const uint64_t direct_budget = g_hooks.direct_bytes.load() ? g_hooks.direct_bytes.load() : kDirectBytes;
    a.use_group_sums = tiles_max > kDirectTiles || (uint64_t)fgroups * k * tiles_max * 4 > direct_budget ? 1u : 0u;
    if (tiles_max) {
      const dim3 grid((unsigned)tiles_max, k);   // one workgroup per tile, started by the hardware in the tiles' order
      if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL((compress_tile_kernel<Bf16, Bf16::kCpt>), grid, dim3(kTileThreads), Bf16::kTileLdsPad, st, a);
      else hipLaunchKernelGGL((compress_tile_kernel<E5m2, E5m2::kCpt>), grid, dim3(kTileThreads), E5m2::kTileLdsPad, st, a);
      if (a.use_group_sums) hipLaunchKernelGGL(tile_group_sum_kernel, dim3(sums_max, k), dim3(64), 0, st, a);
    }
    const dim3 fgrid(fgroups ? fgroups : 1u, k);
    if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL(compress_finish_kernel<Bf16>, fgrid, dim3(kTileThreads), 0, st, a);
    else hipLaunchKernelGGL(compress_finish_kernel<E5m2>, fgrid, dim3(kTileThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
    i += k;
  }
  return SPLITZIP_OK;
}

// one tensor through compress_launch: the codebook on the host (cb) or in device memory (d_cb)
int compress_one(const Words& in, uint64_t n_elems, int dtype, const splitzip_codebook* cb, const splitzip_codebook* d_cb,
                 void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes, bool own_scratch,
                 splitzip_sizes* d_sizes, void* stream) {
  if (!d_sizes || (!cb && !d_cb)) return SPLITZIP_ERR_INVALID_ARG;
  splitzip_item it;
  it.d_in = in.base;
  it.n_elems = n_elems;
  it.d_out = d_out;
  it.out_capacity = out_capacity;
  it.cb = cb;
  return compress_launch(&it, 1, dtype, in, in.table ? n_elems : 0, d_cb, d_workspace, workspace_bytes, own_scratch, d_sizes, stream);
}

// splitzip_decompress with the codebook either on the host (cb) or in device memory (d_cb); the words contiguous or paged
int decompress_impl(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                    const splitzip_codebook* d_cb, const Words& out, splitzip_sizes* d_sizes, void* stream) {
  const void* d_out = out.base;
  if (!dtype_ok(dtype) || !d_comp || (n_elems && !d_out)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_comp) || !aligned16(d_out) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (d_cb ? (reinterpret_cast<uintptr_t>(d_cb) & 3u) != 0 : !codebook_ok(cb, dtype)) return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (comp_bytes < splitzip_fixed_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;

  const Layout L = make_layout(n_elems, dtype);
  DecompressArgs a;
  memset(&a, 0, sizeof a);
  a.comp = static_cast<const uint8_t*>(d_comp);
  a.w = out;
  a.n = n_elems;
  a.comp_bytes = comp_bytes;
  a.sizes = d_sizes;
  a.off_tab = L.off_tab; a.off_sm = L.off_sm; a.off_code = L.off_code; a.off_pos = L.off_pos;
  a.sm_bytes = L.sm_bytes; a.code_bytes = L.code_bytes;
  a.cpw = pick_decompress_cpw(L.n_chunks, dtype);
  a.reg_patch_max = kRegPatchDefault;
  a.n_chunks = (uint32_t)L.n_chunks;
  a.n_tiles = (uint32_t)((L.n_chunks + (uint64_t)kWaves * a.cpw - 1) / (kWaves * a.cpw));
  a.dtype = (uint32_t)dtype;
  a.d_dec = d_cb ? d_cb->dec : nullptr;   // an address in device memory, not read here
  if (!d_cb) memcpy(a.dec, cb->dec, 16);

  const unsigned grid = a.n_tiles ? a.n_tiles : 1u;
  if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL(decompress_kernel<DBf16>, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  else hipLaunchKernelGGL(decompress_kernel<DE5m2>, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

}  // namespace

extern "C" {

int splitzip_compress(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                      void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                      splitzip_sizes* d_sizes, void* stream) {
  return compress_one(contiguous_words(d_in), n_elems, dtype, cb, nullptr, d_out, out_capacity, d_workspace, workspace_bytes, false, d_sizes, stream);
}

uint64_t splitzip_noalloc_max_elems(void) { return 1ull << 30; }

int splitzip_compress_noalloc(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb, void* d_out,
                              size_t out_capacity, splitzip_sizes* d_sizes, void* stream) {
  if (n_elems > splitzip_noalloc_max_elems()) return SPLITZIP_ERR_UNSUPPORTED;
  return compress_one(contiguous_words(d_in), n_elems, dtype, cb, nullptr, d_out, out_capacity, nullptr, 0, true, d_sizes, stream);
}

int splitzip_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                        const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes, void* stream) {
  return decompress_impl(d_comp, comp_bytes, n_elems, dtype, cb, nullptr, contiguous_words(d_out), d_sizes, stream);
}

int splitzip_codebook_device(const uint64_t* d_hist, int dtype, splitzip_codebook* d_cb, void* stream) {
  if (!dtype_ok(dtype) || !d_hist || !d_cb || (reinterpret_cast<uintptr_t>(d_hist) & 7u) || (reinterpret_cast<uintptr_t>(d_cb) & 3u))
    return SPLITZIP_ERR_INVALID_ARG;
  hipLaunchKernelGGL(codebook_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), d_hist, exp_values(dtype),
                     (uint32_t)dtype, d_cb);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_compress_paged(const splitzip_paged* src, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                            void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                            splitzip_sizes* d_sizes, void* stream) {
  Words w;
  if (!dtype_ok(dtype) || !paged_words(src, n_elems, dtype, &w)) return SPLITZIP_ERR_INVALID_ARG;
  return compress_one(w, n_elems, dtype, cb, nullptr, d_out, out_capacity, d_workspace, workspace_bytes, false, d_sizes, stream);
}

int splitzip_decompress_paged(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                              const splitzip_codebook* cb, const splitzip_paged* dst, splitzip_sizes* d_sizes,
                              void* stream) {
  Words w;
  if (!dtype_ok(dtype) || !paged_words(dst, n_elems, dtype, &w)) return SPLITZIP_ERR_INVALID_ARG;
  return decompress_impl(d_comp, comp_bytes, n_elems, dtype, cb, nullptr, w, d_sizes, stream);
}

int splitzip_compress_dcb(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* d_cb,
                          void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                          splitzip_sizes* d_sizes, void* stream) {
  if (!d_cb) return SPLITZIP_ERR_INVALID_ARG;
  return compress_one(contiguous_words(d_in), n_elems, dtype, nullptr, d_cb, d_out, out_capacity, d_workspace, workspace_bytes, false, d_sizes, stream);
}

int splitzip_decompress_dcb(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                            const splitzip_codebook* d_cb, void* d_out, splitzip_sizes* d_sizes, void* stream) {
  if (!d_cb) return SPLITZIP_ERR_INVALID_ARG;
  return decompress_impl(d_comp, comp_bytes, n_elems, dtype, nullptr, d_cb, contiguous_words(d_out), d_sizes, stream);
}

int splitzip_decompress_own(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype, void* d_out,
                            splitzip_sizes* d_sizes, void* stream) {
  if (!d_comp) return SPLITZIP_ERR_INVALID_ARG;
  // the header's 16 decode entries are where a splitzip_codebook keeps its own: the stream serves as one
  static_assert(offsetof(splitzip_codebook, dec) == 0, "dec first");
  const splitzip_codebook* own = reinterpret_cast<const splitzip_codebook*>(static_cast<const uint8_t*>(d_comp) + kHeaderDecOffset);
  return decompress_impl(d_comp, comp_bytes, n_elems, dtype, nullptr, own, contiguous_words(d_out), d_sizes, stream);
}

}  // extern "C"

namespace {

// the batch decompress calls; paging: table and page geometry shared by all items, or contiguous tensors (table null)
// d_cbs (nullable): n_items codebooks in device memory, used instead of the items' own
int decompress_batch_impl(const splitzip_ditem* items, uint32_t n_items, int dtype, const Words& paging, uint64_t paged_room,
                          const splitzip_codebook* d_cbs, bool own_dec, splitzip_sizes* d_sizes, void* stream) {
  if (!dtype_ok(dtype) || (n_items && !items) || (reinterpret_cast<uintptr_t>(d_sizes) & 7u) || (reinterpret_cast<uintptr_t>(d_cbs) & 3u))
    return SPLITZIP_ERR_INVALID_ARG;
  for (uint32_t i = 0; i < n_items; ++i) {
    const splitzip_ditem& it = items[i];
    if (!it.d_comp || (it.n_elems && !it.d_out) || !aligned16(it.d_comp) || !aligned16(it.d_out) ||
        (!d_cbs && !own_dec && !codebook_ok(it.cb, dtype)))
      return SPLITZIP_ERR_INVALID_ARG;
    if (it.n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
    if (paging.table && it.n_elems > paged_room) return SPLITZIP_ERR_INVALID_ARG;
    if (it.comp_bytes < splitzip_fixed_bytes(it.n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
  }
  uint32_t i = 0;
  while (i < n_items) {
    DecompressBatchArgs a;
    memset(&a, 0, sizeof a);
    uint32_t k = 0;
    uint64_t chunks_all = 0, chunks_max = 0;
    for (; i + k < n_items && k < kBatchMax; ++k) {
      const splitzip_ditem& it = items[i + k];
      if (!d_cbs && !own_dec) memcpy(a.dec[k], it.cb->dec, 16);
      a.item[k].comp = static_cast<const uint8_t*>(it.d_comp);
      a.item[k].out = static_cast<uint8_t*>(it.d_out);
      a.item[k].n = it.n_elems;
      a.item[k].comp_bytes = it.comp_bytes;
      const uint64_t c = (it.n_elems + kChunk - 1) / kChunk;
      chunks_all += c;
      if (c > chunks_max) chunks_max = c;
    }
    a.sizes = d_sizes;
    a.d_cbs = d_cbs ? d_cbs + i : nullptr;
    a.own_dec = own_dec ? 1u : 0u;
    a.dtype = (uint32_t)dtype;
    a.paging = paging;
    a.cpw = pick_decompress_cpw(chunks_all, dtype);
    a.reg_patch_max = kRegPatchDefault;
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

}  // namespace

extern "C" {

int splitzip_compress_batch(const splitzip_item* items, uint32_t n_items, int dtype, void* d_workspace,
                            size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream) {
  return compress_launch(items, n_items, dtype, contiguous_words(nullptr), 0, nullptr, d_workspace, workspace_bytes, false, d_sizes, stream);
}

int splitzip_decompress_batch(const splitzip_ditem* items, uint32_t n_items, int dtype, splitzip_sizes* d_sizes,
                              void* stream) {
  return decompress_batch_impl(items, n_items, dtype, contiguous_words(nullptr), 0, nullptr, false, d_sizes, stream);
}

int splitzip_calibrate_batch_device(const splitzip_item* items, uint32_t n_items, int dtype, uint64_t* d_hists,
                                    splitzip_codebook* d_cbs, void* stream) {
  if (!dtype_ok(dtype) || (n_items && (!items || !d_hists || !d_cbs)) || (reinterpret_cast<uintptr_t>(d_hists) & 7u) ||
      (reinterpret_cast<uintptr_t>(d_cbs) & 3u))
    return SPLITZIP_ERR_INVALID_ARG;
  for (uint32_t i = 0; i < n_items; ++i) {
    if ((items[i].n_elems && !items[i].d_in) || !aligned16(items[i].d_in)) return SPLITZIP_ERR_INVALID_ARG;
    if (items[i].n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  }
  if (n_items == 0) return SPLITZIP_OK;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(zero_words_kernel, dim3(64), dim3(256), 0, st, d_hists, 256ull * n_items);
  for (uint32_t i = 0; i < n_items; i += 64) {
    HistBatchArgs a;
    memset(&a, 0, sizeof a);
    const uint32_t k = n_items - i < 64 ? n_items - i : 64;
    uint64_t nvec_max = 1;
    for (uint32_t q = 0; q < k; ++q) {
      a.in[q] = static_cast<const uint8_t*>(items[i + q].d_in);
      a.n[q] = items[i + q].n_elems;
      const uint64_t nvec = (a.n[q] * (dtype == SPLITZIP_BF16 ? 2 : 1) + 15) / 16;
      if (nvec > nvec_max) nvec_max = nvec;
    }
    // workgroups per sample: at least sixteen vectors per thread, and about four workgroups per CU over the launch
    uint64_t gx = (nvec_max + 16 * 1024 - 1) / (16 * 1024);
    const uint64_t most = ((uint64_t)cu_count() * 4 + k - 1) / k;
    if (gx > most) gx = most;
    if (gx < 1) gx = 1;
    if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL(histogram_batch_kernel<true>, dim3((unsigned)gx, k), dim3(1024), 0, st, a, d_hists + 256ull * i);
    else hipLaunchKernelGGL(histogram_batch_kernel<false>, dim3((unsigned)gx, k), dim3(1024), 0, st, a, d_hists + 256ull * i);
  }
  hipLaunchKernelGGL(codebook_kernel, dim3(n_items), dim3(256), 0, st, d_hists, exp_values(dtype), (uint32_t)dtype, d_cbs);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

int splitzip_compress_batch_dcb(const splitzip_item* items, uint32_t n_items, int dtype, const splitzip_codebook* d_cbs,
                                void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream) {
  if (n_items && !d_cbs) return SPLITZIP_ERR_INVALID_ARG;
  return compress_launch(items, n_items, dtype, contiguous_words(nullptr), 0, d_cbs, d_workspace, workspace_bytes, false, d_sizes, stream);
}

int splitzip_decompress_batch_dcb(const splitzip_ditem* items, uint32_t n_items, int dtype, const splitzip_codebook* d_cbs,
                                  splitzip_sizes* d_sizes, void* stream) {
  if (n_items && !d_cbs) return SPLITZIP_ERR_INVALID_ARG;
  return decompress_batch_impl(items, n_items, dtype, contiguous_words(nullptr), 0, d_cbs, false, d_sizes, stream);
}

int splitzip_decompress_batch_own(const splitzip_ditem* items, uint32_t n_items, int dtype, splitzip_sizes* d_sizes,
                                  void* stream) {
  return decompress_batch_impl(items, n_items, dtype, contiguous_words(nullptr), 0, nullptr, true, d_sizes, stream);
}

int splitzip_compress_batch_paged(const splitzip_item* items, uint32_t n_items, int dtype, const splitzip_paged* paging,
                                  void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream) {
  Words w;
  if (!dtype_ok(dtype) || !paging_geometry(paging, dtype, &w)) return SPLITZIP_ERR_INVALID_ARG;
  return compress_launch(items, n_items, dtype, w, (uint64_t)paging->n_blocks * paging->block_elems, nullptr, d_workspace,
                        workspace_bytes, false, d_sizes, stream);
}

int splitzip_decompress_batch_paged(const splitzip_ditem* items, uint32_t n_items, int dtype, const splitzip_paged* paging,
                                    splitzip_sizes* d_sizes, void* stream) {
  Words w;
  if (!dtype_ok(dtype) || !paging_geometry(paging, dtype, &w)) return SPLITZIP_ERR_INVALID_ARG;
  return decompress_batch_impl(items, n_items, dtype, w, (uint64_t)paging->n_blocks * paging->block_elems, nullptr, false, d_sizes, stream);
}

int splitzip_traffic_probe(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes, void* stream) {
  if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || write_bytes > read_bytes)
    return SPLITZIP_ERR_INVALID_ARG;
  const uint64_t nread = read_bytes / 16, nwrite = write_bytes / 16;
  if (!nread) return SPLITZIP_OK;
  uint64_t grid = (uint64_t)cu_count() * 8;
  const uint64_t need = (nread + 4 * kThreads - 1) / (4 * kThreads);
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(traffic_probe_kernel, dim3((unsigned)grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(d_src), nread, static_cast<u32x4*>(d_dst), nwrite);
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}


int splitzip_traffic_probe_shape(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes, uint32_t reads_per_step,
                                 uint32_t writes_per_step, uint32_t wgs_per_cu, uint32_t flags, void* stream) {
  if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || wgs_per_cu > 32 || flags > 63u || (flags & 12u) == 8u || ((flags & 16u) && (flags & 12u)))
    return SPLITZIP_ERR_INVALID_ARG;
  const uint32_t R = reads_per_step, W = writes_per_step;
  const uint64_t nread = R ? read_bytes / 16 : 0, nwrite = W ? write_bytes / 16 : 0;
  const uint64_t rs = R ? (nread + (uint64_t)R * kThreads - 1) / ((uint64_t)R * kThreads) : 0;
  const uint64_t wsteps = W ? (nwrite + (uint64_t)W * kThreads - 1) / ((uint64_t)W * kThreads) : 0;
  const uint64_t steps = rs > wsteps ? rs : wsteps;
  if (!steps) return R || W ? SPLITZIP_OK : SPLITZIP_ERR_INVALID_ARG;
  uint64_t grid = wgs_per_cu ? (uint64_t)cu_count() * wgs_per_cu : steps;   // 0: one step per workgroup
  if (grid > steps) grid = steps;
  if (grid >> 31) return SPLITZIP_ERR_UNSUPPORTED;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  const u32x4* src = static_cast<const u32x4*>(d_src);
  u32x4* dst = static_cast<u32x4*>(d_dst);
  const uint32_t blocked = ((flags & 16u) ? 3u : (flags & 4u) ? ((flags & 8u) ? 2u : 1u) : 0u) | ((flags & 32u) ? 4u : 0u);
  bool found = false;
#define SPLITZIP_SHAPE(RR, WW)                                                                                              \
  if (R == RR && W == WW) {                                                                                                 \
    found = true;                                                                                                           \
    switch (flags & 3u) {                                                                                                   \
      case 0: hipLaunchKernelGGL((traffic_shape_kernel<RR, WW, false, false>), dim3((unsigned)grid), dim3(kThreads), 0, st, src, nread, dst, nwrite, steps, blocked); break; \
      case 1: hipLaunchKernelGGL((traffic_shape_kernel<RR, WW, true, false>), dim3((unsigned)grid), dim3(kThreads), 0, st, src, nread, dst, nwrite, steps, blocked); break;  \
      case 2: hipLaunchKernelGGL((traffic_shape_kernel<RR, WW, false, true>), dim3((unsigned)grid), dim3(kThreads), 0, st, src, nread, dst, nwrite, steps, blocked); break;  \
      default: hipLaunchKernelGGL((traffic_shape_kernel<RR, WW, true, true>), dim3((unsigned)grid), dim3(kThreads), 0, st, src, nread, dst, nwrite, steps, blocked); break;  \
    }                                                                                                                       \
  }
  SPLITZIP_SHAPE(1, 0) SPLITZIP_SHAPE(2, 0) SPLITZIP_SHAPE(4, 0) SPLITZIP_SHAPE(8, 0)
  SPLITZIP_SHAPE(0, 1) SPLITZIP_SHAPE(0, 2) SPLITZIP_SHAPE(0, 4) SPLITZIP_SHAPE(0, 8)
  SPLITZIP_SHAPE(4, 3) SPLITZIP_SHAPE(8, 6) SPLITZIP_SHAPE(16, 12) SPLITZIP_SHAPE(3, 4) SPLITZIP_SHAPE(6, 8) SPLITZIP_SHAPE(12, 16)
  SPLITZIP_SHAPE(1, 1) SPLITZIP_SHAPE(2, 2) SPLITZIP_SHAPE(4, 4)
#undef SPLITZIP_SHAPE
  if (!found) return SPLITZIP_ERR_INVALID_ARG;
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

}  // extern "C"
