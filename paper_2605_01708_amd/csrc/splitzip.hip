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
uint32_t resident_workgroups_batch(int dtype) {
  static uint32_t cached[2][64] = {{0}};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  const int f = dtype == SPLITZIP_BF16 ? 0 : 1;
  if (!cached[f][dev]) {
    int per_cu = 0;
    const hipError_t rc = f == 0 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, compress_batch_kernel<Bf16::kBatchThreads, Bf16>, Bf16::kBatchThreads, 0)
                                 : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, compress_batch_kernel<E5m2::kBatchThreads, E5m2>, E5m2::kBatchThreads, 0);
    if (rc != hipSuccess || per_cu <= 0) return 0;
    cached[f][dev] = (uint32_t)per_cu * (uint32_t)cu_count();
  }
  return cached[f][dev];
}

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
  a->hdr[3] = a->mode | (a->k << 8);
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
  return a.off_pos + a256(a.pos_bytes * n_escapes) + n_escapes;
}

size_t splitzip_variant_compress_bound(uint64_t n_elems, const splitzip_variant* v) {
  return splitzip_variant_total_bytes(n_elems, n_elems, v);
}

size_t splitzip_variant_workspace_bytes(uint64_t n_elems, const splitzip_variant* v) {
  if (!variant_ok(v) || (n_elems >> 32)) return 0;
  VArgs a;
  variant_layout(n_elems, v, &a);
  return a256(4 * a.n_chunks + 4) + a256(4 * (a.n_chunks + 1)) + a256(4 * (uint64_t)a.n_tiles);
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
  variant_tables(v, cb, &a);
  const uint8_t escape = (uint8_t)(0x80u | (v->escape_mode == SPLITZIP_ESC_SENTINEL ? (1u << v->code_bits) - 1u : 0u));
  for (unsigned e = 0; e < 256; ++e) a.lut[e] = cb->member[e] ? cb->enc[e] : escape;

  const hipStream_t st = static_cast<hipStream_t>(stream);
  const uint64_t blocks = (n_elems + kVBlock - 1) / kVBlock;
  const unsigned grid = (unsigned)((blocks + kWaves - 1) / kWaves);
  if (grid) SPLITZIP_V_DISPATCH2(v_dense_kernel, dim3(grid), dim3(kThreads), st, a);
  hipLaunchKernelGGL(v_tile_sum_kernel, dim3(a.n_tiles), dim3(1024), 0, st, a);
  hipLaunchKernelGGL(v_scan_kernel, dim3(a.n_tiles), dim3(1024), 0, st, a);
  if (grid) SPLITZIP_V_DISPATCH1(v_emit_kernel, dim3(grid), dim3(kThreads), st, a);
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

// ---- the exchange words of splitzip_compress_noalloc: one copy per GPU, alive until the process ends ----
// Word 0 is the epoch and starts at 1, everything else at 0: the state splitzip_workspace_init leaves behind.
static __device__ __align__(256) uint32_t scratch[(kWsHeaderBytes + kWsTableBytes) / 4] = {1u};

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

// splitzip_compress with the codebook either on the host (cb) or in device memory (d_cb); the words contiguous or paged
int compress_impl(const Words& in, uint64_t n_elems, int dtype, const splitzip_codebook* cb, const splitzip_codebook* d_cb,
                  void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes,
                  void* stream, bool one_launch = false) {
  const void* d_in = in.base;
  if (!dtype_ok(dtype) || !d_out || !d_workspace || !d_sizes || (n_elems && !d_in)) return SPLITZIP_ERR_INVALID_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_workspace) ||
      (reinterpret_cast<uintptr_t>(d_sizes) & 7u))
    return SPLITZIP_ERR_INVALID_ARG;
  if (d_cb ? (reinterpret_cast<uintptr_t>(d_cb) & 3u) != 0 : !codebook_ok(cb, dtype)) return SPLITZIP_ERR_INVALID_ARG;
  if (n_elems >> 32) return SPLITZIP_ERR_UNSUPPORTED;
  if (out_capacity < splitzip_fixed_bytes(n_elems, dtype)) return SPLITZIP_ERR_CAPACITY;
  // one_launch: the workspace holds the exchange words only (no room to stage the escape values of a call that takes several launches)
  if (workspace_bytes < (one_launch ? kWsHeaderBytes + kWsTableBytes : splitzip_workspace_bytes(n_elems, dtype))) return SPLITZIP_ERR_CAPACITY;

  const Layout L = make_layout(n_elems, dtype);
  CompressArgs a;
  memset(&a, 0, sizeof a);
  a.p = make_planes(in, d_out, n_elems, out_capacity, dtype);
  uint8_t* ws = static_cast<uint8_t*>(d_workspace);
  a.ws_hdr = reinterpret_cast<uint32_t*>(ws);
  a.state = reinterpret_cast<uint64_t*>(ws + kWsHeaderBytes);
  a.val_stage = ws + kWsHeaderBytes + kWsTableBytes;
  a.sizes = d_sizes;
  a.d_cb = d_cb;
  if (!d_cb) {
    memcpy(a.dec, cb->dec, 16);
    for (unsigned v = 0; v < 256; ++v) a.lut[v] = cb->member[v] ? cb->enc[v] : 0x100u;   // indexed by the exponent
  }
  static const int spin_env = env_int("SPLITZIP_SPIN_TICKS", 0);
  a.spin_ticks = spin_env ? (uint64_t)spin_env : kSpinTicks;

  // the grid: every workgroup resident at once, not more workgroups than tiles
  // One workgroup per CU; BF16 with 512 threads, E5M2 with 1024 (swept on 64 and 32 MiB tensors: 256, 512 and 1024
  // threads, one to four workgroups per CU; BF16 does 1.5 % better with eight waves per CU than with sixteen).
  static const int threads_env = env_int("SPLITZIP_COMPRESS_THREADS", 0);
  static const int wgs_per_cu_env = env_int("SPLITZIP_COMPRESS_WGS_PER_CU", 0);
  const int threads = threads_env ? threads_env : (dtype == SPLITZIP_BF16 ? 512 : 1024);
  const int wgs_per_cu = wgs_per_cu_env > 0 ? wgs_per_cu_env : 1;
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
  if (several && one_launch) return SPLITZIP_ERR_UNSUPPORTED;
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
  static const int cpw_env = env_int("SPLITZIP_DECOMPRESS_CPW", 0);
  static const int tiles_per_cu = env_int("SPLITZIP_DECOMPRESS_TILES_PER_CU", 0);
  a.cpw = cpw_env ? (uint32_t)cpw_env : pick_decompress_cpw(L.n_chunks, dtype, tiles_per_cu);
  if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
  static const int reg_patch = env_int("SPLITZIP_DECOMPRESS_REG_PATCH", (int)kRegPatchDefault);
  a.reg_patch_max = (uint32_t)reg_patch;
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
  return compress_impl(contiguous_words(d_in), n_elems, dtype, cb, nullptr, d_out, out_capacity, d_workspace, workspace_bytes, d_sizes, stream);
}

uint64_t splitzip_noalloc_max_elems(void) {
  const uint64_t wgs = (uint64_t)cu_count() < kMaxWorkgroups ? (uint64_t)cu_count() : kMaxWorkgroups;
  return wgs * kMaxRange * kChunk;   // what one launch takes: no staging of escape values is needed below that
}

int splitzip_compress_noalloc(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb, void* d_out,
                              size_t out_capacity, splitzip_sizes* d_sizes, void* stream) {
  if (n_elems > splitzip_noalloc_max_elems()) return SPLITZIP_ERR_UNSUPPORTED;
  void* ws = scratch_on_current_device();
  if (!ws) return SPLITZIP_ERR_HIP;
  // the exchange words are all a call of one launch needs; one that would take several is turned away by the size check
  return compress_impl(contiguous_words(d_in), n_elems, dtype, cb, nullptr, d_out, out_capacity, ws, sizeof(scratch),
                       d_sizes, stream, true);
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
  return compress_impl(w, n_elems, dtype, cb, nullptr, d_out, out_capacity, d_workspace, workspace_bytes, d_sizes, stream);
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
  return compress_impl(contiguous_words(d_in), n_elems, dtype, nullptr, d_cb, d_out, out_capacity, d_workspace, workspace_bytes, d_sizes, stream);
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

// the batch calls; paging: table and page geometry shared by all items, or contiguous tensors (table null)
// d_cbs (nullable): n_items codebooks in device memory, used instead of the items' own
int compress_batch_impl(const splitzip_item* items, uint32_t n_items, int dtype, const Words& paging, uint64_t paged_room,
                        const splitzip_codebook* d_cbs, void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes,
                        void* stream) {
  if (!dtype_ok(dtype) || (n_items && (!items || !d_sizes)) || !d_workspace || !aligned16(d_workspace) ||
      (reinterpret_cast<uintptr_t>(d_sizes) & 7u) || (reinterpret_cast<uintptr_t>(d_cbs) & 3u))
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
  if (workspace_bytes < splitzip_workspace_bytes(n_max, dtype)) return SPLITZIP_ERR_CAPACITY;
  if (n_items == 0) return SPLITZIP_OK;

  static const int wgs_per_cu_env = env_int("SPLITZIP_COMPRESS_WGS_PER_CU", 0);   // 0: what the kernel of the dtype is built for
  const int wgs_per_cu = wgs_per_cu_env > 0 ? wgs_per_cu_env : (dtype == SPLITZIP_BF16 ? Bf16::kBatchWgsPerCu : E5m2::kBatchWgsPerCu);
  const uint32_t resident = resident_workgroups_batch(dtype);
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
      const int rc = compress_impl(item_words(paging, items[i].d_in), items[i].n_elems, dtype, d_cbs ? nullptr : items[i].cb,
                                   d_cbs ? d_cbs + i : nullptr, items[i].d_out, items[i].out_capacity, d_workspace,
                                   workspace_bytes, d_sizes + i, stream);
      if (rc != SPLITZIP_OK) return rc;
      ++i;
      continue;
    }
    // one launch: up to kBatchMax tensors, each with a codebook of its own (its 16 decode entries travel as
    // kernel arguments: codebook_ok has shown that they and the encode table describe the same bijection)
    CompressBatchArgs a;
    memset(&a, 0, sizeof a);
    uint32_t k = 0;
    for (; i + k < n_items && k < kBatchMax; ++k) {
      const splitzip_item& it = items[i + k];
      if ((it.n_elems + kChunk - 1) / kChunk > chunk_cap) break;
      if (!d_cbs) memcpy(a.dec[k], it.cb->dec, 16);
      a.item[k].in = static_cast<const uint8_t*>(it.d_in);
      a.item[k].out = static_cast<uint8_t*>(it.d_out);
      a.item[k].n = it.n_elems;
      a.item[k].capacity = it.out_capacity;
    }
    a.sizes = d_sizes + i;
    a.d_cbs = d_cbs ? d_cbs + i : nullptr;
    a.ws_hdr = reinterpret_cast<uint32_t*>(ws);
    a.state = reinterpret_cast<uint64_t*>(ws + kWsHeaderBytes);
    a.spin_ticks = spin_env ? (uint64_t)spin_env : kSpinTicks;
    a.n_items = k;
    a.dtype = (uint32_t)dtype;
    a.paging = paging;
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
    // A group larger than the kernel fetches exchange words ahead for would put the exchange back on every
    // workgroup's critical path (and have each read that many more words): a smaller grid serves such tensors better.
    const uint32_t kernel_wgs_per_cu = (uint32_t)(dtype == SPLITZIP_BF16 ? Bf16::kBatchWgsPerCu : E5m2::kBatchWgsPerCu);
    const uint32_t ahead = 256u * (kernel_wgs_per_cu < 4u ? kernel_wgs_per_cu : 4u);
    uint32_t Wk = W;
    if (G > ahead && (uint64_t)ahead * kMaxRange >= chunks_max) Wk = G = ahead;
    a.group_wgs = G;
    a.await_extra = (uint32_t)missing;
    const uint32_t grid = (Wk / G) * G;
    if (dtype == SPLITZIP_BF16) hipLaunchKernelGGL((compress_batch_kernel<Bf16::kBatchThreads, Bf16>), dim3(grid), dim3(Bf16::kBatchThreads), 0, st, a);
    else hipLaunchKernelGGL((compress_batch_kernel<E5m2::kBatchThreads, E5m2>), dim3(grid), dim3(E5m2::kBatchThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return SPLITZIP_ERR_HIP;
    i += k;
  }
  return SPLITZIP_OK;
}

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
  static const int cpw_env = env_int("SPLITZIP_DECOMPRESS_CPW", 0);
  static const int tiles_per_cu = env_int("SPLITZIP_DECOMPRESS_TILES_PER_CU", 0);
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
    a.cpw = cpw_env ? (uint32_t)cpw_env : pick_decompress_cpw(chunks_all, dtype, tiles_per_cu);
    if (a.cpw > kMaxCpw) a.cpw = kMaxCpw;
    static const int reg_patch = env_int("SPLITZIP_DECOMPRESS_REG_PATCH", (int)kRegPatchDefault);
    a.reg_patch_max = (uint32_t)reg_patch;
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
  return compress_batch_impl(items, n_items, dtype, contiguous_words(nullptr), 0, nullptr, d_workspace, workspace_bytes, d_sizes, stream);
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
  return compress_batch_impl(items, n_items, dtype, contiguous_words(nullptr), 0, d_cbs, d_workspace, workspace_bytes, d_sizes, stream);
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
  return compress_batch_impl(items, n_items, dtype, w, (uint64_t)paging->n_blocks * paging->block_elems, nullptr, d_workspace,
                             workspace_bytes, d_sizes, stream);
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
  if (!d_src || !d_dst || !aligned16(d_src) || !aligned16(d_dst) || wgs_per_cu > 32 || flags > 15u || (flags & 12u) == 8u)
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
  const uint32_t blocked = (flags & 4u) ? ((flags & 8u) ? 2u : 1u) : 0u;
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
  SPLITZIP_SHAPE(4, 3) SPLITZIP_SHAPE(8, 6) SPLITZIP_SHAPE(3, 4) SPLITZIP_SHAPE(6, 8)
  SPLITZIP_SHAPE(1, 1) SPLITZIP_SHAPE(2, 2) SPLITZIP_SHAPE(4, 4)
#undef SPLITZIP_SHAPE
  if (!found) return SPLITZIP_ERR_INVALID_ARG;
  return hipGetLastError() == hipSuccess ? SPLITZIP_OK : SPLITZIP_ERR_HIP;
}

}  // extern "C"
