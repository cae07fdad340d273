// SplitZip for MI355X: stream layout and small device helpers shared by all kernels.
// Part of the single translation unit splitzip.hip (included inside its anonymous namespace).
#ifndef SPLITZIP_COMMON_HPP
#define SPLITZIP_COMMON_HPP

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kChunk = 1024;
constexpr uint32_t kHalf = 512;
constexpr uint32_t kHeaderBytes = 64;
constexpr uint32_t kHeaderDecOffset = 40;                 // the 16 decode entries inside the header
constexpr int kThreads = 256;                             // decompress / helper kernels
constexpr int kWaves = kThreads / 64;
constexpr uint32_t kMaxCpw = 16;                          // decompress: chunks per wave per tile, at most
constexpr uint32_t kMaxRange = 256;                       // compress: chunks per tile, at most
constexpr uint32_t kWsHeaderBytes = 512;                  // workspace: reserved words in front (cleared by splitzip_workspace_init, read by nobody)
constexpr uint32_t kStatusBytes = 4u << 20;               // workspace: the escape counts of the tiles and their sums
constexpr uint32_t kStageFloor = 64u << 10;               // workspace: the tiles' slots for escape records, at least

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

// Where the words of a tensor live: one contiguous run, or pages of 2^page_shift elements (a multiple of the
// chunk, so a chunk never straddles two pages) found through a table of page indices into a pool.
struct Words {
  uint8_t* base;           // contiguous: the tensor; paged: the pool plus the tensor's offset inside every page
  const uint32_t* table;   // null for a contiguous tensor; else logical page -> index of the page in the pool
  uint64_t page_stride;    // bytes from one page of the pool to the next
  uint32_t page_shift;     // log2 of the elements per page, >= 10
  uint32_t n_pages;        // pages in the pool: indices read from the table are clamped below this
};

__host__ __device__ inline Words contiguous_words(const void* p) {
  Words w;
  w.base = static_cast<uint8_t*>(const_cast<void*>(p));
  w.table = nullptr;
  w.page_stride = 0;
  w.page_shift = 10;
  w.n_pages = 0;
  return w;
}

// the words of one tensor of a batch: its own base, the batch's table and page geometry (none: contiguous)
__host__ __device__ inline Words item_words(const Words& paging, const void* base) {
  Words w = paging;
  w.base = static_cast<uint8_t*>(const_cast<void*>(base));
  return w;
}

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------

// pool page of the chunk with index `chunk` (only for a paged tensor)
__device__ inline uint32_t page_of_chunk(const Words& w, uint64_t chunk) {
  const uint32_t page = w.table[chunk >> (w.page_shift - 10)];
  return page < w.n_pages ? page : w.n_pages - 1;   // a bad table entry never leaves the pool
}

// address of the first element of the chunk that starts at element cbase; `page` is its pool page, read earlier
// with page_of_chunk (ignored for a contiguous tensor)
template <int ES>
__device__ inline uint8_t* chunk_at(const Words& w, uint64_t cbase, uint32_t page) {
  if (!w.table) return w.base + ES * cbase;
  return w.base + (uint64_t)page * w.page_stride + ES * (cbase & ((1ull << w.page_shift) - 1));
}

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

// The 16 decode entries of a codebook as four registers.  Entries that travel in the kernel's arguments are copied
// out of them (dec16_from: the compiler reads kernel arguments with scalar loads); entries in device memory or in
// a stream's header are fetched by one scalar load (load_dec16).  Either way the entries are not behind the
// vector loads in the order of returns, so a table can be built from them while a wave's data loads are still on
// their way (a vector load of the entries would be waited for behind all of those).
__device__ inline u32x4 dec16_from(const uint8_t (&dec)[16]) {
  u32x4 v;
  __builtin_memcpy(&v, dec, 16);
  return v;
}
// dec: an address in device memory (never that of a kernel argument), wave-uniform, 4-byte aligned; the entries
// were written before the launch
__device__ inline u32x4 load_dec16(const uint8_t* dec) {
  const uint64_t p = reinterpret_cast<uint64_t>(dec);
  // (the builtin returns a signed int: without the casts the low half would be sign-extended over the high half)
  const uint32_t p_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  const uint32_t p_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
  const uint64_t sp = ((uint64_t)p_hi << 32) | (uint64_t)p_lo;
  u32x4 v;
  asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(sp) : "memory");
  return v;
}
// entry k (0..15, may differ from lane to lane) of the 16 in v
__device__ inline uint32_t dec16_at(const u32x4& v, uint32_t k) {
  const uint32_t d = k < 8 ? (k < 4 ? v.x : v.y) : (k < 12 ? v.z : v.w);
  return (d >> ((k & 3u) * 8u)) & 0xffu;
}

// Exclusive prefix sum over the lanes of small counts c that are zero in most lanes (escapes per lane), and their
// total (wave-uniform): one ballot per value a count reaches -- set bits below a lane, summed over k, are the
// counts below it.  Three vector instructions per round and usually one round, against a dozen for a full scan.
__device__ inline uint32_t wave_sparse_excl(uint32_t c, uint32_t& excl) {
  uint32_t total = 0;
  excl = 0;
  for (uint32_t k = 1;; ++k) {
    const uint64_t m = __ballot(c >= k);
    if (!m) break;
    excl = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, excl));
    total += (uint32_t)__popcll(m);
  }
  return total;
}

// agent-scope relaxed accesses: performed at the device-wide coherence point, no fences
template <typename T>
__device__ inline void st_agent(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ inline T ld_agent(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

#endif  // SPLITZIP_COMMON_HPP
