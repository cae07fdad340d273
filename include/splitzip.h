/*
 * splitzip.h -- C ABI of the SplitZip codec for AMD Instinct MI355X (gfx950).
 *
 * SplitZip is a lossless codec for BF16 (and FP8 E5M2) KV-cache tensors
 * (paper section 3, "SplitZip").  Every word is split into a sign+mantissa
 * part that is stored verbatim and an exponent that is mapped through an
 * offline-calibrated table of the 16 most frequent exponents to a 4-bit code,
 * two codes per byte.  Exponents outside the table get a dummy code and are
 * recorded in a sparse escape stream of (chunk-relative 16-bit position, raw
 * exponent) records; the decoder applies them as a scatter correction after
 * the dense unpack / table lookup / recombination.
 *
 * All entry points are plain C: pointers and sizes only.  "d_" pointers are
 * device (HBM) addresses, "h_"/unprefixed pointers are host addresses.  Nothing
 * in this library allocates device memory, synchronises a stream or the
 * device, or reads device memory from the host: device work is enqueued on
 * the caller's stream and results (including sizes) are written by kernels.
 * Calls return 0 (SPLITZIP_OK) or a negative splitzip_error.
 *
 * Compressed stream (little endian; the offset table follows the header, every
 * other section starts 256-byte aligned so that the planes fall on whole cache
 * lines and HBM channel granules; pad bytes are zero; A(x) = x rounded up to
 * 256; C = ceil(N/1024)):
 *
 *   header     64 B        u32 magic "SZP1", u16 version 1, u8 dtype, u8 code
 *                          bits (4), u32 chunk elements (1024), u32 0,
 *                          u64 N, u64 M (escapes), u64 total bytes,
 *                          u8 dec[16], u8 zero[8]
 *   chunk_off  4(C+1) B    u32 exclusive prefix sums of the per-chunk escape
 *                          counts; chunk_off[C] = M
 *   sm plane   BF16: N B, byte i = a_i (eq. (1)).  E5M2: ceil(3N/8) B,
 *              LSB-first bit stream, bit 3i+k = bit k of a_i
 *   code plane ceil(N/2) B, byte j = code[2j] | code[2j+1] << 4
 *   esc_pos    2M B        u16 chunk-relative positions, ascending elements
 *   esc_val    M B         u8 raw exponents, same order
 *
 *   total = A(64 + 4(C+1)) + A(sm) + A(ceil(N/2)) + A(2M) + M
 *
 * The payload (planes + 3M) is the paper's B_SZ = N + N/2 + 3M (section 3.2).
 */
#ifndef SPLITZIP_H
#define SPLITZIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPLITZIP_BF16 = 0,     /* 16-bit words: 1 sign, 8 exponent, 7 mantissa bits */
  SPLITZIP_FP8_E5M2 = 1, /* 8-bit words: 1 sign, 5 exponent, 2 mantissa bits (paper appendix "SplitZip on FP8") */
  SPLITZIP_FP8_E4M3 = 2  /* 8-bit words: 1 sign, 4 exponent, 3 mantissa bits; accepted by the splitzip_variant_* calls only
                            (a 4-bit code cannot shrink a 4-bit exponent, same appendix) */
} splitzip_dtype;

typedef enum {
  SPLITZIP_OK = 0,
  SPLITZIP_ERR_INVALID_ARG = -1, /* null / misaligned pointer, inconsistent codebook, bad dtype */
  SPLITZIP_ERR_UNSUPPORTED = -2, /* n_elems >= 2^32 (offsets are 32-bit) */
  SPLITZIP_ERR_CAPACITY = -3,    /* output / workspace / stream smaller than the fixed part needs */
  SPLITZIP_ERR_HIP = -4          /* a HIP runtime call (kernel launch) failed */
} splitzip_error;

/* bits of splitzip_sizes.status, written by kernels */
enum {
  SPLITZIP_STATUS_OVERFLOW = 1u,   /* compress: escapes did not fit out_capacity; total_bytes is the size needed */
  SPLITZIP_STATUS_BAD_STREAM = 2u, /* decompress: header / offsets / positions inconsistent; offending records skipped */
  SPLITZIP_STATUS_INTERNAL = 4u    /* reserved: no call of this version sets it (earlier versions reported a timed-out
                                      exchange between workgroups here; the kernels no longer wait for one another) */
};

/* The three calibration tables of section 3.3.  Plain data, host memory,
 * caller-owned, copyable.  For E5M2 only indices 0..31 of enc/member are used. */
typedef struct {
  uint8_t dec[16];     /* 4-bit code -> exponent; code k is the k-th most frequent exponent */
  uint8_t enc[256];    /* exponent -> 4-bit code; 0 (the dummy code, section 3.4) for non-members */
  uint8_t member[256]; /* 1 if the exponent is in the codebook (escape detection) */
  uint32_t dtype;      /* splitzip_dtype the tables were built for */
} splitzip_codebook;

typedef struct {
  uint64_t total_bytes; /* size of the whole compressed stream */
  uint64_t n_escapes;   /* M */
  uint32_t status;      /* SPLITZIP_STATUS_* bits, 0 = fine */
  uint32_t reserved;
} splitzip_sizes;

/* Section 3.3 "Calibration": histogram the exponents of a HOST sample of
 * n_elems words, take the 16 most frequent (ties to the smaller exponent;
 * never-seen exponents fill up in ascending order) and build the three
 * tables.  hist_out (nullable) receives the 256 exponent counts.  Host only;
 * touches no GPU. */
int splitzip_calibrate(const void* h_sample, uint64_t n_elems, int dtype, splitzip_codebook* out,
                       uint64_t* hist_out);

/* The same from a histogram of exponent counts (host memory, 256 entries; for
 * E5M2 the first 32 count). */
int splitzip_codebook_from_hist(const uint64_t hist[256], int dtype, splitzip_codebook* out);

/* Section 3.3 with the counting on the device: adds the exponent counts of a
 * DEVICE sample of n_elems words to d_hist (256 device words, 8-byte aligned,
 * zeroed by the caller before the first sample; several calls accumulate a
 * calibration set of several tensors).  Enqueued on `stream`.  The caller
 * copies the 2 KB to the host and calls splitzip_codebook_from_hist.  This is
 * the paper's "dynamic" codebook (ablation "pre-calibration vs. dynamic
 * codebook") when done per call. */
int splitzip_histogram(const void* d_sample, uint64_t n_elems, int dtype, uint64_t* d_hist, void* stream);

/* A codebook that never leaves the device (calibration per call without a
 * host round trip): splitzip_codebook_device ranks 256 device counts exactly
 * as splitzip_codebook_from_hist does and writes the three tables into a
 * splitzip_codebook in DEVICE memory (4-byte aligned); the _dcb calls are
 * splitzip_compress / splitzip_decompress with such a codebook.  The tables
 * are read by the kernels, so they cannot be checked by the host: a codebook
 * that was not written by splitzip_codebook_device gives undefined streams
 * (never out-of-bounds accesses).  All enqueued on `stream`. */
int splitzip_codebook_device(const uint64_t* d_hist, int dtype, splitzip_codebook* d_cb, void* stream);
int splitzip_compress_dcb(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* d_cb,
                          void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                          splitzip_sizes* d_sizes, void* stream);
int splitzip_decompress_dcb(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                            const splitzip_codebook* d_cb, void* d_out, splitzip_sizes* d_sizes, void* stream);

/* Tables for a given list of 16 distinct exponents (code k = dec[k]); used to
 * restore a saved codebook.  INVALID_ARG on duplicates / out-of-range values. */
int splitzip_codebook_from_dec(const uint8_t dec[16], int dtype, splitzip_codebook* out);

/* Stream sizes.  fixed = header + chunk_off + both planes (independent of the
 * data); total adds the escape sections for M escapes; bound = total at M = N.
 * Return 0 for an invalid dtype or n_elems >= 2^32. */
size_t splitzip_fixed_bytes(uint64_t n_elems, int dtype);
size_t splitzip_total_bytes(uint64_t n_elems, uint64_t n_escapes, int dtype);
size_t splitzip_compress_bound(uint64_t n_elems, int dtype);

/* Device scratch of a compress call of up to n_elems: a status area of 4 MiB
 * (the escape count of every 16 KB tile of the tensor) and a staging area of
 * n_elems bytes and a little more (the tiles' escape records until their rank
 * in the stream is known).  A compress call is two kernel launches: the first
 * does the dense work tile by tile, the second ranks and places the escape
 * records; no workgroup ever waits for another, so the calls run correctly
 * whatever else the device is doing and however little of a launch fits the
 * device at a time.  No word of a workspace needs a defined value before a
 * call: splitzip_workspace_init exists for symmetry (it clears a small
 * header) and is cheap.  Calls that share a workspace must not overlap in
 * time (same stream, or otherwise ordered); calls with workspaces of their
 * own may run side by side on different streams.  Decompress calls and the
 * variant calls use no workspace of this kind. */
size_t splitzip_workspace_bytes(uint64_t n_elems, int dtype);
int splitzip_workspace_init(void* d_workspace, size_t workspace_bytes, void* stream);

/* Section 3.2, encoding path (dense split / table / pack fused with escape
 * detection, counting and position-ordered compaction, appendix A) on device
 * buffers, enqueued on `stream` (a hipStream_t; NULL = default stream).
 *   d_in        N words (16-bit for BF16, 8-bit for E5M2), 16-byte aligned, read only
 *   d_out       >= out_capacity bytes, 16-byte aligned (256 for full speed); receives the stream
 *   d_sizes     device (or pinned host) splitzip_sizes, written by the kernel
 * out_capacity below splitzip_fixed_bytes() -> SPLITZIP_ERR_CAPACITY, nothing
 * enqueued.  If the fixed part fits but the escapes do not, everything that
 * fits is written, status gets SPLITZIP_STATUS_OVERFLOW and total_bytes is
 * the size a retry needs.  n_elems == 0 is valid (header and one offset).
 * Two launches on `stream` (three above 32 Mi elements of BF16).
 * The output is a pure function of (input, codebook): independent of
 * scheduling, capacity slack and earlier calls. */
int splitzip_compress(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                      void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                      splitzip_sizes* d_sizes, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc:
 * splitzip_compress without a workspace argument.  Status and staging areas
 * live in an array of 1 MiB inside the library's code object (256 KiB of tile
 * counts, 768 KiB of staged escape records), one copy per GPU, held until the
 * process ends; the call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine).  Same arguments otherwise, same stream bytes
 * and sizes record as splitzip_compress.  Limit: n_elems <=
 * splitzip_noalloc_max_elems() = 2^30; beyond it SPLITZIP_ERR_UNSUPPORTED and
 * nothing is enqueued.  (Tensors above 64 Mi elements get tiles larger than
 * 16 KB so that their counts fit, and a tile whose escape records outgrow its
 * share of the staging area -- a few dozen per tile at 64 MiB of BF16 -- is
 * encoded a second time by the finishing launch: correct at any escape rate,
 * slower above a few percent.)  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU -- different streams, no ordering --
 * race on it; order them, or use splitzip_compress with a workspace per
 * stream. */
uint64_t splitzip_noalloc_max_elems(void);
int splitzip_compress_noalloc(const void* d_in, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                              void* d_out, size_t out_capacity, splitzip_sizes* d_sizes, void* stream);

/* Section 3.2, decoding path: nibble unpack, 16-entry table, recombination by
 * eq. (2), then the sparse overwrite of the exponent field at every recorded
 * escape position.
 *   d_comp      the stream, comp_bytes readable bytes, 16-byte aligned
 *   d_out       n_elems words, 16-byte aligned
 *   d_sizes     nullable.  total_bytes / n_escapes are copied from the header;
 *               status bits are OR-ed into the existing value (sticky), so the
 *               caller zeroes it once and can watch many calls with one word.
 * n_elems and the codebook come from the caller, never from a hidden read of
 * the stream; a stream whose header disagrees, or whose offsets / positions
 * point outside their sections, sets SPLITZIP_STATUS_BAD_STREAM and the
 * offending records are skipped (no out-of-bounds access).  comp_bytes below
 * splitzip_fixed_bytes() -> SPLITZIP_ERR_CAPACITY. */
int splitzip_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                        const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes,
                        void* stream);

/* Several tensors per launch -- all layers' K and V of a KV cache, or of a
 * prefill chunk (the pipeline of the appendix "The Potential of Hiding Codec
 * Overhead with Pipeline Overlap" feeds the codec such batches).  Each item is
 * compressed exactly as splitzip_compress would (same stream bytes); what a
 * single call pays per tensor for two launches -- the ramps of the dense pass
 * and the short finishing pass -- is paid once per 64 tensors.  Every item
 * names its own codebook: per-layer codebooks (the
 * section "Ablation on Layer-Wise Coverage") cost no more than shared ones.
 * `items` is a HOST array, read before the call returns.
 * d_sizes is a device array of n_items records.  Argument errors are found
 * before anything is enqueued.  Same workspace rules as splitzip_compress
 * (size it for the largest item; the items of a launch share its staging
 * area, a larger workspace gives every tile more room for escape records). */
typedef struct {
  const void* d_in;
  uint64_t n_elems;
  void* d_out;
  size_t out_capacity;
  const splitzip_codebook* cb;
} splitzip_item;
int splitzip_compress_batch(const splitzip_item* items, uint32_t n_items, int dtype, void* d_workspace,
                            size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream);

/* Several streams per launch; each item as splitzip_decompress.  d_sizes
 * (nullable) is ONE record: the status bits of all items are OR-ed into it,
 * total_bytes / n_escapes are those of whichever item wrote last. */
typedef struct {
  const void* d_comp;
  size_t comp_bytes;
  uint64_t n_elems;
  void* d_out;
  const splitzip_codebook* cb;
} splitzip_ditem;
int splitzip_decompress_batch(const splitzip_ditem* items, uint32_t n_items, int dtype, splitzip_sizes* d_sizes,
                              void* stream);

/* Calibration per tensor for a whole batch, on the device (the "dynamic"
 * codebook of the ablation "pre-calibration vs. dynamic codebook", and the
 * per-layer codebooks of "Ablation on Layer-Wise Coverage", without a host
 * round trip): splitzip_calibrate_batch_device counts the exponents of every
 * items[k].d_in (n_elems words; d_out, out_capacity and cb are not looked at)
 * into d_hists + 256 k and ranks them into d_cbs[k], exactly as
 * splitzip_histogram and splitzip_codebook_device do for one tensor, in three
 * launches per 64 tensors.  d_hists: n_items x 256 device words, 8-byte
 * aligned, zeroed by the call; d_cbs: n_items splitzip_codebook in device
 * memory, 4-byte aligned.  The _batch_dcb calls are the batch calls with
 * tensor k under d_cbs[k]; the items' own cb fields are not looked at.  As
 * with the _dcb calls the host cannot check such codebooks. */
int splitzip_calibrate_batch_device(const splitzip_item* items, uint32_t n_items, int dtype, uint64_t* d_hists,
                                    splitzip_codebook* d_cbs, void* stream);
int splitzip_compress_batch_dcb(const splitzip_item* items, uint32_t n_items, int dtype, const splitzip_codebook* d_cbs,
                                void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream);
int splitzip_decompress_batch_dcb(const splitzip_ditem* items, uint32_t n_items, int dtype, const splitzip_codebook* d_cbs,
                                  splitzip_sizes* d_sizes, void* stream);

/* Decompress with the codebook the stream itself carries: its header holds the
 * 16 decode entries, which is all a decoder needs (section 3.2, decoding
 * path).  A receiver of streams made under per-tensor or per-call codebooks
 * needs no side channel for them.  Everything else as splitzip_decompress /
 * splitzip_decompress_batch (the items' cb fields are not looked at); the
 * header check then vouches for everything but the entries themselves, and
 * entries that are no exponents of the dtype give a wrong tensor, never an
 * access out of bounds. */
int splitzip_decompress_own(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype, void* d_out,
                            splitzip_sizes* d_sizes, void* stream);
int splitzip_decompress_batch_own(const splitzip_ditem* items, uint32_t n_items, int dtype, splitzip_sizes* d_sizes,
                                  void* stream);

/* Measurement aid: a plain streaming kernel that reads read_bytes from d_src
 * and writes write_bytes (<= read_bytes) to d_dst with 128-bit accesses, i.e.
 * the memory traffic of the codec without its arithmetic.  Both sizes are
 * rounded down to a multiple of 16. */
int splitzip_traffic_probe(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes,
                           void* stream);

/* Measurement aid: the same kind of kernel with its shape as arguments, for
 * finding the bandwidth the memory system gives a streaming kernel at best
 * (the ceiling the codec's kernels are compared with).  Per step a workgroup
 * of 256 threads reads reads_per_step and writes writes_per_step coalesced
 * runs of 4 KB; (reads, writes) is one of (1,0) (2,0) (4,0) (8,0) read only,
 * (0,1) (0,2) (0,4) (0,8) write only, (4,3) (8,6) (16,12) the compress mix,
 * (3,4) (6,8) (12,16) the decompress mix, (1,1) (2,2) (4,4) a copy; wgs_per_cu
 * is 1 to 32 workgroups per CU that stay for the whole launch, or 0 for one
 * workgroup per step, started by the hardware in order.  Every load of a step
 * is issued before the first is waited for, and every store before the next
 * step's loads.  flags: bit 0 non-temporal loads, bit 1 non-temporal stores,
 * bit 2 every workgroup owns one contiguous block of steps (otherwise the
 * steps are dealt round robin), bit 3 (with bit 2) every workgroup starts at
 * a different place inside its block, bit 4 (without bits 2 and 3) the steps
 * are handed out through a counter in the 4 bytes behind the written bytes,
 * which the caller has set to zero, bit 5 (with the shape (4,3)) the stores
 * have the codec's widths, 8 and 4 bytes per thread.  read_bytes of d_src are
 * read and write_bytes of d_dst written (each rounded down to a multiple of
 * 16; the side with 0 runs per step is not touched, but both pointers must be
 * valid).  Anything else gives
 * SPLITZIP_ERR_INVALID_ARG. */
int splitzip_traffic_probe_shape(const void* d_src, size_t read_bytes, void* d_dst, size_t write_bytes,
                                 uint32_t reads_per_step, uint32_t writes_per_step, uint32_t wgs_per_cu,
                                 uint32_t flags, void* stream);

/* ---- Paged and strided tensors ------------------------------------------------
 *
 * Serving stacks keep the KV cache in fixed-size pages of a pool and find a
 * sequence's pages through a block table (the serving integration of the
 * paper's section 4, "Experiments", moves such caches).  These calls compress a tensor straight
 * out of such a pool and decompress straight into one: the stream is exactly
 * that of splitzip_compress on the gathered, contiguous tensor.  Logical
 * element i lives at
 *   d_pool + d_block_table[i / block_elems] * page_stride_bytes + offset_bytes
 *          + (i % block_elems) * element size.
 * A tensor whose tokens are strided (token stride above heads x head_dim) is
 * the same thing with one token per page and the identity as the table. */
typedef struct {
  void* d_pool;                  /* device address of the pool, 16-byte aligned */
  const uint32_t* d_block_table; /* device array of n_blocks page indices into the pool; entries at or above
                                    n_pool_blocks are clamped to the last page (never an access outside the pool) */
  uint32_t n_blocks;             /* entries of the table; n_blocks * block_elems >= n_elems */
  uint32_t n_pool_blocks;        /* pages in the pool */
  uint32_t block_elems;          /* elements of this tensor per page: a power of two, at least 1024 */
  uint32_t reserved;             /* 0 */
  uint64_t page_stride_bytes;    /* distance between pages of the pool, a multiple of 16 */
  uint64_t offset_bytes;         /* where this tensor's elements start inside every page (the V half, a layer's
                                    slot), a multiple of 16; offset + block_elems * element size <= page stride */
} splitzip_paged;

/* splitzip_compress / splitzip_decompress with the words in a paged pool.  All
 * other arguments, the stream format, the sizes record and the error codes are
 * those of the contiguous calls; a description that breaks one of the rules
 * above gives SPLITZIP_ERR_INVALID_ARG.  Decompress writes the n_elems words
 * and nothing else of the pool. */
int splitzip_compress_paged(const splitzip_paged* src, uint64_t n_elems, int dtype, const splitzip_codebook* cb,
                            void* d_out, size_t out_capacity, void* d_workspace, size_t workspace_bytes,
                            splitzip_sizes* d_sizes, void* stream);
int splitzip_decompress_paged(const void* d_comp, size_t comp_bytes, uint64_t n_elems, int dtype,
                              const splitzip_codebook* cb, const splitzip_paged* dst, splitzip_sizes* d_sizes,
                              void* stream);

/* The batch calls with every tensor in a paged pool behind ONE block table -- all layers' K and V of one
 * sequence, the usual layout of a serving stack.  `paging` gives the table and the page geometry
 * (d_block_table, n_blocks, n_pool_blocks, block_elems, page_stride_bytes; its d_pool is ignored and its
 * offset_bytes only enters the check that a page holds block_elems words behind it).  item.d_in (item.d_out
 * for decompress) is the address of the tensor's words in page 0 of ITS pool -- pool base plus the tensor's
 * offset inside a page -- so every tensor may sit in a pool of its own as long as all share the table and
 * the geometry.  Everything else as splitzip_compress_batch / splitzip_decompress_batch. */
int splitzip_compress_batch_paged(const splitzip_item* items, uint32_t n_items, int dtype, const splitzip_paged* paging,
                                  void* d_workspace, size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream);
int splitzip_decompress_batch_paged(const splitzip_ditem* items, uint32_t n_items, int dtype, const splitzip_paged* paging,
                                    splitzip_sizes* d_sizes, void* stream);

/* ---- Format variants of the paper's ablations --------------------------------
 *
 * The same codec with its knobs turned the way the ablations turn them
 * (sections "Ablation on Top-k Exponent Coding" and "Ablation on
 * Escape-Position Metadata", appendices "Ablation on Chunk Size" and
 * "SplitZip on FP8"): 3-bit codes over a top-8 codebook, a top-15 codebook
 * with the last 4-bit code as an escape sentinel and no stored positions,
 * 256-element chunks with 8-bit positions, 32-bit absolute positions without
 * chunks, and E4M3 words.  These calls exist to measure those formats beside
 * the main one on the same device; they run through one generic set of kernels
 * (dense pass with per-chunk counts and staged escape records, sums, finishing
 * pass; dense decode with the correction applied in LDS) that is NOT the tuned
 * path of splitzip_compress
 * and splitzip_decompress.  The main format is one of the variants, so all of
 * them can be compared through the same kernels.
 *
 * Version-2 stream: as the layout at the top of this file, with
 *   header     u16 version 2, u8 code bits, u32 chunk elements (0 in the
 *              absolute mode), and in place of the u32 0: u8 escape mode,
 *              u8 k, u16 0; dec[] slots >= k are 0
 *   chunk_off  4(C+1) B with C = ceil(N / chunk); absent in the absolute mode
 *   sm plane   ceil(N sb / 8) B, sb = 8, 3, 4 bits for BF16, E5M2, E4M3
 *   code plane ceil(N cb / 8) B; both planes are LSB-first bit streams
 *   esc_pos    u16[M] (chunk > 256) or u8[M]; nothing in the sentinel mode;
 *              u32[M] element indices in the absolute mode
 *   esc_val    u8[M], or M values of value_bits bits each (header byte 14 holds
 *              value_bits then, else 0)
 * With (BF16 or E5M2, 4, 16, SPLITZIP_ESC_POS, 1024, whole-byte values) every byte behind the
 * header equals the main format's stream. */
typedef enum {
  SPLITZIP_ESC_POS = 0,      /* chunk-relative positions + exponents (the main format's way) */
  SPLITZIP_ESC_SENTINEL = 1, /* the all-ones code marks an escape; exponents only, in element order */
  SPLITZIP_ESC_ABS32 = 2     /* 32-bit element indices + exponents, no chunks and no offset table */
} splitzip_escape_mode;

typedef struct {
  uint32_t dtype;       /* splitzip_dtype */
  uint32_t code_bits;   /* 3 or 4 */
  uint32_t k;           /* codebook entries in use: 1 .. 2^code_bits (one less in the sentinel mode) */
  uint32_t escape_mode; /* splitzip_escape_mode */
  uint32_t chunk_elems; /* 256 or 1024; ignored in the absolute mode */
  uint32_t value_bits;  /* bits per escape value: 0 or 8 = a whole byte (the main format's record); or the exponent
                           field's own width, 5 for E5M2 and 4 for E4M3: the value section is then an LSB-first bit
                           stream of ceil(M value_bits / 8) bytes.  The top-8 columns of the paper's FP8 table (ratios
                           1.049 and 0.933) count 21 and 20 bits per escape, i.e. this width. */
} splitzip_variant;

/* 1 if the library can run this variant, else 0 */
int splitzip_variant_supported(const splitzip_variant* v);

/* Sizes as for the main format (0 for an unsupported variant or n_elems >= 2^32). */
size_t splitzip_variant_total_bytes(uint64_t n_elems, uint64_t n_escapes, const splitzip_variant* v);
size_t splitzip_variant_compress_bound(uint64_t n_elems, const splitzip_variant* v);
/* Device scratch of one compress call: per-chunk counts, their sums, and a slot of staged escape records per 1024
 * elements (about n_elems / 2 bytes).  No initialisation needed. */
size_t splitzip_variant_workspace_bytes(uint64_t n_elems, const splitzip_variant* v);

/* Section 3.3 with v->k entries: counts the exponents of a HOST sample and
 * ranks them as splitzip_calibrate does; the first k of that ranking form the
 * codebook (out->dec[k..15] = 0, only those k are members).  hist_out as for
 * splitzip_calibrate (E4M3 uses the first 16 bins). */
int splitzip_variant_calibrate(const void* h_sample, uint64_t n_elems, const splitzip_variant* v,
                               splitzip_codebook* out, uint64_t* hist_out);
/* The same from the first k entries of a decoding table. */
int splitzip_variant_codebook_from_dec(const uint8_t* dec, const splitzip_variant* v, splitzip_codebook* out);

/* Compress / decompress in the variant's format.  Arguments, alignment rules,
 * the sizes record (total_bytes, n_escapes, status; OVERFLOW and BAD_STREAM as
 * for the main calls) and the error codes are those of splitzip_compress and
 * splitzip_decompress; d_workspace needs splitzip_variant_workspace_bytes and
 * 16-byte alignment.  Three kernel launches per compress call (dense pass
 * that also stages the escape records, sums of the per-chunk counts, finishing
 * pass; a fourth packs values narrower than a byte), one per decompress call
 * (two in the absolute mode), all on `stream`. */
int splitzip_variant_compress(const void* d_in, uint64_t n_elems, const splitzip_variant* v,
                              const splitzip_codebook* cb, void* d_out, size_t out_capacity, void* d_workspace,
                              size_t workspace_bytes, splitzip_sizes* d_sizes, void* stream);
int splitzip_variant_decompress(const void* d_comp, size_t comp_bytes, uint64_t n_elems, const splitzip_variant* v,
                                const splitzip_codebook* cb, void* d_out, splitzip_sizes* d_sizes, void* stream);

const char* splitzip_strerror(int err);
int splitzip_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPLITZIP_H */
