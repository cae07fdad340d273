// SplitZip for MI355X: calibration histogram, workspace initialisation and the plain streaming kernel used as a measurement aid.
// Part of the single translation unit splitzip.hip (included inside its anonymous namespace).
#ifndef SPLITZIP_AUX_KERNELS_HPP
#define SPLITZIP_AUX_KERNELS_HPP

// ---------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------

// Calibration histogram (section 3.3) of a device sample: exponent counts, added to hist[256].
// Every workgroup counts into 64 copies of the bins in LDS, one per lane, interleaved: the count of bin b in
// the copy of lane l is word 64 b + l, so a lane only ever touches its own bank and no two lanes of a wave an
// address in common, whatever they count.  (Eight copies in rows of 256 words, the first version, sent all
// lanes that count the same exponent -- most of them, the distribution being what it is -- to one bank: 39 % of
// the LDS cycles were conflict cycles.)  The waves of a workgroup share the copies, hence atomic adds.
// Non-zero totals go to the global bins at the end.
template <bool BF16>
__device__ inline void histogram_body(const uint8_t* in, uint64_t n, uint64_t* hist) {
  constexpr int BINS = BF16 ? 256 : 32;
  __shared__ uint32_t bins[BINS * 64];
  const int tid = threadIdx.x;
  for (int i = tid; i < BINS * 64; i += 1024) bins[i] = 0;
  __syncthreads();
  uint32_t* mine = bins + (tid & 63);
  const uint64_t bytes = n * (BF16 ? 2 : 1), nvec = bytes / 16;
  const u32x4* v = reinterpret_cast<const u32x4*>(in);
  auto count = [&](const u32x4& q) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      if (BF16) {
        atomicAdd(&mine[((w[d] >> 7) & 0xffu) * 64], 1u);
        atomicAdd(&mine[((w[d] >> 23) & 0xffu) * 64], 1u);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) atomicAdd(&mine[((w[d] >> (8 * j + 2)) & 31u) * 64], 1u);
      }
    }
  };
  // four vectors per thread in flight: the loads of a step are all issued before the first is counted
  const uint64_t step = (uint64_t)gridDim.x * 1024;
  uint64_t i = blockIdx.x * 1024ull + tid;
  for (; i + 3 * step < nvec; i += 4 * step) {
    u32x4 q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) q[u] = ld_stream(v + i + u * step);
#pragma unroll
    for (int u = 0; u < 4; ++u) count(q[u]);
  }
  for (; i < nvec; i += step) count(ld_stream(v + i));
  // the words behind the last whole vector, by workgroup 0
  if (blockIdx.x == 0) {
    for (uint64_t i = nvec * 16 + (uint64_t)tid * (BF16 ? 2 : 1); i < bytes; i += 1024 * (BF16 ? 2 : 1)) {
      const uint32_t e = BF16 ? ((uint32_t)(in[i] | (in[i + 1] << 8)) >> 7) & 0xffu : ((uint32_t)in[i] >> 2) & 31u;
      atomicAdd(&mine[e * 64], 1u);
    }
  }
  __syncthreads();
  if (tid < BINS) {
    uint64_t c = 0;
#pragma unroll 8
    for (int r = 0; r < 64; ++r) c += bins[tid * 64 + ((r + tid) & 63)];   // thread t starts at copy t: no two on one bank
    if (c) atomicAdd(reinterpret_cast<unsigned long long*>(&hist[tid]), (unsigned long long)c);
  }
}

template <bool BF16>
__global__ __launch_bounds__(1024) void histogram_kernel(const uint8_t* in, uint64_t n, uint64_t* hist) {
  histogram_body<BF16>(in, n, hist);
}

// the same for several samples in one launch: blockIdx.y picks the sample, its counts go to hists + 256 y
struct HistBatchArgs {
  const uint8_t* in[64];
  uint64_t n[64];
};
template <bool BF16>
__global__ __launch_bounds__(1024) void histogram_batch_kernel(const HistBatchArgs a, uint64_t* hists) {
  histogram_body<BF16>(a.in[blockIdx.y], a.n[blockIdx.y], hists + 256 * blockIdx.y);
}

__global__ void zero_words_kernel(uint64_t* p, uint64_t nwords) {
  for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < nwords; i += (uint64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Section 3.3 on the device: the three tables from 256 exponent counts.  One workgroup per codebook
// (workgroup b: counts hist + 256 b, tables cb + b); thread v ranks exponent v by (count descending,
// exponent ascending) among the format's exponents, the 16 first ranks form the codebook.
__global__ __launch_bounds__(256) void codebook_kernel(const uint64_t* hist, uint32_t n_values, uint32_t dtype,
                                                       splitzip_codebook* cb) {
  hist += 256 * blockIdx.x;
  cb += blockIdx.x;
  __shared__ uint64_t h[256];
  const uint32_t v = threadIdx.x;
  h[v] = v < n_values ? hist[v] : 0;
  __syncthreads();
  uint32_t rank = 0;
  for (uint32_t u = 0; u < n_values; ++u) rank += (h[u] > h[v] || (h[u] == h[v] && u < v)) ? 1u : 0u;
  const bool in = v < n_values && rank < 16;
  cb->enc[v] = in ? (uint8_t)rank : (uint8_t)0;
  cb->member[v] = in ? 1 : 0;
  if (in) cb->dec[rank] = (uint8_t)v;
  if (v == 0) cb->dtype = dtype;
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
    // a step inside both buffers runs without a condition per access: all its loads are on their way before the
    // first is waited for, and its stores follow one another without a wait in between
    const bool whole = (4 * (s + 1)) * kThreads <= nread && (3 * (s + 1)) * kThreads <= nwrite;
    if (whole) {
      const u32x4* sp = src + 4 * s * kThreads + threadIdx.x;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = ld_stream(sp + i * kThreads);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint64_t idx = (4 * s + i) * kThreads + threadIdx.x;
        v[i] = idx < nread ? ld_stream(src + idx) : u32x4{0u, 0u, 0u, 0u};
      }
    }
    v[0].x ^= v[3].x; v[1].y ^= v[3].y; v[2].z ^= v[3].z; v[0].w ^= v[3].w;
    if (whole) {
      u32x4* dp = dst + 3 * s * kThreads + threadIdx.x;
#pragma unroll
      for (int i = 0; i < 3; ++i) st_stream(dp + i * kThreads, v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const uint64_t idx = (3 * s + i) * kThreads + threadIdx.x;
        if (idx < nwrite) st_stream(dst + idx, v[i]);
      }
    }
  }
}

// The same with its shape as arguments, for finding out what the memory system gives a streaming kernel at best:
// per step a workgroup reads R coalesced 4 KB runs and writes W (either may be 0: write only, read only), with
// temporal or non-temporal accesses; the steps are dealt to the workgroups round robin (neighbouring workgroups
// work on neighbouring runs) or in one contiguous block each (the way the codec's kernels own their chunks).
template <int R, int W, bool NTL, bool NTS>
__global__ __launch_bounds__(kThreads) void traffic_shape_kernel(const u32x4* src, uint64_t nread, u32x4* dst, uint64_t nwrite,
                                                                  uint64_t steps, uint32_t blocked_in) {
  const uint32_t blocked = blocked_in & 3u;
  const bool blocked_narrow = (blocked_in & 4u) != 0;
  const uint64_t per = (steps + gridDim.x - 1) / gridDim.x;
  const uint64_t s0 = blocked ? blockIdx.x * per : blockIdx.x;
  const uint64_t s_end = blocked ? (s0 + per < steps ? s0 + per : steps) : steps, stride = blocked ? 1 : gridDim.x;
  // blocked == 2: every workgroup starts somewhere else inside its block and wraps around, so that the workgroups
  // are not all at the same distance from the start of their blocks at the same time
  const uint64_t len = s_end > s0 ? s_end - s0 : 0, rot = blocked == 2 && len ? (blockIdx.x * 37ull) % len : 0;
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  // blocked == 3: the steps are handed out in order through a counter (the word behind the written bytes, zeroed
  // by the caller): the next step's number is fetched while this step's runs are on their way
  __shared__ uint32_t s_ticket[2];
  uint32_t* counter = reinterpret_cast<uint32_t*>(dst + nwrite);
  uint64_t tk = 0;
  if (blocked == 3) {
    if (threadIdx.x == 0) s_ticket[0] = atomicAdd(counter, 1u);
    __syncthreads();
    tk = s_ticket[0];
  }
  for (uint64_t q = 0; blocked == 3 ? tk < steps : s0 + q * stride < s_end; ++q) {
    const uint64_t s = blocked == 3 ? tk : blocked == 2 ? s0 + (q + rot) % len : s0 + q * stride;
    if (blocked == 3) {
      if (threadIdx.x == 0) s_ticket[(q + 1) & 1] = atomicAdd(counter, 1u);
      __syncthreads();
      tk = s_ticket[(q + 1) & 1];
    }
    u32x4 v[R > 0 ? R : 1];
    v[0] = u32x4{(uint32_t)s, threadIdx.x, 0u, 0u};
    // A step that lies inside both buffers entirely (all but the last, as a rule) runs without a condition per
    // access: every load of the step is on its way before the first is waited for, and so is every store.
    const bool whole = (R == 0 || ((uint64_t)R * (s + 1)) * kThreads <= nread) && (W == 0 || ((uint64_t)W * (s + 1)) * kThreads <= nwrite);
    if (whole) {
      const u32x4* sp = src + (uint64_t)R * s * kThreads + threadIdx.x;
#pragma unroll
      for (int i = 0; i < R; ++i) v[i] = NTL ? ld_stream(sp + i * kThreads) : sp[i * kThreads];
    } else {
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const uint64_t idx = ((uint64_t)R * s + i) * kThreads + threadIdx.x;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (idx < nread) v[i] = NTL ? ld_stream(src + idx) : src[idx];
      }
    }
    if (W == 0) {
#pragma unroll
      for (int i = 0; i < R; ++i) acc ^= v[i];
    }
    if (blocked_narrow) {
      // the codec's store shapes: two thirds of the step's bytes as 8-byte stores, one third as 4-byte stores
      if (W == 3 && whole) {
        uint8_t* base = reinterpret_cast<uint8_t*>(dst + (uint64_t)W * s * kThreads);
#pragma unroll
        for (int i = 0; i < 4; ++i) st_stream(reinterpret_cast<u32x2*>(base) + i * kThreads + threadIdx.x, u32x2{v[i % (R > 0 ? R : 1)].x, v[i % (R > 0 ? R : 1)].y});
#pragma unroll
        for (int i = 0; i < 4; ++i) st_stream(reinterpret_cast<uint32_t*>(base + 8192) + i * kThreads + threadIdx.x, v[i % (R > 0 ? R : 1)].z);
      }
      continue;
    }
    if (whole) {
      u32x4* dp = dst + (uint64_t)W * s * kThreads + threadIdx.x;
#pragma unroll
      for (int i = 0; i < W; ++i) {
        const u32x4 o = v[R > 0 ? i % R : 0];
        if (NTS) st_stream(dp + i * kThreads, o);
        else dp[i * kThreads] = o;
      }
    } else {
#pragma unroll
      for (int i = 0; i < W; ++i) {
        const uint64_t idx = ((uint64_t)W * s + i) * kThreads + threadIdx.x;
        const u32x4 o = v[R > 0 ? i % R : 0];
        if (idx < nwrite) {
          if (NTS) st_stream(dst + idx, o);
          else dst[idx] = o;
        }
      }
    }
  }
  // read only: the words must be used; no tensor holds this pattern in every lane
  if (W == 0 && acc.x == 0x5a17c0deu && acc.y == 0x5a17c0deu && acc.z == 0x5a17c0deu && acc.w == 0x5a17c0deu) dst[0] = acc;
}

#endif  // SPLITZIP_AUX_KERNELS_HPP
