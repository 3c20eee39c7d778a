// Frontier / gather-set dedup (implied by Sec. 4.2.2: each vertex of a mini-batch's
// sample result counts once).  The sampler sets one bit per sampled vertex; this file
// turns the bitmap into the ascending list of set bits, which is the sorted-unique
// order without any sort.  One workgroup covers kChunkBits vertices; a first kernel
// counts set bits per chunk, a second sums the counts of the chunks before it, scans
// its own 256 per-thread counts and writes the ids.
#include "common.hpp"

namespace lgp {
namespace {

__device__ __forceinline__ int wave_inclusive_scan(int x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  return x;
}

// Exclusive scan of one int per thread over a 256-thread workgroup; *total = sum.
__device__ __forceinline__ int block_exclusive_scan(int x, int* total) {
  __shared__ int wave_sum[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int inc = wave_inclusive_scan(x);
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int sw = wave_sum[w];
    if (w < wave) before += sw;
    all += sw;
  }
  __syncthreads();
  *total = all;
  return before + inc - x;
}

// This thread's share of counts[0 .. n): eight loads in flight per round, so that a workgroup far down the
// bitmap (thousands of chunks before it) waits for one or two round trips to L2, not for one per 256 chunks.
__device__ __forceinline__ int sum_before(const int32_t* __restrict__ counts, int n) {
  int part = 0;
  for (int k0 = 0; k0 < n; k0 += kCompactThreads * 8) {
    int v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = k0 + j * kCompactThreads + int(threadIdx.x);
      v[j] = k < n ? counts[k] : 0;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) part += v[j];
  }
  return part;
}

__global__ __launch_bounds__(kCompactThreads) void count_bits_kernel(const uint64_t* __restrict__ bits,
                                                                     int32_t* __restrict__ chunk_counts) {
  const uint64_t* w = bits + int64_t(blockIdx.x) * kChunkWords + int64_t(threadIdx.x) * kWordsPerThread;
  int c = 0;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) c += __popcll(w[q]);
  int total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) chunk_counts[blockIdx.x] = total;
}

template <bool WITH_OUT>
__global__ __launch_bounds__(kCompactThreads) void emit_bits_kernel(
    uint64_t* __restrict__ bits, uint64_t* __restrict__ or_into, const int32_t* __restrict__ chunk_counts,
    int32_t* __restrict__ out, int64_t out_cap, int32_t* __restrict__ n_out, uint32_t* __restrict__ bump,
    uint32_t* __restrict__ d_err, int shift) {
  const int64_t word0 = int64_t(blockIdx.x) * kChunkWords + int64_t(threadIdx.x) * kWordsPerThread;
  uint64_t w[kWordsPerThread];
  int c = 0;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) {
    w[q] = bits[word0 + q];
    c += __popcll(w[q]);
  }
  int64_t pos = 0;
  if (WITH_OUT) {
    const int part = sum_before(chunk_counts, int(blockIdx.x));
    int before_chunks, mine_total;
    block_exclusive_scan(part, &before_chunks);
    const int excl = block_exclusive_scan(c, &mine_total);
    pos = int64_t(before_chunks) + excl;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
      const int64_t total = int64_t(before_chunks) + mine_total;
      *n_out = int32_t(total <= out_cap ? total : out_cap);
      if (total > out_cap) atomicOr(d_err, ERR_OVERRUN);
    }
  }
  if (c == 0) return;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) {
    uint64_t x = w[q];
    if (x == 0) continue;
    if (or_into) or_into[word0 + q] |= x;
    bits[word0 + q] = 0;
    const int64_t id0 = (word0 + q) * 64;
    while (x) {
      const int b = __ffsll((unsigned long long)x) - 1;
      const int32_t id = int32_t((id0 + b) >> shift);
      if (WITH_OUT) {
        if (pos < out_cap) out[pos] = id;
        ++pos;
      }
      if (bump) atomicAdd(&bump[id], 1u);
      x &= x - 1;
    }
  }
}

// ---- intra-batch pipeline: frontier list + "reached first by this hop" list in one pass ---------------
// Same two-kernel scheme with two counts per chunk: all marked vertices (the next frontier) and those
// not yet in `seen` (the vertices whose feature rows can be extracted now).
__global__ __launch_bounds__(kCompactThreads) void count_new_bits_kernel(const uint64_t* __restrict__ bits,
                                                                         const uint64_t* __restrict__ seen,
                                                                         int32_t* __restrict__ chunk_counts,
                                                                         int32_t* __restrict__ new_counts) {
  const int64_t word0 = int64_t(blockIdx.x) * kChunkWords + int64_t(threadIdx.x) * kWordsPerThread;
  int c = 0, cn = 0;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) {
    const uint64_t x = bits[word0 + q];
    c += __popcll(x);
    if (x) cn += __popcll(x & ~seen[word0 + q]);
  }
  int total, total_new;
  block_exclusive_scan(c, &total);
  block_exclusive_scan(cn, &total_new);
  if (threadIdx.x == 0) {
    chunk_counts[blockIdx.x] = total;
    new_counts[blockIdx.x] = total_new;
  }
}

template <bool WITH_OUT>
__global__ __launch_bounds__(kCompactThreads) void emit_new_bits_kernel(
    uint64_t* __restrict__ bits, uint64_t* __restrict__ seen, const int32_t* __restrict__ chunk_counts,
    const int32_t* __restrict__ new_counts, int32_t* __restrict__ out, int64_t out_cap, int32_t* __restrict__ n_out,
    int32_t* __restrict__ listed, int64_t listed_cap, int32_t* __restrict__ seg, int32_t* __restrict__ n_listed,
    uint32_t* __restrict__ d_err, int shift) {
  const int64_t word0 = int64_t(blockIdx.x) * kChunkWords + int64_t(threadIdx.x) * kWordsPerThread;
  uint64_t w[kWordsPerThread], fresh[kWordsPerThread];
  int c = 0, cn = 0;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) {
    w[q] = bits[word0 + q];
    fresh[q] = w[q] ? (w[q] & ~seen[word0 + q]) : 0ull;
    c += __popcll(w[q]);
    cn += __popcll(fresh[q]);
  }
  const int part = sum_before(chunk_counts, int(blockIdx.x));
  const int part_new = sum_before(new_counts, int(blockIdx.x));
  int before, before_new, mine, mine_new;
  block_exclusive_scan(part, &before);
  block_exclusive_scan(part_new, &before_new);
  const int excl = block_exclusive_scan(c, &mine);
  const int excl_new = block_exclusive_scan(cn, &mine_new);
  const int64_t base = seg[0];
  int64_t pos = int64_t(before) + excl;
  int64_t pos_new = base + before_new + excl_new;
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
    const int64_t total = int64_t(before) + mine;
    if (WITH_OUT) {
      *n_out = int32_t(total <= out_cap ? total : out_cap);
      if (total > out_cap) atomicOr(d_err, ERR_OVERRUN);
    }
    int64_t end = base + before_new + mine_new;
    if (end > listed_cap) {
      atomicOr(d_err, ERR_OVERRUN);
      end = listed_cap;
    }
    seg[1] = int32_t(end);
    if (n_listed) *n_listed = int32_t(end);
  }
  if (c == 0) return;
#pragma unroll
  for (int q = 0; q < kWordsPerThread; ++q) {
    uint64_t x = w[q];
    if (x == 0) continue;
    if (fresh[q]) seen[word0 + q] |= x;
    bits[word0 + q] = 0;
    const int64_t id0 = (word0 + q) * 64;
    const uint64_t f = fresh[q];
    while (x) {
      const int b = __ffsll((unsigned long long)x) - 1;
      const int32_t id = int32_t((id0 + b) >> shift);
      if (WITH_OUT) {
        if (pos < out_cap) out[pos] = id;
        ++pos;
      }
      if ((f >> b) & 1ull) {
        if (pos_new < listed_cap) listed[pos_new] = id;
        ++pos_new;
      }
      x &= x - 1;
    }
  }
}

__global__ __launch_bounds__(256) void begin_listing_kernel(const int32_t* __restrict__ seeds, int64_t n_seeds,
                                                            int32_t* __restrict__ listed, int32_t* __restrict__ seg,
                                                            int32_t* __restrict__ counters, int32_t n_counters) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (t == 0) {
    seg[0] = 0;
    seg[1] = int32_t(n_seeds);
  }
  if (t < n_counters) counters[t] = 0;
  for (int64_t i = t; i < n_seeds; i += int64_t(gridDim.x) * 256) listed[i] = seeds[i];
}

__global__ void sum_stats_kernel(const int32_t* __restrict__ seg_counters, int32_t n_seg, int32_t* __restrict__ stats) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int32_t hit = 0, miss = 0;
    for (int32_t k = 0; k < n_seg; ++k) {
      hit += seg_counters[3 * k];
      miss += seg_counters[3 * k + 1];
    }
    stats[0] = hit;
    stats[1] = miss;
  }
}

}  // namespace

void launch_compact(const DeviceInfo& di, uint64_t* bits, uint64_t* or_into, int64_t n_chunks, int32_t* chunk_counts,
                    int32_t* out, int64_t out_cap, int32_t* n_out, uint32_t* bump, uint32_t* d_err, hipStream_t s) {
  if (n_out) {
    hipLaunchKernelGGL(count_bits_kernel, dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits, chunk_counts);
    hipLaunchKernelGGL((emit_bits_kernel<true>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits, or_into,
                       chunk_counts, out, out_cap, n_out, bump, d_err, di.spread_shift);
  } else {
    hipLaunchKernelGGL((emit_bits_kernel<false>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits,
                       or_into, chunk_counts, out, out_cap, n_out, bump, d_err, di.spread_shift);
  }
}

void launch_compact_new(const DeviceInfo& di, uint64_t* bits, uint64_t* seen, int64_t n_chunks, int32_t* chunk_counts,
                        int32_t* new_counts, int32_t* out, int64_t out_cap, int32_t* n_out, int32_t* listed,
                        int64_t listed_cap, int32_t* seg, int32_t* n_listed, uint32_t* d_err, hipStream_t s) {
  hipLaunchKernelGGL(count_new_bits_kernel, dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits, seen,
                     chunk_counts, new_counts);
  if (n_out)
    hipLaunchKernelGGL((emit_new_bits_kernel<true>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits, seen,
                       chunk_counts, new_counts, out, out_cap, n_out, listed, listed_cap, seg, n_listed, d_err,
                       di.spread_shift);
  else
    hipLaunchKernelGGL((emit_new_bits_kernel<false>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, bits, seen,
                       chunk_counts, new_counts, out, out_cap, n_out, listed, listed_cap, seg, n_listed, d_err,
                       di.spread_shift);
}

void launch_begin_listing(const DeviceInfo& di, const int32_t* seeds, int64_t n_seeds, int32_t* listed, int32_t* seg,
                          int32_t* counters, int32_t n_counters, hipStream_t s) {
  int64_t blocks = (n_seeds + 255) / 256;
  if (blocks > di.num_cus * 4) blocks = di.num_cus * 4;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(begin_listing_kernel, dim3(unsigned(blocks)), dim3(256), 0, s, seeds, n_seeds, listed, seg,
                     counters, n_counters);
}

void launch_sum_stats(const int32_t* seg_counters, int32_t n_seg, int32_t* stats, hipStream_t s) {
  hipLaunchKernelGGL(sum_stats_kernel, dim3(1), dim3(64), 0, s, seg_counters, n_seg, stats);
}

}  // namespace lgp
