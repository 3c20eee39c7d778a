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
    int part = 0;
    for (int k = threadIdx.x; k < int(blockIdx.x); k += kCompactThreads) part += chunk_counts[k];
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

}  // namespace lgp
