// Frontier / gather-set dedup (implied by Sec. 4.2.2: each vertex of a mini-batch's
// sample result counts once).  The sampler stores a 1 into a byte map, one byte per
// vertex: plain stores, because device-scope atomics on this multi-die GPU are executed
// at the memory side (about 32 bytes of HBM traffic each) and were the sampler's
// bottleneck when a bit map was used.  This file turns the byte map into the ascending
// list of marked vertices -- the sorted-unique order without any sort.
//
// One workgroup covers kChunkIds vertices; each of its 4 waves owns a contiguous quarter
// and reads it in coalesced 16-byte pieces (16 flags per lane per step).  A first kernel
// counts marks per chunk; the second sums the counts of the chunks before it, ranks its
// own marks with wave scans and writes the ids.  It also clears the map and, if asked,
// copies the marks into the gather-set map and bumps a per-vertex counter.
#include "common.hpp"

namespace lgp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kSteps = int(kChunkIds / 4 / (64 * 16));   // 16-byte pieces per lane per wave = 16

__device__ __forceinline__ int wave_inclusive_scan(int x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  return x;
}

// 16 flag bytes (each 0 or 1) -> 16-bit mask, bit k = byte k.
__device__ __forceinline__ uint32_t flags_to_mask(u32x4 v) {
  const uint32_t a = (v.x * 0x01020408u) >> 24, b = (v.y * 0x01020408u) >> 24;
  const uint32_t c = (v.z * 0x01020408u) >> 24, d = (v.w * 0x01020408u) >> 24;
  return (a & 15u) | ((b & 15u) << 4) | ((c & 15u) << 8) | ((d & 15u) << 12);
}

__device__ __forceinline__ int block_sum(int x, int* lds4) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int inc = wave_inclusive_scan(x);
  if (lane == 63) lds4[wave] = inc;
  __syncthreads();
  const int total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(kCompactThreads) void count_marks_kernel(const uint8_t* __restrict__ map,
                                                                      int32_t* __restrict__ chunk_counts) {
  __shared__ int lds4[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const u32x4* p = reinterpret_cast<const u32x4*>(map + int64_t(blockIdx.x) * kChunkIds + int64_t(wave) * (kChunkIds / 4));
  int c = 0;
#pragma unroll
  for (int k = 0; k < kSteps; ++k) c += __popc(flags_to_mask(p[k * 64 + lane]));
  const int total = block_sum(c, lds4);
  if (threadIdx.x == 0) chunk_counts[blockIdx.x] = total;
}

template <bool WITH_OUT>
__global__ __launch_bounds__(kCompactThreads) void emit_marks_kernel(
    uint8_t* __restrict__ map, uint8_t* __restrict__ or_into, const int32_t* __restrict__ chunk_counts,
    int32_t* __restrict__ out, int64_t out_cap, int32_t* __restrict__ n_out, uint32_t* __restrict__ bump,
    uint32_t* __restrict__ d_err) {
  __shared__ int lds4[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t id_base = int64_t(blockIdx.x) * kChunkIds + int64_t(wave) * (kChunkIds / 4);
  u32x4* p = reinterpret_cast<u32x4*>(map + id_base);
  u32x4 v[kSteps];
  uint32_t m[kSteps];
  int c = 0;
#pragma unroll
  for (int k = 0; k < kSteps; ++k) v[k] = p[k * 64 + lane];
#pragma unroll
  for (int k = 0; k < kSteps; ++k) {
    m[k] = flags_to_mask(v[k]);
    c += __popc(m[k]);
  }
  int64_t pos = 0;
  if (WITH_OUT) {
    int part = 0;
    for (int k = threadIdx.x; k < int(blockIdx.x); k += kCompactThreads) part += chunk_counts[k];
    const int before_chunks = block_sum(part, lds4);
    const int wave_total = __shfl(wave_inclusive_scan(c), 63, 64);
    if (lane == 0) lds4[wave] = wave_total;
    __syncthreads();
    int before_waves = 0;
    for (int w = 0; w < wave; ++w) before_waves += lds4[w];
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
      const int64_t total = int64_t(before_chunks) + lds4[0] + lds4[1] + lds4[2] + lds4[3];
      *n_out = int32_t(total <= out_cap ? total : out_cap);
      if (total > out_cap) atomicOr(d_err, ERR_OVERRUN);
    }
    pos = int64_t(before_chunks) + before_waves;
    if (wave_total == 0) return;
  }
#pragma unroll
  for (int k = 0; k < kSteps; ++k) {
    const int ck = __popc(m[k]);
    int64_t my = pos;
    if (WITH_OUT) {
      const int inc = wave_inclusive_scan(ck);
      my = pos + inc - ck;
      pos += __shfl(inc, 63, 64);
    }
    if (m[k] == 0) continue;
    const int64_t piece = int64_t(k) * 64 + lane;
    if (or_into) {
      u32x4* q = reinterpret_cast<u32x4*>(or_into + id_base) + piece;
      *q = *q | v[k];
    }
    p[piece] = u32x4{0u, 0u, 0u, 0u};
    uint32_t x = m[k];
    const int64_t id0 = id_base + piece * 16;
    while (x) {
      const int b = __ffs(int(x)) - 1;
      const int32_t id = int32_t(id0 + b);
      if (WITH_OUT) {
        if (my < out_cap) out[my] = id;
        ++my;
      }
      if (bump) atomicAdd(&bump[id], 1u);
      x &= x - 1;
    }
  }
}

}  // namespace

void launch_compact(const DeviceInfo& di, uint8_t* map, uint8_t* or_into, int64_t n_chunks, int32_t* chunk_counts,
                    int32_t* out, int64_t out_cap, int32_t* n_out, uint32_t* bump, uint32_t* d_err, hipStream_t s) {
  (void)di;
  if (n_out) {
    hipLaunchKernelGGL(count_marks_kernel, dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, map, chunk_counts);
    hipLaunchKernelGGL((emit_marks_kernel<true>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, map, or_into,
                       chunk_counts, out, out_cap, n_out, bump, d_err);
  } else {
    hipLaunchKernelGGL((emit_marks_kernel<false>), dim3(unsigned(n_chunks)), dim3(kCompactThreads), 0, s, map,
                       or_into, chunk_counts, out, out_cap, n_out, bump, d_err);
  }
}

}  // namespace lgp
