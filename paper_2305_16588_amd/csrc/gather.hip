// Feature extractor (Sec. 2.2 step 3; Sec. 5 "feature extractor") for gfx950:
// cache lookup + hit/miss partition, then two row-gather launches -- hits move
// HBM -> HBM, misses are read in place from CPU memory over PCIe.
//
// Row gather: a wavefront takes 64 list entries (one coalesced load of the row / source
// indices), then walks the 64 rows as one flat run of 16-byte chunks, so every lane
// issues 128-bit loads and stores, a row of any 16-byte-multiple width keeps all lanes
// busy, and several loads per lane are in flight before the first store.  The
// (row, source) pair a chunk belongs to is fetched from the owning lane by a
// cross-lane read, the LDS-crossbar path (ds_bpermute) -- the rows themselves never
// need to sit in LDS because a chunk is loaded and stored by the same lane.
#include "common.hpp"

namespace lgp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__global__ void zero_counters_kernel(int32_t* counters) {
  if (threadIdx.x < 2) counters[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void partition_kernel(
    const int32_t* __restrict__ ids, int64_t n_max, const int32_t* __restrict__ n_dev,
    const int32_t* __restrict__ f_remap, int64_t num_vertices, int32_t* __restrict__ hit_row,
    int32_t* __restrict__ hit_src, int32_t* __restrict__ miss_row, int32_t* __restrict__ miss_src,
    int32_t* __restrict__ counters, uint32_t* __restrict__ d_err) {
  int64_t n = n_dev ? int64_t(*n_dev) : n_max;
  if (n > n_max) n = n_max;
  const int lane = threadIdx.x & 63;
  const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int64_t base = int64_t(blockIdx.x) * 256; base < n; base += int64_t(gridDim.x) * 256) {
    const int64_t i = base + threadIdx.x;
    const bool active = i < n;
    const int32_t id = active ? ids[i] : 0;
    const bool ok = active && uint32_t(id) < uint64_t(num_vertices);
    if (active && !ok) atomicOr(d_err, ERR_BAD_ID);
    const int32_t slot = ok ? f_remap[id] : -1;
    const bool hit = ok && slot >= 0;
    const bool miss = ok && slot < 0;
    const uint64_t hm = __ballot(hit), mm = __ballot(miss);
    int hbase = 0, mbase = 0;
    if (lane == 0) {
      if (hm) hbase = atomicAdd(&counters[0], __popcll(hm));
      if (mm) mbase = atomicAdd(&counters[1], __popcll(mm));
    }
    hbase = __shfl(hbase, 0, 64);
    mbase = __shfl(mbase, 0, 64);
    if (hit) {
      const int pos = hbase + __popcll(hm & lower);
      hit_row[pos] = int32_t(i);
      hit_src[pos] = slot;
    } else if (miss) {
      const int pos = mbase + __popcll(mm & lower);
      miss_row[pos] = int32_t(i);
      miss_src[pos] = id;
    }
  }
}

template <typename VecT, bool STREAMING>
__device__ __forceinline__ VecT load_chunk(const VecT* p) {
  if (STREAMING) return __builtin_nontemporal_load(p);
  return *p;
}

template <typename VecT, int UNROLL, bool STREAMING>
__global__ __launch_bounds__(256) void gather_rows_kernel(const VecT* __restrict__ src, VecT* __restrict__ dst,
                                                          uint32_t cpr, uint64_t inv_cpr,
                                                          const int32_t* __restrict__ row,
                                                          const int32_t* __restrict__ srcrow, int64_t n_max,
                                                          const int32_t* __restrict__ n_dev) {
  int64_t n = n_dev ? int64_t(*n_dev) : n_max;
  if (n > n_max) n = n_max;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t(blockIdx.x) * 256 + threadIdx.x) >> 6;
  const int64_t n_waves = int64_t(gridDim.x) * 4;
  for (int64_t e0 = wave * 64; e0 < n; e0 += n_waves * 64) {
    const int64_t e = e0 + lane;
    const int32_t my_row = e < n ? (row ? row[e] : int32_t(e)) : 0;
    const int32_t my_src = e < n ? srcrow[e] : 0;
    const uint32_t entries = uint32_t(n - e0 < 64 ? n - e0 : 64);
    const uint32_t total = entries * cpr;          // chunks in this wave's 64 rows
    for (uint32_t f0 = 0; f0 < total; f0 += 64 * UNROLL) {
      VecT val[UNROLL];
      int64_t doff[UNROLL];
      bool ok[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t flat = f0 + u * 64 + lane;
        ok[u] = flat < total;
        const uint32_t k = ok[u] ? uint32_t((uint64_t(flat) * inv_cpr) >> 32) : 0u;   // flat / cpr
        const uint32_t col = flat - k * cpr;
        const int32_t r = __shfl(my_row, int(k), 64);
        const int32_t sr = __shfl(my_src, int(k), 64);
        doff[u] = int64_t(r) * cpr + col;
        if (ok[u]) val[u] = load_chunk<VecT, STREAMING>(src + (int64_t(sr) * cpr + col));
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (ok[u]) dst[doff[u]] = val[u];
    }
  }
}

template <typename VecT, int UNROLL>
void launch_rows(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                 const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, bool streaming, hipStream_t s) {
  const uint32_t cpr = uint32_t(row_bytes / int64_t(sizeof(VecT)));
  const uint64_t inv = (uint64_t(1) << 32) / cpr + 1;          // exact for flat < 64 * cpr, cpr <= 4096
  int64_t blocks = (n_max + 255) / 256;                        // one wave per 64 rows
  const int64_t full = int64_t(di.num_cus) * 8;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  if (streaming)
    hipLaunchKernelGGL((gather_rows_kernel<VecT, UNROLL, true>), dim3(unsigned(blocks)), dim3(256), 0, s,
                       static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, inv, row, srcrow, n_max, n_dev);
  else
    hipLaunchKernelGGL((gather_rows_kernel<VecT, UNROLL, false>), dim3(unsigned(blocks)), dim3(256), 0, s,
                       static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, inv, row, srcrow, n_max, n_dev);
}

__global__ void copy_i32_kernel(const int32_t* src, int32_t* dst, int n) {
  if (int(threadIdx.x) < n) dst[threadIdx.x] = src[threadIdx.x];
}

}  // namespace

void launch_partition(const DeviceInfo& di, const int32_t* ids, int64_t n_max, const int32_t* n_dev,
                      const int32_t* f_remap, int64_t num_vertices, int32_t* hit_row, int32_t* hit_src,
                      int32_t* miss_row, int32_t* miss_src, int32_t* counters, uint32_t* d_err, hipStream_t s) {
  hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, s, counters);
  int64_t blocks = (n_max + 255) / 256;
  const int64_t full = int64_t(di.num_cus) * 8;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(partition_kernel, dim3(unsigned(blocks)), dim3(256), 0, s, ids, n_max, n_dev, f_remap,
                     num_vertices, hit_row, hit_src, miss_row, miss_src, counters, d_err);
}

void launch_gather_rows(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                        const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, bool streaming, hipStream_t s) {
  if (n_max <= 0) return;
  const uintptr_t align = uintptr_t(src) | uintptr_t(dst) | uintptr_t(row_bytes);
  if ((align & 15u) == 0)
    launch_rows<u32x4, 4>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, streaming, s);
  else if ((align & 7u) == 0)
    launch_rows<u32x2, 4>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, streaming, s);
  else if ((align & 3u) == 0)
    launch_rows<uint32_t, 4>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, streaming, s);
  else
    launch_rows<uint16_t, 4>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, streaming, s);
}

void launch_copy_i32(const int32_t* src, int32_t* dst, int n, hipStream_t s) {
  hipLaunchKernelGGL(copy_i32_kernel, dim3(1), dim3(64), 0, s, src, dst, n);
}

}  // namespace lgp
