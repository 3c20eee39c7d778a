// Graph constructor (Sec. 5, operator 4): turn the sampled results into one bipartite CSR
// block per hop in local numbering.  Frontiers are ascending unique id lists, so "position
// of vertex u in a frontier" is served by a V-entry table that is scattered with the
// frontier's positions and then read once per sampled edge: two independent random
// accesses per element instead of a dependent binary-search chain.  The table is never
// cleared -- only entries written for the current frontier are ever read.
#include "common.hpp"

namespace lgp {
namespace {

__global__ void scatter_pos_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev, int64_t cap,
                                   int32_t* __restrict__ table) {
  int64_t n = *n_dev;
  if (n > cap) n = cap;
  for (int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; j < n; j += int64_t(gridDim.x) * blockDim.x)
    table[ids[j]] = int32_t(j);   // ids come out of the dedup compaction: always in range
}

__global__ void lookup_pos_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev, int64_t cap,
                                  const int32_t* __restrict__ table, int64_t num_vertices,
                                  int32_t* __restrict__ out) {
  int64_t n = *n_dev;
  if (n > cap) n = cap;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += int64_t(gridDim.x) * blockDim.x) {
    const int32_t v = ids[i];
    out[i] = uint32_t(v) < uint64_t(num_vertices) ? table[v] : -1;   // an invalid seed has no row
  }
}

__device__ __forceinline__ int64_t wave_inclusive_scan64(int64_t x) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int64_t y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  return x;
}

// Sum of one value per thread over a 256-thread workgroup (everyone gets the total) and the
// exclusive prefix of the calling thread.
__device__ __forceinline__ int64_t block_exclusive_scan64(int64_t x, int64_t* total) {
  __shared__ int64_t wave_sum[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t inc = wave_inclusive_scan64(x);
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  int64_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int64_t sw = wave_sum[w];
    if (w < wave) before += sw;
    all += sw;
  }
  __syncthreads();
  *total = all;
  return before + inc - x;
}

__global__ __launch_bounds__(256) void tile_sums_kernel(const int32_t* __restrict__ cnt,
                                                        const int32_t* __restrict__ n_dev, int64_t cap,
                                                        int64_t* __restrict__ tile_sums) {
  int64_t n = *n_dev;
  if (n > cap) n = cap;
  const int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * 4;
  int64_t mine = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (base + q < n) mine += cnt[base + q];
  int64_t total;
  block_exclusive_scan64(mine, &total);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void offsets_kernel(const int32_t* __restrict__ cnt,
                                                      const int32_t* __restrict__ n_dev, int64_t cap,
                                                      const int64_t* __restrict__ tile_sums,
                                                      int64_t* __restrict__ indptr) {
  int64_t n = *n_dev;
  if (n > cap) n = cap;
  const int64_t tile0 = int64_t(blockIdx.x) * kScanTile;
  if (tile0 > n) return;                                 // tile0 == n still writes indptr[n]
  int64_t part = 0;
  for (int64_t k = threadIdx.x; k < int64_t(blockIdx.x); k += 256) part += tile_sums[k];
  int64_t before_tiles;
  block_exclusive_scan64(part, &before_tiles);
  const int64_t base = tile0 + int64_t(threadIdx.x) * 4;
  int32_t c[4];
  int64_t mine = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    c[q] = base + q < n ? cnt[base + q] : 0;
    mine += c[q];
  }
  int64_t tile_total;
  int64_t run = before_tiles + block_exclusive_scan64(mine, &tile_total);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (base + q <= n) indptr[base + q] = run;             // entry n holds the edge total
    run += c[q];
  }
}

__global__ __launch_bounds__(256) void relabel_kernel(const int32_t* __restrict__ nbr,
                                                      const int64_t* __restrict__ indptr, int32_t f,
                                                      const int32_t* __restrict__ n_dev, int64_t cap,
                                                      const int32_t* __restrict__ table,
                                                      int32_t* __restrict__ blk_src) {
  int64_t n = *n_dev;
  if (n > cap) n = cap;
  const int64_t total = n * f;
  for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += int64_t(gridDim.x) * blockDim.x) {
    const int32_t u = nbr[t];
    if (u < 0) continue;                                   // padding: valid samples fill the front of a row
    const int64_t i = t / f;
    blk_src[indptr[i] + (t - i * f)] = table[u];
  }
}

inline unsigned grid_for(const DeviceInfo& di, int64_t n) {
  int64_t blocks = (n + 255) / 256;
  const int64_t full = int64_t(di.num_cus) * 8;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  return unsigned(blocks);
}

}  // namespace

void launch_scatter_pos(const DeviceInfo& di, const int32_t* ids, const int32_t* n_dev, int64_t cap, int32_t* table,
                        hipStream_t s) {
  hipLaunchKernelGGL(scatter_pos_kernel, dim3(grid_for(di, cap)), dim3(256), 0, s, ids, n_dev, cap, table);
}

void launch_lookup_pos(const DeviceInfo& di, const int32_t* ids, const int32_t* n_dev, int64_t cap,
                       const int32_t* table, int64_t num_vertices, int32_t* out, hipStream_t s) {
  hipLaunchKernelGGL(lookup_pos_kernel, dim3(grid_for(di, cap)), dim3(256), 0, s, ids, n_dev, cap, table, num_vertices,
                     out);
}

void launch_counts_to_offsets(const DeviceInfo& di, const int32_t* cnt, const int32_t* n_dev, int64_t cap,
                              int64_t* tile_sums, int64_t* indptr, hipStream_t s) {
  (void)di;
  const unsigned tiles = unsigned(cap / kScanTile + 1);   // one more so that indptr[n] is written when n % tile == 0
  hipLaunchKernelGGL(tile_sums_kernel, dim3(tiles), dim3(256), 0, s, cnt, n_dev, cap, tile_sums);
  hipLaunchKernelGGL(offsets_kernel, dim3(tiles), dim3(256), 0, s, cnt, n_dev, cap, tile_sums, indptr);
}

void launch_relabel(const DeviceInfo& di, const int32_t* nbr, const int64_t* indptr, int32_t fanout,
                    const int32_t* n_dev, int64_t cap, const int32_t* table, int32_t* blk_src, hipStream_t s) {
  hipLaunchKernelGGL(relabel_kernel, dim3(grid_for(di, cap * fanout)), dim3(256), 0, s, nbr, indptr, fanout, n_dev,
                     cap, table, blk_src);
}

}  // namespace lgp
