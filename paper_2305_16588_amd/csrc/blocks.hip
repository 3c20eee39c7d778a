// Graph constructor (Sec. 5, operator 4): turn the sampled results into one bipartite CSR
// block per hop in local numbering.  Frontiers are ascending unique id lists, so "position
// of vertex u in a frontier" is served by a V-entry table that is scattered with the
// frontier's positions and then read once per sampled edge: two independent random
// accesses per element instead of a dependent binary-search chain.  A table is never
// cleared -- only entries written for the current frontier are ever read.  There is one
// table per list (the extracted id list and every frontier after the seeds), so all hops go
// through the same four launches, each covering its lists through blockIdx.y: scatter
// positions, per-tile edge counts, offsets, then feature rows + relabelled sources.
#include "common.hpp"

#include <algorithm>

namespace lgp {
namespace {

__device__ __forceinline__ int64_t clamped(const int32_t* n_dev, int64_t cap) {
  const int64_t n = *n_dev;
  return n > cap ? cap : n;
}

// blockIdx.y = 0: positions inside the extracted id list go to table 0; y = j >= 1: positions
// inside frontier j go to table j.
__global__ void scatter_pos_kernel(BlocksArgs a) {
  const int j = blockIdx.y;
  const int32_t* ids = j == 0 ? a.gather_ids : a.frontier[j];
  const int64_t n = j == 0 ? clamped(a.n_gather, a.gather_cap) : clamped(a.n_frontier + j, a.cap[j]);
  int32_t* table = a.table + int64_t(j) * a.num_vertices;
  for (int64_t k = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += int64_t(gridDim.x) * blockDim.x)
    table[ids[k]] = int32_t(k);   // ids come out of the dedup compaction: always in range
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

// blockIdx.y = hop.  Edge count of every tile of kScanTile destinations.
__global__ __launch_bounds__(256) void tile_sums_kernel(BlocksArgs a) {
  const int h = blockIdx.y;
  const int64_t n = clamped(a.n_frontier + h, a.cap[h]);
  const int64_t tile0 = int64_t(blockIdx.x) * kScanTile;
  if (tile0 > n) return;
  const int32_t* cnt = a.cnt[h];
  const int64_t base = tile0 + int64_t(threadIdx.x) * 4;
  int64_t mine = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (base + q < n) mine += cnt[base + q];
  int64_t total;
  block_exclusive_scan64(mine, &total);
  if (threadIdx.x == 0) a.tile_sums[a.tile_base[h] + blockIdx.x] = total;
}

// blockIdx.y = hop.  blk_indptr[i] = cnt[0] + ... + cnt[i - 1] for i <= n (64-bit sums).
__global__ __launch_bounds__(256) void offsets_kernel(BlocksArgs a) {
  const int h = blockIdx.y;
  const int64_t n = clamped(a.n_frontier + h, a.cap[h]);
  const int64_t tile0 = int64_t(blockIdx.x) * kScanTile;
  if (tile0 > n) return;                                 // tile0 == n still writes indptr[n]
  const int32_t* cnt = a.cnt[h];
  const int64_t* tile_sums = a.tile_sums + a.tile_base[h];
  int64_t* indptr = a.blk_indptr[h];
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

// blockIdx.y = j <= n_hops: feat_row[j][i] = position of frontier j's vertex i in the extracted
// id list (table 0).  y = n_hops + 1 + h: blk_src of hop h = positions of its samples in
// frontier h + 1 (table h + 1), packed at the offsets of blk_indptr[h].
__global__ __launch_bounds__(256) void lookup_relabel_kernel(BlocksArgs a) {
  const int y = blockIdx.y;
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  const int64_t first = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (y <= a.n_hops) {
    const int32_t* ids = a.frontier[y];
    int32_t* out = a.feat_row[y];
    const int64_t n = clamped(a.n_frontier + y, a.cap[y]);
    for (int64_t i = first; i < n; i += stride) {
      const int32_t v = ids[i];
      out[i] = uint32_t(v) < uint64_t(a.num_vertices) ? a.table[v] : -1;   // an invalid seed has no row
    }
  } else {
    const int h = y - a.n_hops - 1;
    const int32_t f = a.fanout[h];
    const int32_t* nbr = a.nbr[h];
    const int64_t* indptr = a.blk_indptr[h];
    const int32_t* table = a.table + int64_t(h + 1) * a.num_vertices;
    int32_t* blk_src = a.blk_src[h];
    const int64_t total = clamped(a.n_frontier + h, a.cap[h]) * f;
    for (int64_t t = first; t < total; t += stride) {
      const int32_t u = nbr[t];
      if (u < 0) continue;                                 // padding: valid samples fill the front of a row
      const int64_t i = t / f;
      blk_src[indptr[i] + (t - i * f)] = table[u];
    }
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

void launch_build_blocks(const DeviceInfo& di, const BlocksArgs& a, hipStream_t s) {
  const int L = a.n_hops;
  int64_t max_list = a.gather_cap, max_tiles = 1, max_work = 1;
  for (int h = 0; h <= L; ++h) {
    if (h >= 1) max_list = std::max(max_list, a.cap[h]);
    max_work = std::max(max_work, a.cap[h]);
    if (h < L) {
      max_tiles = std::max(max_tiles, a.cap[h] / kScanTile + 1);   // one more so that indptr[n] is written when n % tile == 0
      max_work = std::max(max_work, a.cap[h] * a.fanout[h]);
    }
  }
  hipLaunchKernelGGL(scatter_pos_kernel, dim3(grid_for(di, max_list), unsigned(L + 1)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(tile_sums_kernel, dim3(unsigned(max_tiles), unsigned(L)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(offsets_kernel, dim3(unsigned(max_tiles), unsigned(L)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(lookup_relabel_kernel, dim3(grid_for(di, max_work), unsigned(2 * L + 1)), dim3(256), 0, s, a);
}

}  // namespace lgp
