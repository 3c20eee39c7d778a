// Feature extractor (Sec. 2.2 step 3; Sec. 5 "feature extractor") for gfx950:
// cache lookup + hit/miss partition, then two row-gather launches -- hits move
// HBM -> HBM, misses are read in place from CPU memory over PCIe.
//
// Two row-gather kernels share the work.  The group kernel further down gives every row a
// group of lanes: it serves the misses, the cache fill and the hits on rows that straddle
// 128-byte lines.  The flat kernel serves hits on rows made of whole lines:
// a wavefront takes 64 list entries (one coalesced load of the row / source
// indices), then walks the 64 rows as one flat run of 16-byte chunks, so every lane
// issues 128-bit loads and stores, a row of any 16-byte-multiple width keeps all lanes
// busy, and several loads per lane are in flight before the first store.  The
// (row, source) pair a chunk belongs to is fetched from the owning lane by a
// cross-lane read, the LDS-crossbar path (ds_bpermute) -- the rows themselves never
// need to sit in LDS because a chunk is loaded and stored by the same lane.
#include "common.hpp"

#include <hip/hip_ext.h>

#include <algorithm>

namespace lgp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__global__ void zero_counters_kernel(int32_t* counters, int n) {
  if (int(threadIdx.x) < n) counters[threadIdx.x] = 0;
}

// Each wave looks up 4 x 64 consecutive ids; the workgroup reserves its share of every
// list with ONE atomic per list (the global counters are the only contended words), then
// every lane writes its entries at wave-ballot ranks, so the lists stay in ascending row
// order inside a workgroup.  List 0 = hits, list 1 = misses; with NL = 3 a hit whose slot lies
// outside [local_lo, local_hi) -- another clique member's region of the cache -- goes to list 2.
constexpr int kPartItems = 4;
template <int NL>
__global__ __launch_bounds__(256) void partition_kernel(
    const int32_t* __restrict__ ids, int64_t n_max, const int32_t* __restrict__ n_dev,
    const int32_t* __restrict__ f_remap, int64_t num_vertices, PartLists out, int32_t local_lo, int32_t local_hi,
    int32_t* __restrict__ counters, uint32_t* __restrict__ d_err, const int32_t* __restrict__ window) {
  __shared__ int wave_cnt[NL][4], block_base[NL];
  int64_t n = n_dev ? int64_t(*n_dev) : n_max;
  int64_t lo = 0;
  if (window) {                                     // entries [window[0], window[1]) of ids
    lo = window[0] < 0 ? 0 : window[0];
    n = window[1];
  }
  if (n > n_max) n = n_max;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  constexpr int kTile = 256 * kPartItems;
  for (int64_t base = lo + int64_t(blockIdx.x) * kTile; base < n; base += int64_t(gridDim.x) * kTile) {
    int32_t src[kPartItems];
    uint64_t mask[NL][kPartItems];
    int cnt[NL];
#pragma unroll
    for (int l = 0; l < NL; ++l) cnt[l] = 0;
#pragma unroll
    for (int j = 0; j < kPartItems; ++j) {
      const int64_t i = base + wave * (64 * kPartItems) + j * 64 + lane;
      const bool active = i < n;
      const int32_t id = active ? ids[i] : 0;
      const bool ok = active && uint32_t(id) < uint64_t(num_vertices);
      if (active && !ok) atomicOr(d_err, ERR_BAD_ID);
      const int32_t slot = ok ? f_remap[id] : -1;
      int which = -1;                               // list of this entry
      if (ok) which = slot < 0 ? 1 : (NL == 3 && (slot < local_lo || slot >= local_hi)) ? 2 : 0;
      src[j] = which == 1 ? id : slot;
#pragma unroll
      for (int l = 0; l < NL; ++l) {
        mask[l][j] = __ballot(which == l);
        cnt[l] += __popcll(mask[l][j]);
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int l = 0; l < NL; ++l) wave_cnt[l][wave] = cnt[l];
    }
    __syncthreads();
    if (threadIdx.x < NL) {
      const int l = threadIdx.x;
      const int t = wave_cnt[l][0] + wave_cnt[l][1] + wave_cnt[l][2] + wave_cnt[l][3];
      block_base[l] = t ? atomicAdd(&counters[l], t) : 0;
    }
    __syncthreads();
    int pos[NL];
#pragma unroll
    for (int l = 0; l < NL; ++l) {
      pos[l] = block_base[l];
      for (int w = 0; w < wave; ++w) pos[l] += wave_cnt[l][w];
    }
#pragma unroll
    for (int j = 0; j < kPartItems; ++j) {
      const int64_t i = base + wave * (64 * kPartItems) + j * 64 + lane;
      const uint64_t bit = 1ull << lane;
#pragma unroll
      for (int l = 0; l < NL; ++l) {
        if (mask[l][j] & bit) {
          const int at = pos[l] + __popcll(mask[l][j] & lower);
          out.row[l][at] = int32_t(i);
          out.src[l][at] = src[j];
        }
        pos[l] += __popcll(mask[l][j]);
      }
    }
    __syncthreads();                               // LDS is reused by the next tile
  }
}

__device__ __forceinline__ void direct_stats(const DirectIds& dir, int64_t n) {
  if (dir.stats && blockIdx.x == 0 && threadIdx.x == 0) {
    dir.stats[dir.stats_slot] = int32_t(n > 0 ? n : 0);
    dir.stats[1 - dir.stats_slot] = 0;
  }
}

// Translate one entry of the source-row array; -1 = skip this row.
__device__ __forceinline__ int32_t direct_source(const DirectIds& dir, int32_t entry, bool in_range) {
  if (dir.num_vertices == 0 || !in_range) return in_range ? entry : -1;
  if (uint32_t(entry) >= uint64_t(dir.num_vertices)) {
    atomicOr(dir.d_err, ERR_BAD_ID);
    return -1;
  }
  return dir.remap ? dir.remap[entry] : entry;
}

// ---- cache hits: HBM -> HBM ------------------------------------------------
// A wavefront takes 64 list entries and walks their rows as one flat run of chunks:
// all 64 lanes stay busy for any row width and UNROLL loads per lane are in flight
// before the first store.  Output rows are written once and not read again by this
// path, so they are stored non-temporally.
template <typename VecT, int UNROLL, bool NT_LOAD>
__global__ __launch_bounds__(256) void gather_rows_flat_kernel(const VecT* __restrict__ src, VecT* __restrict__ dst,
                                                               uint32_t cpr, uint64_t inv_cpr,
                                                               const int32_t* __restrict__ row,
                                                               const int32_t* __restrict__ srcrow, int64_t n_max,
                                                               const int32_t* __restrict__ n_dev, DirectIds dir,
                                                               int epw) {
  int64_t n = n_dev ? int64_t(*n_dev) : n_max;
  int64_t lo = 0;
  if (dir.window) {                                 // entries [window[0], window[1]) only
    lo = dir.window[0] < 0 ? 0 : dir.window[0];
    n = dir.window[1];
  }
  if (n > n_max) n = n_max;
  direct_stats(dir, n - lo);
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t(blockIdx.x) * 256 + threadIdx.x) >> 6;
  const int64_t n_waves = int64_t(gridDim.x) * 4;
  // epw (<= 64) list entries per wave and pass: fewer for wide rows, so that a pass moves a few tens of
  // KiB and the passes spread evenly over the waves whatever the (device-side) number of entries is
  for (int64_t e0 = lo + wave * epw; e0 < n; e0 += n_waves * epw) {
    const int64_t e = e0 + lane;
    const bool mine = lane < epw && e < n;
    const int32_t my_row = mine ? (row ? row[e] : int32_t(e)) : 0;
    const int32_t my_src = direct_source(dir, mine ? (srcrow ? srcrow[e] : int32_t(e)) : 0, mine);
    const uint32_t entries = uint32_t(n - e0 < epw ? n - e0 : epw);
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
        ok[u] = ok[u] && sr >= 0;
        doff[u] = int64_t(r) * cpr + col;
        if (ok[u])
          val[u] = NT_LOAD ? __builtin_nontemporal_load(src + int64_t(sr) * cpr + col) : src[int64_t(sr) * cpr + col];
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (ok[u]) __builtin_nontemporal_store(val[u], dst + doff[u]);
    }
  }
}

// ---- cache misses and cache fill: CPU memory -> HBM over PCIe ---------------
// Reads of CPU memory are not cached on the GPU and travel as whole 128-byte lines, so
// a line requested by two different load instructions crosses the link twice.  Here a
// group of G >= chunks-per-row lanes owns a whole row, so one instruction requests each
// line of the row exactly once; UNROLL rows per group are in flight before the first
// store.  Rows wider than 64 chunks are walked in 64-chunk pieces.  HBM_SOURCE selects the
// variant used for cache hits on rows that straddle lines (cached loads, streaming stores).
template <typename VecT, int G, int UNROLL, bool HBM_SOURCE>
__global__ __launch_bounds__(256) void gather_rows_group_kernel(const VecT* __restrict__ src, VecT* __restrict__ dst,
                                                                uint32_t cpr, const int32_t* __restrict__ row,
                                                                const int32_t* __restrict__ srcrow, int64_t n_max,
                                                                const int32_t* __restrict__ n_dev, DirectIds dir) {
  int64_t n = n_dev ? int64_t(*n_dev) : n_max;
  int64_t lo = 0;
  if (dir.window) {
    lo = dir.window[0] < 0 ? 0 : dir.window[0];
    n = dir.window[1];
  }
  if (n > n_max) n = n_max;
  direct_stats(dir, n - lo);
  const uint32_t sub = threadIdx.x % G;
  const int64_t group = (int64_t(blockIdx.x) * 256 + threadIdx.x) / G;
  const int64_t n_groups = int64_t(gridDim.x) * (256 / G);
  // The list entries of the next pass are loaded before the rows of this one, so that a pass waits
  // for one round trip to memory (its rows), not two in a row (entries, then rows).
  int32_t next_src[UNROLL], next_row[UNROLL];
  const int64_t first = lo + group * UNROLL;
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const int64_t e = first + u;
    next_src[u] = e < n ? (srcrow ? srcrow[e] : int32_t(e)) : 0;
    next_row[u] = e < n ? (row ? row[e] : int32_t(e)) : 0;
  }
  for (int64_t e0 = first; e0 < n; e0 += n_groups * UNROLL) {
    int64_t so[UNROLL], dof[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const bool ok = e0 + u < n;
      const int32_t sr = direct_source(dir, next_src[u], ok);
      so[u] = sr >= 0 ? int64_t(sr) * cpr : -1;
      dof[u] = int64_t(next_row[u]) * cpr;
      const int64_t e = e0 + n_groups * UNROLL + u;
      next_src[u] = e < n ? (srcrow ? srcrow[e] : int32_t(e)) : 0;
      next_row[u] = e < n ? (row ? row[e] : int32_t(e)) : 0;
    }
    for (uint32_t c0 = 0; c0 < cpr; c0 += G) {
      const uint32_t col = c0 + sub;
      VecT val[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (so[u] >= 0 && col < cpr) val[u] = HBM_SOURCE ? src[so[u] + col] : __builtin_nontemporal_load(src + so[u] + col);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        if (so[u] >= 0 && col < cpr) {
          if (HBM_SOURCE) __builtin_nontemporal_store(val[u], dst + dof[u] + col);
          else dst[dof[u] + col] = val[u];
        }
    }
  }
}

inline unsigned blocks_for(int64_t work_blocks, int64_t limit) {
  int64_t b = work_blocks < limit ? work_blocks : limit;
  return unsigned(b < 1 ? 1 : b);
}

// Where a gather kernel is launched: on stream s, and -- when a and b are given -- with its own start
// and stop times recorded into those two events (hipExtLaunchKernelGGL), which costs no extra packets
// on the stream, unlike a pair of hipEventRecord calls around the launch.
struct Where {
  hipStream_t s;
  hipEvent_t a, b;
  int64_t hbm_blocks;   // most workgroups an HBM-bound gather may use
  int64_t items;        // entries to size the grid for (<= n_max: a window covers part of the array)
};

template <typename K, typename... Args>
void launch_on(const Where& w, K kernel, unsigned blocks, Args... args) {
  if (w.a && w.b) hipExtLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, w.s, w.a, w.b, 0, args...);
  else hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, w.s, args...);
}

template <typename VecT>
void launch_flat(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                 const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, const DirectIds& dir, const Where& s) {
  const uint32_t cpr = uint32_t(row_bytes / int64_t(sizeof(VecT)));
  const uint64_t inv = (uint64_t(1) << 32) / cpr + 1;          // exact for flat < 64 * cpr, cpr <= 4096
  // Three workgroups (12 waves) per CU: the flat walk keeps 4 x 16 bytes per lane in flight, and more
  // waves than that only add concurrent streams for the memory system to interleave -- measured hit
  // gather at 8 / 4 / 3 / 2 workgroups per CU: 51.3 / 48.9 / 48.3 / 49.0 us on 505 k 256-byte rows,
  // 163.1 / 157.4 / 155.3 / 156.5 us on 855 k 512-byte rows, 335.7 / 315.3 / 310.4 / 307.2 us on 379 k
  // 2-KiB rows.  A narrower gather also leaves room for a sampler running beside it on another stream.
  // A wave takes at most 32 KiB of rows per pass (64 rows of up to 512 bytes, 16 rows of 2 KiB): the number
  // of entries is only known on the device, and with 128 KiB passes a launch of 233 k 2-KiB rows left most
  // waves with one pass and a few with two (216.6 -> 195.7 us; 379 k such rows: 311.5 -> 263.8 us).
  int epw = 64;
  while (epw > 4 && int64_t(epw) * row_bytes > 32768) epw >>= 1;
  const unsigned blocks = blocks_for((s.items + 4 * epw - 1) / (4 * epw), std::min<int64_t>(s.hbm_blocks, int64_t(di.num_cus) * 3));
  // Rows made of whole 128-byte lines are read once: stream them past L2 (+2.5 % at 512-B and 2-KiB
  // rows).  Rows that straddle lines share their boundary lines between consecutive load
  // instructions, and L2 has to merge those (non-temporal loads cost 7 % on 400-B rows).
  if (row_bytes % 128 == 0)
    launch_on(s, gather_rows_flat_kernel<VecT, 4, true>, blocks,
                       static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, inv, row, srcrow, n_max, n_dev, dir, epw);
  else
    launch_on(s, gather_rows_flat_kernel<VecT, 4, false>, blocks,
                       static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, inv, row, srcrow, n_max, n_dev, dir, epw);
}

template <typename VecT, int G>
void launch_group_g(const DeviceInfo& di, const void* src, void* dst, uint32_t cpr, const int32_t* row,
                    const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, const DirectIds& dir, const Where& s) {
  constexpr int U = 4;
  // PCIe needs far fewer waves than HBM to stay saturated (bandwidth x latency is ~150 KB): one
  // workgroup per four CUs holds ~1 MB of reads in flight, and measured rates FALL with wider grids
  // (400-B rows 44.9 -> 44.0 GB/s, 2-KiB rows 57.5 -> 55.7 GB/s from 64 to 512 workgroups), because the
  // excess requests only queue up in front of the link.
  const unsigned blocks = blocks_for((s.items + (256 / G) * U - 1) / ((256 / G) * U), std::max(1, di.num_cus / 4));
  launch_on(s, gather_rows_group_kernel<VecT, G, U, false>, blocks,
                     static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, row, srcrow, n_max, n_dev, dir);
}

// Cache hits whose rows straddle 128-byte lines (e.g. 400-byte rows): one lane group per row, one
// row per group in flight.  Every line of a row is then requested by a single load instruction,
// which beats the flat walk by ~5 % on such rows; rows made of whole lines stay with the flat kernel.
template <typename VecT, int G>
void launch_group_hbm_g(const DeviceInfo& di, const void* src, void* dst, uint32_t cpr, const int32_t* row,
                        const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, const DirectIds& dir,
                        const Where& s) {
  // one row per group in flight needs more waves than the flat walk: 6 workgroups per CU (400-byte rows,
  // 512 k hits: 138.7 / 107.6 / 95.6 / 90.7 / 91.4 us at 2 / 3 / 4 / 6 / 8 workgroups per CU)
  const unsigned blocks = blocks_for((s.items + 256 / G - 1) / (256 / G), std::min<int64_t>(s.hbm_blocks, int64_t(di.num_cus) * 6));
  launch_on(s, gather_rows_group_kernel<VecT, G, 1, true>, blocks,
                     static_cast<const VecT*>(src), static_cast<VecT*>(dst), cpr, row, srcrow, n_max, n_dev, dir);
}

template <typename VecT>
void launch_group_hbm(const DeviceInfo& di, const void* src, void* dst, uint32_t cpr, const int32_t* row,
                      const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, const DirectIds& dir, const Where& s) {
  if (cpr <= 4) launch_group_hbm_g<VecT, 4>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else if (cpr <= 8) launch_group_hbm_g<VecT, 8>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else if (cpr <= 16) launch_group_hbm_g<VecT, 16>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else launch_group_hbm_g<VecT, 32>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
}

template <typename VecT>
void launch_group(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                  const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, const DirectIds& dir, const Where& s) {
  const uint32_t cpr = uint32_t(row_bytes / int64_t(sizeof(VecT)));
  if (cpr <= 4) launch_group_g<VecT, 4>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else if (cpr <= 8) launch_group_g<VecT, 8>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else if (cpr <= 16) launch_group_g<VecT, 16>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else if (cpr <= 32) launch_group_g<VecT, 32>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
  else launch_group_g<VecT, 64>(di, src, dst, cpr, row, srcrow, n_max, n_dev, dir, s);
}

}  // namespace

void launch_partition(const DeviceInfo& di, const int32_t* ids, int64_t n_max, const int32_t* n_dev,
                      const int32_t* f_remap, int64_t num_vertices, const PartLists& out, int n_lists,
                      int32_t local_lo, int32_t local_hi, int32_t* counters, uint32_t* d_err, hipStream_t s,
                      const int32_t* window, int64_t grid_items) {
  const bool three = n_lists == 3;
  hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, s, counters, three ? 3 : 2);
  const int64_t items = (window && grid_items > 0 && grid_items < n_max) ? grid_items : n_max;
  int64_t blocks = (items + 256 * kPartItems - 1) / (256 * kPartItems);
  const int64_t full = int64_t(di.num_cus) * 8;
  if (blocks > full) blocks = full;
  if (blocks < 1) blocks = 1;
  if (three)
    hipLaunchKernelGGL(partition_kernel<3>, dim3(unsigned(blocks)), dim3(256), 0, s, ids, n_max, n_dev, f_remap,
                       num_vertices, out, local_lo, local_hi, counters, d_err, window);
  else
    hipLaunchKernelGGL(partition_kernel<2>, dim3(unsigned(blocks)), dim3(256), 0, s, ids, n_max, n_dev, f_remap,
                       num_vertices, out, 0, 0, counters, d_err, window);
}

void launch_gather_rows(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                        const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, bool streaming, hipStream_t stream,
                        const DirectIds& dir, hipEvent_t ev_start, hipEvent_t ev_stop, bool beside_pcie,
                        int64_t grid_items) {
  if (n_max <= 0) return;
  // An HBM-bound gather is capped at 8 workgroups per CU (each kernel narrows that further).  One that runs beside a
  // PCIe-bound kernel is throttled by the PCIe reads queued ahead of it whatever its width, and
  // in turn delays them; two workgroups per CU keep it out of the link's way (measured on 400-byte
  // rows, 506 k hits beside 253 k misses: the miss gather takes 2.40 ms beside a full-width hit
  // gather, 2.24 ms beside a narrow one, and the step 2.49 ms instead of 2.66 ms).
  const Where s{stream, ev_start, ev_stop, int64_t(di.num_cus) * (beside_pcie ? 2 : 8),
                (grid_items > 0 && grid_items < n_max) ? grid_items : n_max};
  const uintptr_t align = uintptr_t(src) | uintptr_t(dst) | uintptr_t(row_bytes);
#define LGP_ROWS(VecT)                                                                        \
  do {                                                                                        \
    if (streaming) launch_group<VecT>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, dir, s); \
    else if (row_bytes % 128 != 0 && row_bytes / sizeof(VecT) <= 32)                               \
      launch_group_hbm<VecT>(di, src, dst, uint32_t(row_bytes / sizeof(VecT)), row, srcrow, n_max, n_dev, dir, s); \
    else launch_flat<VecT>(di, src, dst, row_bytes, row, srcrow, n_max, n_dev, dir, s);            \
  } while (0)
  if ((align & 15u) == 0) LGP_ROWS(u32x4);
  else if ((align & 7u) == 0) LGP_ROWS(u32x2);
  else if ((align & 3u) == 0) LGP_ROWS(uint32_t);
  else LGP_ROWS(uint16_t);
#undef LGP_ROWS
}

}  // namespace lgp
