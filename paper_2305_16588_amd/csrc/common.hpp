// Internal declarations shared by the translation units of liblegion_prep.
// Host-side launchers only; kernels live in the .hip files.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "legion_prep.h"

namespace lgp {

// Device-side error bits (sticky, OR-ed into ctx->d_err).
enum : uint32_t { ERR_BAD_ID = 1u, ERR_OVERRUN = 2u };

// One dedup bitmap chunk = what one workgroup of the compaction kernels covers.
constexpr int kCompactThreads = 256;
constexpr int kWordsPerThread = 4;                                   // 64-bit words
constexpr int64_t kChunkWords = int64_t(kCompactThreads) * kWordsPerThread;
constexpr int64_t kChunkBits = kChunkWords * 64;                     // 65536 vertices per workgroup

// Vertex v is bit (v << spread_shift) of a dedup bitmap.  Every sample is one atomic OR on the
// bitmap, and atomics on the same cache line serialise; a graph whose plain bitmap is a few lines
// or a few hundred KB therefore gets a sparser one (measured: sampling 0.060 -> 0.031 ms at 10 k
// vertices with shift 5, 0.144 -> 0.134 ms at 2.4 M with shift 2; at 10 M and beyond any spreading
// only adds bytes to the compaction scans).
constexpr int kMaxSpreadShift = 5;
constexpr int64_t kSpreadTargetBits = int64_t(1) << 24;

struct DeviceInfo {
  int device = 0;
  int num_cus = 256;
  int spread_shift = 0;
};

// Row table: one 64-bit entry per vertex, resident in HBM, so that finding a vertex's adjacency
// costs one load whether or not the row is cached.
//   bit 63      1 = the row's column ids are in the topology cache, 0 = in CPU memory
//   bits 62..24 offset of the row's first column id inside that array (39 bits)
//   bits 23..0  degree; kRowDegOverflow means "too large to pack: use the CPU-resident CSR"
constexpr uint64_t kRowCachedBit = 1ull << 63;
constexpr uint32_t kRowDegOverflow = 0xFFFFFFu;
constexpr int kRowStartShift = 24;
constexpr uint64_t kRowStartMask = (1ull << 39) - 1;

// Pointers every sampling kernel needs.
struct TopoView {
  const uint64_t* row_tab;   // row table (HBM)
  const void* h_indptr;      // CPU-resident CSR (GPU-addressable); offsets only read for overflow rows
  const int32_t* h_indices;
  const int32_t* t_indices;  // cached column ids (HBM)
  int32_t indptr_bytes;
  int64_t num_vertices;
};

// ---- sampler.hip ----------------------------------------------------------
// Expand frontier[0 .. *n_frontier) with fan-out f at hop `hop`.  Writes nbr / cnt
// (either may be null), sets the bit of every sampled neighbour in `mark_bits` (bit v << di.spread_shift),
// adds cnt to topo_hot[v] if topo_hot is given.  With self_bits given (first hop) the
// frontier is the seed list: exactly `cap` ids, *n_frontier is written (= cap) instead of
// read, and every valid seed's own bit is set in self_bits.
void launch_sample_hop(const DeviceInfo& di, const TopoView& tv, const int32_t* frontier, int32_t* n_frontier,
                       int64_t cap, int32_t fanout, int32_t hop, uint64_t rng_seed, int32_t* nbr, int32_t* cnt,
                       uint32_t* mark_bits, uint32_t* self_bits, uint32_t* topo_hot, uint32_t* d_err, hipStream_t s);

// acc[0] += n[0] + ... + n[count - 1]   (frontier sizes of one pre-sampling batch)
void launch_accumulate_sizes(const int32_t* n, int32_t count, unsigned long long* acc, hipStream_t s);

// ---- compact.hip ----------------------------------------------------------
// Turn the bitmap `bits` (n_chunks * kChunkWords 64-bit words, vertex v at bit v << di.spread_shift)
// into the ascending id list out[0 .. *n_out).  If or_into is given, bits are OR-ed into it; `bits` is
// cleared.  If bump is given, bump[id] += 1 for every set bit.  With n_out == nullptr no
// list is produced: only the OR / clear / bump side effects happen.
void launch_compact(const DeviceInfo& di, uint64_t* bits, uint64_t* or_into, int64_t n_chunks, int32_t* chunk_counts,
                    int32_t* out, int64_t out_cap, int32_t* n_out, uint32_t* bump, uint32_t* d_err, hipStream_t s);

// Compaction for the intra-batch pipeline: like launch_compact(bits, or_into = seen, ...), and in addition the
// vertices marked in `bits` but not yet in `seen` -- the ones this hop reached first -- are appended, ascending,
// to listed[seg[0] ..], and seg[1] = seg[0] + their number (seg: device int32 pair).  With n_out == nullptr no
// frontier list is written; n_listed, if given, also receives seg[1].  new_counts: n_chunks ints of scratch.
void launch_compact_new(const DeviceInfo& di, uint64_t* bits, uint64_t* seen, int64_t n_chunks, int32_t* chunk_counts,
                        int32_t* new_counts, int32_t* out, int64_t out_cap, int32_t* n_out, int32_t* listed,
                        int64_t listed_cap, int32_t* seg, int32_t* n_listed, uint32_t* d_err, hipStream_t s);
// seg[0] = 0, seg[1] = n_seeds, listed[0 .. n_seeds) = seeds, counters[0 .. n_counters) = 0.
void launch_begin_listing(const DeviceInfo& di, const int32_t* seeds, int64_t n_seeds, int32_t* listed, int32_t* seg,
                          int32_t* counters, int32_t n_counters, hipStream_t s);
// stats[0 .. 2) = column sums of the n_seg x 3 matrix seg_counters (first two columns), one thread.
void launch_sum_stats(const int32_t* seg_counters, int32_t n_seg, int32_t* stats, hipStream_t s);

// ---- gather.hip -----------------------------------------------------------
// Look up every id in the feature remap and append (row, slot) to the hit list (list 0) or
// (row, id) to the miss list (list 1).  With n_lists = 3, hits whose slot lies outside
// [local_lo, local_hi) go to list 2 instead: rows cached by another member of a clique.
// counters[l] = entries of list l, l < n_lists (zeroed here).
struct PartLists {
  int32_t* row[3];
  int32_t* src[3];
};
void launch_partition(const DeviceInfo& di, const int32_t* ids, int64_t n_max, const int32_t* n_dev,
                      const int32_t* f_remap, int64_t num_vertices, const PartLists& out, int n_lists,
                      int32_t local_lo, int32_t local_hi, int32_t* counters, uint32_t* d_err, hipStream_t s,
                      const int32_t* window = nullptr, int64_t grid_items = 0);
// "Direct" launches skip the partition: when every row is cached (or none is) the source-row
// array is the caller's id list itself.
struct DirectIds {
  const int32_t* remap;   // id -> cache slot (everything cached); nullptr = the id is the source row (nothing cached)
  int64_t num_vertices;   // > 0: entries are vertex ids, validate them; 0: entries are trusted list entries
  int32_t* stats;         // {n_hit, n_miss} to fill in, or nullptr
  int32_t stats_slot;     // which of the two gets the row count
  uint32_t* d_err;
  const int32_t* window;  // device {begin, end}: only these entries of the array are gathered (nullptr = all)
};

// dst[row[e], :] = src[srcrow[e], :] for e < *n_dev (or n_max if n_dev is null); rows are
// row_bytes wide; `row` and `srcrow` may each be null (= e).  streaming = source is read once over
// PCIe (non-temporal loads, one lane group per row).
// With ev_start and ev_stop given (and n_max > 0) the kernel's own start and stop times are recorded
// into them.  beside_pcie: this HBM-bound gather runs at the same time as a PCIe-bound one.  With
// dir.window given, entries [window[0], window[1]) are gathered (their output rows keep their absolute
// numbers) and grid_items is the most entries the window can hold, for sizing the grid.
void launch_gather_rows(const DeviceInfo& di, const void* src, void* dst, int64_t row_bytes, const int32_t* row,
                        const int32_t* srcrow, int64_t n_max, const int32_t* n_dev, bool streaming, hipStream_t s,
                        const DirectIds& dir = DirectIds{nullptr, 0, nullptr, 0, nullptr, nullptr},
                        hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr, bool beside_pcie = false,
                        int64_t grid_items = 0);

// ---- blocks.hip -----------------------------------------------------------
constexpr int kScanTile = 1024;   // elements per workgroup of the counts -> offsets scan
// Everything one graph-constructor call reads and writes.  cap[h] = 0 marks a frontier that
// is empty in the worst case: its lists are not touched, its hop still gets blk_indptr[h][0] = 0.
struct BlocksArgs {
  int32_t n_hops;
  int64_t num_vertices;
  const int32_t* frontier[LGP_MAX_HOPS + 1];   // [0] = the seeds
  const int32_t* n_frontier;                   // device int32[n_hops + 1]
  int64_t cap[LGP_MAX_HOPS + 1];
  const int32_t* gather_ids;
  const int32_t* n_gather;
  int64_t gather_cap;
  const int32_t* nbr[LGP_MAX_HOPS];
  const int32_t* cnt[LGP_MAX_HOPS];
  int32_t fanout[LGP_MAX_HOPS];
  int64_t* blk_indptr[LGP_MAX_HOPS];
  int32_t* blk_src[LGP_MAX_HOPS];
  int32_t* feat_row[LGP_MAX_HOPS + 1];
  int32_t* table;                              // n_hops + 1 tables of num_vertices entries each
  int64_t* tile_sums;                          // hop h owns cap[h] / kScanTile + 1 entries from tile_base[h]
  int64_t tile_base[LGP_MAX_HOPS];
};
void launch_build_blocks(const DeviceInfo& di, const BlocksArgs& a, hipStream_t s);

// ---- cache.hip ------------------------------------------------------------
struct CachePlan {
  int64_t n_topo = 0, topo_edges = 0, n_feat = 0;
  uint64_t topo_bytes = 0, feat_bytes = 0;
};
// Rank vertices by (hotness descending, id ascending) into order[V].  Synchronous parts
// use `s`.  Returns hipSuccess or the failing HIP status.
hipError_t rank_by_hotness(const uint32_t* hot, int64_t num_vertices, int32_t* order, hipStream_t s);
// deg[v] = indptr[v + 1] - indptr[v], streamed from CPU memory.
void launch_degrees(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, int64_t num_vertices,
                    int32_t* deg, hipStream_t s);
// Inclusive scan of the Eq. 3 cost (deg * 4 + 8) along `order`; cost_scan has V entries.
hipError_t scan_topo_cost(const int32_t* deg, const int32_t* order, int64_t num_vertices, uint64_t* cost_scan,
                          hipStream_t s);
// result[0] = number of entries of the ascending array scan[0..n) that are <= budget,
// result[1] = scan[that - 1] (0 if none).  Device-side binary search.
void launch_prefix_within_budget(const uint64_t* scan, int64_t n, uint64_t budget, uint64_t* result, hipStream_t s);
// t_indptr[r] = edges before rank r, r = 0 .. n_topo (derived from the cost scan).
void launch_topo_offsets(const DeviceInfo& di, const uint64_t* cost_scan, int64_t n_topo, int64_t* t_indptr,
                         hipStream_t s);
// Copy the adjacency of order[0 .. n_topo) from CPU memory into the cached CSR.
void launch_fill_topo(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, const int32_t* h_indices,
                      const int32_t* order, int64_t n_topo, const int64_t* t_indptr, int32_t* t_indices,
                      hipStream_t s);
// Inclusive scan of hot[order[r]] along a ranking (64-bit sums); hot_scan has V entries.
hipError_t scan_hotness(const uint32_t* hot, const int32_t* order, int64_t num_vertices, uint64_t* hot_scan,
                        hipStream_t s);
// One thread per candidate plan: boundary of Eq. 3 by binary search in the cost scan, Eq. 6 by
// division, sums from the hotness scans, exact 128-bit comparison key; *best = first smallest key.
void launch_alpha_search(const uint64_t* cost_scan, const uint64_t* hot_t_scan, const uint64_t* hot_f_scan,
                         int64_t num_vertices, uint64_t row_bytes, const uint64_t* m_topo, uint64_t total_budget,
                         uint64_t n_tsum, uint64_t per_row, int32_t n_alpha, lgp_plan_point* points, int32_t* best,
                         hipStream_t s);
void launch_fill_i32(const DeviceInfo& di, int32_t* p, int64_t n, int32_t value, hipStream_t s);
// out = in reordered by ascending Philox key of the position (one permutation per epoch).  Synchronises `s`.
hipError_t shuffle_by_key(const DeviceInfo& di, const int32_t* in, int32_t* out, int64_t n, uint64_t seed,
                          uint32_t epoch, hipStream_t s);
// Algorithm 1 for k_g hotness rows: column sums, ranking, arg-max owner, per-GPU queues.  counts
// (device uint64[k_g]) receives the queue lengths.  Synchronises `s`.
hipError_t cslp_rank(const DeviceInfo& di, int32_t k_g, int64_t num_vertices, const uint32_t* hot, uint64_t* acc,
                     int32_t* order, int32_t* owner, int32_t* queues, unsigned long long* counts, hipStream_t s);
// row_tab[v] = (not cached, CPU offset, degree) for every vertex, streamed from the CPU-resident offsets.
void launch_init_row_table(const DeviceInfo& di, const void* h_indptr, int32_t indptr_bytes, int64_t num_vertices,
                           uint64_t* row_tab, hipStream_t s);
// row_tab[order[r]] = (cached, t_indptr[r], degree) for r < n_topo (rows too long to pack keep their CPU entry).
void launch_set_cached_rows(const DeviceInfo& di, const int32_t* order, int64_t n_topo, const int64_t* t_indptr,
                            uint64_t* row_tab, hipStream_t s);
// p[k] = k for k < n.
void launch_iota_i32(const DeviceInfo& di, int32_t* p, int64_t n, hipStream_t s);
// remap[order[r]] = r for r < n.
void launch_scatter_rank(const DeviceInfo& di, const int32_t* order, int64_t n, int32_t* remap, hipStream_t s);

}  // namespace lgp
