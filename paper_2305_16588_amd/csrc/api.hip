// C ABI of liblegion_prep: argument checking, context state, launch sequencing.  Every step of the
// method runs in the kernels; the only arithmetic of the method done on the host is closed-form
// sizing that needs no data -- Eq. 6's row count (budget / row bytes) and the alpha grid of Sec. 4.3.3.
#include "common.hpp"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

using namespace lgp;

// Scratch of lgp_gather_features_static: the hit / miss counters (first 64 words) and the four partition
// lists (hit rows, hit slots, miss rows, miss ids; LGP_STATIC_GATHER_MAX_IDS entries each) -- 64 MiB that
// every GPU this library runs on holds until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; kernels and copies use the per-device address kept in g_scratch.
constexpr int64_t kStaticMaxIds = LGP_STATIC_GATHER_MAX_IDS;
constexpr int64_t kStaticHeadWords = 64;
static __device__ __align__(256) int32_t scratch[kStaticHeadWords + 4 * kStaticMaxIds];

namespace {

constexpr int kMaxDevices = 64;
int32_t* g_scratch[kMaxDevices] = {};   // device address of `scratch` on each GPU, filled by lgp_create
std::mutex g_scratch_mutex;

// Look up, once per device and with that device current, where `scratch` lives on it.
hipError_t resolve_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return hipSuccess;   // the static entry point refuses such a device
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch[device]) return hipSuccess;
  void* p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!p) return hipErrorInvalidSymbol;
  g_scratch[device] = static_cast<int32_t*>(p);
  return hipSuccess;
}

enum ProfKind { PK_SAMPLE = 0, PK_PARTITION = 1, PK_HIT = 2, PK_MISS = 3, PK_COUNT = 4 };

struct EvPair {
  hipEvent_t a, b;
  int kind;
};

}  // namespace

struct lgp_ctx {
  DeviceInfo di;
  lgp_graph g{};           // pointers already translated to device-visible addresses
  int64_t row_bytes = 0;
  int64_t n_chunks = 0;    // dedup bitmap chunks

  uint64_t* row_tab = nullptr;   // per-vertex (cached?, offset, degree)
  int32_t* f_remap = nullptr;
  uint32_t* topo_hot = nullptr;
  uint32_t* feat_hot = nullptr;
  bool have_hot = false;
  uint64_t* fbits = nullptr;   // frontier dedup bitmap
  uint64_t* gbits = nullptr;   // gather-set dedup bitmap
  int32_t* chunk_counts = nullptr;
  uint32_t* d_err = nullptr;
  int32_t* counters = nullptr;  // {n_hit, n_miss, n_peer}

  // caches
  int32_t* order_t = nullptr;
  int32_t* order_f = nullptr;
  int64_t* t_indptr = nullptr;
  int32_t* t_indices = nullptr;
  void* fc = nullptr;
  bool fc_identity = false;   // the feature cache holds every vertex, laid out in vertex order (slot = id)
  CachePlan plan;
  // clique cache: member g holds cached vertices [clique_tn[g], clique_tn[g+1]) of order_t (edges
  // [clique_te[g], clique_te[g+1]) of t_indices) and feature slots [clique_fn[g], clique_fn[g+1])
  int32_t clique_k = 0;         // 0 = the cache was built for one GPU
  int64_t clique_tn[LGP_MAX_CLIQUE + 1] = {};
  int64_t clique_te[LGP_MAX_CLIQUE + 1] = {};
  int64_t clique_fn[LGP_MAX_CLIQUE + 1] = {};

  // gather scratch: hit / miss / peer-hit lists
  int32_t* lists = nullptr;
  int64_t list_cap = 0;

  // graph-constructor scratch
  int32_t* pos_table = nullptr;   // pos_tables tables of V entries: position of a vertex in one list of the batch
  int32_t pos_tables = 0;
  int64_t* tile_sums = nullptr;
  int64_t tile_cap = 0;

  // pre-sampling scratch
  int32_t* hs_frontier[LGP_MAX_HOPS] = {};
  int64_t hs_cap[LGP_MAX_HOPS] = {};
  int32_t* hs_n = nullptr;
  unsigned long long* hs_expansions = nullptr;   // device counter: sum of frontier sizes of the last pre-sampling
  int64_t hs_batches = 0;

  hipStream_t miss_stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;

  // intra-batch pipeline (lgp_sample_extract): the extractor's stream, one event per group of rows,
  // the groups' bounds and their hit / miss counts
  hipStream_t extract_stream = nullptr;
  hipEvent_t ev_group[LGP_MAX_HOPS + 2] = {};
  hipEvent_t ev_extracted = nullptr;
  int32_t* seg = nullptr;            // int32[LGP_MAX_HOPS + 2]
  int32_t* seg_counters = nullptr;   // int32[(LGP_MAX_HOPS + 1) * 3]
  int32_t* new_counts = nullptr;     // per compaction chunk: vertices reached first by the hop

  int profiling = 0;        // 0 off, 1 every per-batch kernel group, 2 the two row gathers only
  bool overlap = false;     // run the miss gather on its own stream beside the hit gather
  bool reserved = false;    // lgp_reserve fixed the scratch sizes: nothing grows any more
  std::vector<EvPair> ev_used;
  std::vector<EvPair> ev_free;

  std::string last_error;
};

namespace {

int fail(lgp_ctx* ctx, int status, const std::string& what) {
  if (ctx) ctx->last_error = what;
  return status;
}

int fail_hip(lgp_ctx* ctx, hipError_t e, const char* what) {
  (void)hipGetLastError();
  const int st = (e == hipErrorOutOfMemory) ? LGP_ENOMEM : LGP_EHIP;
  return fail(ctx, st, std::string(what) + ": " + hipGetErrorString(e));
}

#define LGP_HIP(ctx, call)                                    \
  do {                                                        \
    hipError_t e_ = (call);                                   \
    if (e_ != hipSuccess) return fail_hip((ctx), e_, #call); \
  } while (0)

// Resolve a caller pointer to an address kernels can use.
int device_visible(lgp_ctx* ctx, const void* p, const void** out, const char* name) {
  hipPointerAttribute_t attr;
  std::memset(&attr, 0, sizeof(attr));
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, LGP_EINVAL, std::string(name) + " is not pinned host memory nor device memory");
  }
  if (attr.type == hipMemoryTypeHost) {
    void* d = nullptr;
    e = hipHostGetDevicePointer(&d, const_cast<void*>(p), 0);
    if (e != hipSuccess || !d) {
      (void)hipGetLastError();
      return fail(ctx, LGP_EINVAL, std::string(name) + " is pinned but not mapped into the GPU address space");
    }
    *out = d;
    return LGP_OK;
  }
  if (attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged) {
    *out = p;
    return LGP_OK;
  }
  return fail(ctx, LGP_EINVAL, std::string(name) + " is not pinned host memory nor device memory");
}

template <typename T>
hipError_t dev_alloc(T** p, size_t count) {
  return hipMalloc(reinterpret_cast<void**>(p), std::max<size_t>(count, 1) * sizeof(T));
}

void free_cache(lgp_ctx* c) {
  if (c->t_indptr) (void)hipFree(c->t_indptr);
  if (c->t_indices) (void)hipFree(c->t_indices);
  if (c->fc) (void)hipFree(c->fc);
  c->t_indptr = nullptr;
  c->t_indices = nullptr;
  c->fc = nullptr;
  c->fc_identity = false;
  c->plan = CachePlan();
  c->clique_k = 0;
}

TopoView topo_view(const lgp_ctx* c) {
  TopoView tv;
  tv.row_tab = c->row_tab;
  tv.h_indptr = c->g.indptr;
  tv.h_indices = c->g.indices;
  tv.t_indices = c->t_indices;
  tv.indptr_bytes = c->g.indptr_bytes;
  tv.num_vertices = c->g.num_vertices;
  return tv;
}

int check_fanouts(lgp_ctx* ctx, const int32_t* fanouts, int32_t n_hops) {
  if (!fanouts) return fail(ctx, LGP_EINVAL, "fanouts is null");
  if (n_hops < 1) return fail(ctx, LGP_EINVAL, "n_hops must be >= 1");
  if (n_hops > LGP_MAX_HOPS) return fail(ctx, LGP_EUNSUPPORTED, "n_hops exceeds LGP_MAX_HOPS");
  for (int h = 0; h < n_hops; ++h) {
    if (fanouts[h] < 1) return fail(ctx, LGP_EINVAL, "fanout must be >= 1");
    if (fanouts[h] > LGP_MAX_FANOUT) return fail(ctx, LGP_EUNSUPPORTED, "fanout exceeds LGP_MAX_FANOUT");
  }
  return LGP_OK;
}

// Worst-case frontier sizes: need[0] = n_seeds, need[h] = min(V, need[h-1] * f[h-1]), h <= n_hops.
void worst_case(const lgp_ctx* c, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, int64_t* need,
                int64_t* gather_need) {
  const int64_t V = c->g.num_vertices;
  int64_t total = n_seeds;
  need[0] = n_seeds;
  for (int h = 0; h < n_hops; ++h) {
    const int64_t samples = need[h] * fanouts[h];
    total += samples;
    need[h + 1] = std::min(V, samples);
  }
  *gather_need = std::min(V, total);
}

// A pair of events for a launch that records its own start and stop times (nothing is enqueued here).
EvPair prof_pair(lgp_ctx* c, int kind) {
  EvPair p{nullptr, nullptr, kind};
  if (c->profiling == 0 || (c->profiling == 2 && kind != PK_HIT && kind != PK_MISS)) return p;
  if (!c->ev_free.empty()) {
    p = c->ev_free.back();
    c->ev_free.pop_back();
    p.kind = kind;
  } else if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) {
    (void)hipGetLastError();
    if (p.a) (void)hipEventDestroy(p.a);
    p.a = p.b = nullptr;
  }
  return p;
}

// Bracket a group of launches: a is recorded now, b by prof_end.
EvPair prof_begin(lgp_ctx* c, int kind, hipStream_t s) {
  EvPair p = prof_pair(c, kind);
  if (p.a) (void)hipEventRecord(p.a, s);
  return p;
}

void prof_keep(lgp_ctx* c, const EvPair& p) {
  if (p.a) c->ev_used.push_back(p);
}

void prof_end(lgp_ctx* c, EvPair& p, hipStream_t s) {
  if (!p.a) return;
  (void)hipEventRecord(p.b, s);
  c->ev_used.push_back(p);
}

// Sampling of one mini-batch; out == nullptr is the pre-sampling mode (hotness only).
int sample_core(lgp_ctx* c, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                uint64_t rng_seed, const lgp_sample_out* out, hipStream_t s) {
  const bool hot_mode = (out == nullptr);
  const int64_t V = c->g.num_vertices;
  uint32_t* fbits32 = reinterpret_cast<uint32_t*>(c->fbits);
  uint32_t* gbits32 = reinterpret_cast<uint32_t*>(c->gbits);
  int32_t* n_frontier = hot_mode ? c->hs_n : out->n_frontier;
  const TopoView tv = topo_view(c);

  const int32_t* frontier = seeds;
  int64_t cap = n_seeds;
  const bool want_last = !hot_mode && out->frontier[n_hops] != nullptr;
  for (int h = 0; h < n_hops; ++h) {
    // the last hop's samples only feed the gather set, so they are marked there directly -- unless
    // the caller wants the last frontier as a list of its own
    const bool last = (h + 1 == n_hops) && !want_last;
    launch_sample_hop(c->di, tv, frontier, n_frontier + h, cap, fanouts[h], h, rng_seed,
                      hot_mode ? nullptr : out->nbr[h], hot_mode ? nullptr : out->cnt[h], last ? gbits32 : fbits32,
                      h == 0 ? gbits32 : nullptr, hot_mode ? c->topo_hot : nullptr, c->d_err, s);
    if (!last) {
      int32_t* next = hot_mode ? c->hs_frontier[h + 1] : out->frontier[h + 1];
      const int64_t next_cap = hot_mode ? c->hs_cap[h + 1] : out->cap[h + 1];
      launch_compact(c->di, c->fbits, c->gbits, c->n_chunks, c->chunk_counts, next, next_cap, n_frontier + h + 1,
                     nullptr, c->d_err, s);
      frontier = next;
      cap = next_cap;
    }
  }
  if (hot_mode)
    launch_compact(c->di, c->gbits, nullptr, c->n_chunks, c->chunk_counts, nullptr, 0, nullptr, c->feat_hot, c->d_err,
                   s);
  else
    launch_compact(c->di, c->gbits, nullptr, c->n_chunks, c->chunk_counts, out->gather_ids, out->gather_cap,
                   out->n_gather, nullptr, c->d_err, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(c, e, "sampling kernel launch");
  return LGP_OK;
}

// Ranking + Eq. 3 / Eq. 6 sizes.  Leaves order_t / order_f filled; returns the
// cost scan (caller frees) when keep_scan is set.
int plan_core(lgp_ctx* c, uint64_t topo_budget, uint64_t feat_budget, CachePlan* plan, uint64_t** keep_scan,
              hipStream_t s) {
  const int64_t V = c->g.num_vertices;
  if (!c->have_hot) return fail(c, LGP_ESTATE, "no hotness yet: call lgp_build_hotness or lgp_set_hotness first");
  if (!c->order_t) LGP_HIP(c, dev_alloc(&c->order_t, size_t(V)));
  if (!c->order_f) LGP_HIP(c, dev_alloc(&c->order_f, size_t(V)));
  LGP_HIP(c, rank_by_hotness(c->topo_hot, V, c->order_t, s));
  LGP_HIP(c, rank_by_hotness(c->feat_hot, V, c->order_f, s));

  int32_t* deg = nullptr;
  uint64_t* scan = nullptr;
  uint64_t* result = nullptr;
  int st = LGP_OK;
  hipError_t e = dev_alloc(&deg, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&scan, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&result, 2);
  uint64_t host_result[2] = {0, 0};
  if (e == hipSuccess) {
    launch_degrees(c->di, c->g.indptr, c->g.indptr_bytes, V, deg, s);
    e = scan_topo_cost(deg, c->order_t, V, scan, s);
  }
  if (e == hipSuccess) {
    launch_prefix_within_budget(scan, V, topo_budget, result, s);
    e = hipMemcpyAsync(host_result, result, sizeof(host_result), hipMemcpyDeviceToHost, s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) st = fail_hip(c, e, "cache planning");
  if (deg) (void)hipFree(deg);
  if (result) (void)hipFree(result);
  if (st == LGP_OK) {
    plan->n_topo = int64_t(host_result[0]);
    plan->topo_bytes = host_result[1];
    plan->topo_edges = int64_t((host_result[1] - 8u * host_result[0]) / 4u);
    plan->n_feat = (c->row_bytes > 0 && c->g.features) ? std::min<int64_t>(V, int64_t(feat_budget / uint64_t(c->row_bytes))) : 0;
    plan->feat_bytes = uint64_t(plan->n_feat) * uint64_t(c->row_bytes);
  }
  if (keep_scan && st == LGP_OK) *keep_scan = scan;
  else if (scan) (void)hipFree(scan);
  return st;
}

// Scratch of the per-batch operators.  Each grows on demand (a growth step synchronises the stream and
// reallocates) unless lgp_reserve fixed the sizes, after which a larger request is refused.
int ensure_lists(lgp_ctx* c, int64_t n, hipStream_t s) {
  if (n <= c->list_cap) return LGP_OK;
  if (c->reserved) return fail(c, LGP_ECAPACITY, "more ids than lgp_reserve provided partition lists for");
  LGP_HIP(c, hipStreamSynchronize(s));
  LGP_HIP(c, hipStreamSynchronize(c->miss_stream));
  if (c->lists) (void)hipFree(c->lists);
  c->lists = nullptr;
  c->list_cap = 0;
  LGP_HIP(c, dev_alloc(&c->lists, size_t(n) * 6));
  c->list_cap = n;
  return LGP_OK;
}

int ensure_block_scratch(lgp_ctx* c, int32_t tables, int64_t tiles, hipStream_t s) {
  if (c->pos_tables >= tables && c->tile_cap >= tiles) return LGP_OK;
  if (c->reserved) return fail(c, LGP_ECAPACITY, "more hops or seeds than lgp_reserve provided graph-constructor scratch for");
  LGP_HIP(c, hipStreamSynchronize(s));
  if (c->pos_tables < tables) {
    if (c->pos_table) (void)hipFree(c->pos_table);
    c->pos_table = nullptr;
    c->pos_tables = 0;
    LGP_HIP(c, dev_alloc(&c->pos_table, size_t(tables) * size_t(c->g.num_vertices)));
    c->pos_tables = tables;
  }
  if (c->tile_cap < tiles) {
    if (c->tile_sums) (void)hipFree(c->tile_sums);
    c->tile_sums = nullptr;
    c->tile_cap = 0;
    LGP_HIP(c, dev_alloc(&c->tile_sums, size_t(tiles)));
    c->tile_cap = tiles;
  }
  return LGP_OK;
}

int ensure_presample_frontiers(lgp_ctx* c, const int64_t* need, int32_t n_hops, hipStream_t s) {
  for (int h = 1; h < n_hops; ++h) {
    if (c->hs_cap[h] >= need[h]) continue;
    if (c->reserved) return fail(c, LGP_ECAPACITY, "larger pre-sampling batches than lgp_reserve provided frontiers for");
    LGP_HIP(c, hipStreamSynchronize(s));
    if (c->hs_frontier[h]) (void)hipFree(c->hs_frontier[h]);
    c->hs_frontier[h] = nullptr;
    c->hs_cap[h] = 0;
    LGP_HIP(c, dev_alloc(&c->hs_frontier[h], size_t(need[h])));
    c->hs_cap[h] = need[h];
  }
  return LGP_OK;
}

int64_t scan_tiles(const int64_t* cap, int32_t n_hops) {
  int64_t tiles = 0;
  for (int h = 0; h < n_hops; ++h) tiles += cap[h] / kScanTile + 1;
  return tiles;
}

// member < 0: plain two-way extraction; member >= 0: three-way, as that member of the clique cache.
// fixed != nullptr: the counters and lists live in that caller-provided block (kStaticHeadWords words, then
// 2 * n_lists lists of fixed_cap entries); nothing is allocated, created or timed on this path.
// window != nullptr (device {begin, end}): only those entries of ids are extracted, into the output rows of the
// same numbers; window_items bounds their count (for sizing the grids).
int gather_core(lgp_ctx* c, int32_t member, const int32_t* ids, int64_t n_max, const int32_t* n_dev, void* out,
                       int32_t* stats, void* stream, int32_t* fixed = nullptr, int64_t fixed_cap = 0,
                       const int32_t* window = nullptr, int64_t window_items = 0) {
  if (n_max < 0 || (n_max > 0 && (!ids || !out))) return fail(c, LGP_EINVAL, "ids / out / n_max");
  if (!c->g.features) return fail(c, LGP_ESTATE, "the graph was created without a feature table");
  if (n_max >= (int64_t(1) << 31)) return fail(c, LGP_EUNSUPPORTED, "more than 2^31 - 1 rows in one call");
  const uintptr_t a = uintptr_t(out) | uintptr_t(c->row_bytes);
  const int64_t vec = (a & 15u) == 0 ? 16 : (a & 7u) == 0 ? 8 : (a & 3u) == 0 ? 4 : (a & 1u) == 0 ? 2 : 0;
  if (vec == 0 || c->row_bytes / vec > 4096) return fail(c, LGP_EUNSUPPORTED, "output alignment too small for this row width");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  const bool three = member >= 0;
  int32_t* counters = stats ? stats : fixed ? fixed : c->counters;
  const int saved_profiling = c->profiling;
  if (fixed) c->profiling = 0;                     // timing events are created on demand: not on this path
  struct Restore {
    lgp_ctx* c;
    int mode;
    ~Restore() { c->profiling = mode; }
  } restore{c, saved_profiling};
  PartLists L = {};
  if (n_max == 0) {
    launch_partition(c->di, ids, 0, nullptr, c->f_remap, c->g.num_vertices, L, three ? 3 : 2, 0, 0, counters, c->d_err,
                     s);
    return LGP_OK;
  }
  const int64_t V = c->g.num_vertices;
  EvPair ev;
  if (!three && c->plan.n_feat == V) {
    // every row is cached: no partition, the id list is looked up by the gather itself
    ev = prof_pair(c, PK_HIT);
    launch_gather_rows(c->di, c->fc, out, c->row_bytes, nullptr, ids, n_max, n_dev, false, s,
                       DirectIds{c->fc_identity ? nullptr : c->f_remap, V, counters, 0, c->d_err, window}, ev.a, ev.b,
                       false, window_items);
    prof_keep(c, ev);
  } else if (!three && c->plan.n_feat == 0) {
    // nothing is cached: every id is its own source row in CPU memory
    ev = prof_pair(c, PK_MISS);
    launch_gather_rows(c->di, c->g.features, out, c->row_bytes, nullptr, ids, n_max, n_dev, true, s,
                       DirectIds{nullptr, V, counters, 1, c->d_err, window}, ev.a, ev.b, false, window_items);
    prof_keep(c, ev);
  } else {
    if (fixed) {
      if (n_max > fixed_cap) return fail(c, LGP_ECAPACITY, "n_max exceeds LGP_STATIC_GATHER_MAX_IDS");
    } else {
      const int st = ensure_lists(c, n_max, s);
      if (st != LGP_OK) return st;
    }
    int32_t* const lists = fixed ? fixed + kStaticHeadWords : c->lists;
    const int64_t cap = fixed ? fixed_cap : c->list_cap;
    for (int l = 0; l < (three ? 3 : 2); ++l) {
      L.row[l] = lists + (2 * l) * cap;
      L.src[l] = lists + (2 * l + 1) * cap;
    }
    ev = prof_begin(c, PK_PARTITION, s);
    launch_partition(c->di, ids, n_max, n_dev, c->f_remap, V, L, three ? 3 : 2,
                     three ? int32_t(c->clique_fn[member]) : 0, three ? int32_t(c->clique_fn[member + 1]) : 0, counters,
                     c->d_err, s, window, window_items);
    prof_end(c, ev, s);
    // Hits first (HBM -> HBM, short), then misses (PCIe, long).  With overlap enabled the
    // misses run on a second stream beside the hits and rejoin `s` afterwards.
    hipStream_t ms = s;
    if (c->overlap) {
      ms = c->miss_stream;
      LGP_HIP(c, hipEventRecord(c->ev_fork, s));
      LGP_HIP(c, hipStreamWaitEvent(ms, c->ev_fork, 0));
    }
    const DirectIds listed{nullptr, 0, nullptr, 0, nullptr, nullptr};
    const int64_t items = (window && window_items > 0 && window_items < n_max) ? window_items : n_max;
    ev = prof_pair(c, PK_HIT);
    launch_gather_rows(c->di, c->fc, out, c->row_bytes, L.row[0], L.src[0], n_max, counters, false, s, listed, ev.a,
                       ev.b, c->overlap, items);
    prof_keep(c, ev);
    if (three) {   // rows a peer caches: on this one device a second HBM gather, from the peers' regions
      ev = prof_pair(c, PK_HIT);
      launch_gather_rows(c->di, c->fc, out, c->row_bytes, L.row[2], L.src[2], n_max, counters + 2, false, s, listed,
                         ev.a, ev.b, c->overlap, items);
      prof_keep(c, ev);
    }
    ev = prof_pair(c, PK_MISS);
    launch_gather_rows(c->di, c->g.features, out, c->row_bytes, L.row[1], L.src[1], n_max, counters + 1, true, ms,
                       listed, ev.a, ev.b, false, items);
    prof_keep(c, ev);
    if (c->overlap) {
      LGP_HIP(c, hipEventRecord(c->ev_join, ms));
      LGP_HIP(c, hipStreamWaitEvent(s, c->ev_join, 0));
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(c, e, "gather kernel launch");
  return LGP_OK;
}

}  // namespace

extern "C" {

const char* lgp_strerror(int status) {
  switch (status) {
    case LGP_OK: return "ok";
    case LGP_EINVAL: return "invalid argument";
    case LGP_ESTATE: return "call made in the wrong state";
    case LGP_ECAPACITY: return "caller buffer too small for the worst case";
    case LGP_EUNSUPPORTED: return "unsupported size or width";
    case LGP_EHIP: return "HIP runtime error";
    case LGP_ENOMEM: return "out of memory";
    case LGP_EDEVICE: return "a kernel reported an invalid vertex id or a buffer overrun";
    default: return "unknown status";
  }
}

const char* lgp_last_error(const lgp_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

int lgp_host_alloc(size_t bytes, void** out) {
  if (!out) return LGP_EINVAL;
  *out = nullptr;
  void* p = nullptr;
  hipError_t e = hipHostMalloc(&p, bytes ? bytes : 1, hipHostMallocDefault);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return LGP_ENOMEM;
  }
  *out = p;
  return LGP_OK;
}

int lgp_host_free(void* ptr) {
  if (!ptr) return LGP_OK;
  if (hipHostFree(ptr) != hipSuccess) {
    (void)hipGetLastError();
    return LGP_EHIP;
  }
  return LGP_OK;
}

int lgp_create(const lgp_graph* g, int device, lgp_ctx** out) {
  if (!g || !out) return LGP_EINVAL;
  *out = nullptr;
  if (g->num_vertices < 1 || g->num_edges < 0 || !g->indptr || (g->num_edges > 0 && !g->indices)) return LGP_EINVAL;
  if (g->indptr_bytes != 4 && g->indptr_bytes != 8) return LGP_EINVAL;
  if (g->num_vertices >= (int64_t(1) << 31) || g->num_edges >= (int64_t(1) << 39)) return LGP_EUNSUPPORTED;
  if (g->features && (g->feat_dim < 1 || g->elem_bytes < 1)) return LGP_EINVAL;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) {
    (void)hipGetLastError();
    return LGP_EINVAL;
  }
  lgp_ctx* c = new (std::nothrow) lgp_ctx();
  if (!c) return LGP_ENOMEM;
  int st = LGP_OK;
  auto bail = [&](int status) {
    lgp_destroy(c);
    return status;
  };
  if (hipSetDevice(device) != hipSuccess) return bail(LGP_EHIP);
  if (resolve_scratch(device) != hipSuccess) {
    (void)hipGetLastError();
    return bail(LGP_EHIP);
  }
  c->di.device = device;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) == hipSuccess) c->di.num_cus = prop.multiProcessorCount;
  c->g = *g;
  const void* p = nullptr;
  if ((st = device_visible(c, g->indptr, &p, "indptr")) != LGP_OK) return bail(st);
  c->g.indptr = p;
  if (g->indices) {
    if ((st = device_visible(c, g->indices, &p, "indices")) != LGP_OK) return bail(st);
    c->g.indices = static_cast<const int32_t*>(p);
  }
  if (g->features) {
    if ((st = device_visible(c, g->features, &p, "features")) != LGP_OK) return bail(st);
    c->g.features = p;
    c->row_bytes = int64_t(g->feat_dim) * g->elem_bytes;
    // the row gather divides by the chunk count with a 32-bit reciprocal (<= 4096 chunks per row)
    const uintptr_t a = uintptr_t(p) | uintptr_t(c->row_bytes);
    const int64_t vec = (a & 15u) == 0 ? 16 : (a & 7u) == 0 ? 8 : (a & 3u) == 0 ? 4 : (a & 1u) == 0 ? 2 : 0;
    if (vec == 0 || c->row_bytes / vec > 4096) return bail(LGP_EUNSUPPORTED);
  }
  const int64_t V = g->num_vertices;
  // Small graphs get a sparser dedup bitmap (vertex v = bit v << spread_shift, up to 2^24 bits): the
  // sampler's atomics on a bitmap of a few cache lines serialise on those lines.
  c->di.spread_shift = 0;
  while (c->di.spread_shift < kMaxSpreadShift && (V << (c->di.spread_shift + 1)) <= kSpreadTargetBits)
    ++c->di.spread_shift;
  c->n_chunks = ((V << c->di.spread_shift) + kChunkBits - 1) / kChunkBits;
  const size_t words = size_t(c->n_chunks) * size_t(kChunkWords);
  hipError_t e = hipSuccess;
  auto step = [&](hipError_t r) {
    if (e == hipSuccess) e = r;
  };
  step(dev_alloc(&c->row_tab, size_t(V)));
  step(dev_alloc(&c->f_remap, size_t(V)));
  step(dev_alloc(&c->topo_hot, size_t(V)));
  step(dev_alloc(&c->feat_hot, size_t(V)));
  step(dev_alloc(&c->fbits, words));
  step(dev_alloc(&c->gbits, words));
  step(dev_alloc(&c->chunk_counts, size_t(c->n_chunks)));
  step(dev_alloc(&c->d_err, 1));
  step(dev_alloc(&c->counters, 3));
  step(dev_alloc(&c->hs_n, LGP_MAX_HOPS + 1));
  step(dev_alloc(&c->hs_expansions, 1));
  step(dev_alloc(&c->seg, LGP_MAX_HOPS + 2));
  step(dev_alloc(&c->seg_counters, (LGP_MAX_HOPS + 1) * 3));
  step(dev_alloc(&c->new_counts, size_t(c->n_chunks)));
  if (e == hipSuccess) e = hipMemset(c->f_remap, 0xff, sizeof(int32_t) * size_t(V));
  if (e == hipSuccess) e = hipMemset(c->topo_hot, 0, sizeof(uint32_t) * size_t(V));
  if (e == hipSuccess) e = hipMemset(c->feat_hot, 0, sizeof(uint32_t) * size_t(V));
  if (e == hipSuccess) e = hipMemset(c->fbits, 0, sizeof(uint64_t) * words);
  if (e == hipSuccess) e = hipMemset(c->gbits, 0, sizeof(uint64_t) * words);
  if (e == hipSuccess) e = hipMemset(c->d_err, 0, sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->counters, 0, 3 * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(c->hs_expansions, 0, sizeof(unsigned long long));
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->miss_stream, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->extract_stream, hipStreamNonBlocking);
  for (int k = 0; k < LGP_MAX_HOPS + 2 && e == hipSuccess; ++k)
    e = hipEventCreateWithFlags(&c->ev_group[k], hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_extracted, hipEventDisableTiming);
  if (e == hipSuccess) {
    launch_init_row_table(c->di, c->g.indptr, c->g.indptr_bytes, V, c->row_tab, nullptr);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return bail(e == hipErrorOutOfMemory ? LGP_ENOMEM : LGP_EHIP);
  }
  *out = c;
  return LGP_OK;
}

int lgp_destroy(lgp_ctx* c) {
  if (!c) return LGP_OK;
  (void)hipSetDevice(c->di.device);
  (void)hipDeviceSynchronize();
  free_cache(c);
  void* ptrs[] = {c->row_tab, c->f_remap, c->topo_hot, c->feat_hot, c->fbits, c->gbits, c->chunk_counts,
                  c->d_err,   c->counters, c->order_t, c->order_f,  c->lists, c->hs_n, c->pos_table, c->tile_sums, c->hs_expansions,
                  c->seg, c->seg_counters, c->new_counts};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  for (int h = 0; h < LGP_MAX_HOPS; ++h)
    if (c->hs_frontier[h]) (void)hipFree(c->hs_frontier[h]);
  for (auto* v : {&c->ev_used, &c->ev_free})
    for (EvPair& p : *v) {
      (void)hipEventDestroy(p.a);
      (void)hipEventDestroy(p.b);
    }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  if (c->miss_stream) (void)hipStreamDestroy(c->miss_stream);
  for (hipEvent_t ev : c->ev_group)
    if (ev) (void)hipEventDestroy(ev);
  if (c->ev_extracted) (void)hipEventDestroy(c->ev_extracted);
  if (c->extract_stream) (void)hipStreamDestroy(c->extract_stream);
  (void)hipGetLastError();
  delete c;
  return LGP_OK;
}

int lgp_build_hotness(lgp_ctx* c, const int32_t* train_ids, int64_t n_train, int32_t batch, const int32_t* fanouts,
                      int32_t n_hops, uint64_t base_seed, int64_t max_batches, void* stream) {
  if (!c) return LGP_EINVAL;
  if (!train_ids || n_train < 0 || batch < 1) return fail(c, LGP_EINVAL, "train_ids / n_train / batch");
  int st = check_fanouts(c, fanouts, n_hops);
  if (st != LGP_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  const int64_t V = c->g.num_vertices;
  int64_t need[LGP_MAX_HOPS + 1], gather_need;
  worst_case(c, std::min<int64_t>(batch, std::max<int64_t>(n_train, 1)), fanouts, n_hops, need, &gather_need);
  st = ensure_presample_frontiers(c, need, n_hops, s);
  if (st != LGP_OK) return st;
  launch_fill_i32(c->di, reinterpret_cast<int32_t*>(c->topo_hot), V, 0, s);
  launch_fill_i32(c->di, reinterpret_cast<int32_t*>(c->feat_hot), V, 0, s);
  launch_fill_i32(c->di, reinterpret_cast<int32_t*>(c->hs_expansions), 2, 0, s);
  int64_t n_batches = (n_train + batch - 1) / batch;
  if (max_batches >= 0 && max_batches < n_batches) n_batches = max_batches;
  for (int64_t b = 0; b < n_batches; ++b) {
    const int64_t lo = b * batch;
    const int32_t nb = int32_t(std::min<int64_t>(batch, n_train - lo));
    st = sample_core(c, train_ids + lo, nb, fanouts, n_hops, base_seed + uint64_t(b), nullptr, s);
    if (st != LGP_OK) return st;
    launch_accumulate_sizes(c->hs_n, n_hops, c->hs_expansions, s);
  }
  c->hs_batches = n_batches;
  c->have_hot = true;
  return LGP_OK;
}

int lgp_get_presample_stats(lgp_ctx* c, int64_t* n_batches, int64_t* n_expansions) {
  if (!c) return LGP_EINVAL;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  unsigned long long v = 0;
  LGP_HIP(c, hipMemcpy(&v, c->hs_expansions, sizeof(v), hipMemcpyDeviceToHost));
  if (n_batches) *n_batches = c->hs_batches;
  if (n_expansions) *n_expansions = int64_t(v);
  return LGP_OK;
}

int lgp_get_hotness(lgp_ctx* c, uint32_t* topo_hot, uint32_t* feat_hot) {
  if (!c) return LGP_EINVAL;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  const size_t bytes = sizeof(uint32_t) * size_t(c->g.num_vertices);
  if (topo_hot) LGP_HIP(c, hipMemcpy(topo_hot, c->topo_hot, bytes, hipMemcpyDeviceToHost));
  if (feat_hot) LGP_HIP(c, hipMemcpy(feat_hot, c->feat_hot, bytes, hipMemcpyDeviceToHost));
  return LGP_OK;
}

int lgp_set_hotness(lgp_ctx* c, const uint32_t* topo_hot, const uint32_t* feat_hot) {
  if (!c) return LGP_EINVAL;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  const size_t bytes = sizeof(uint32_t) * size_t(c->g.num_vertices);
  if (topo_hot) LGP_HIP(c, hipMemcpy(c->topo_hot, topo_hot, bytes, hipMemcpyHostToDevice));
  if (feat_hot) LGP_HIP(c, hipMemcpy(c->feat_hot, feat_hot, bytes, hipMemcpyHostToDevice));
  c->have_hot = true;
  return LGP_OK;
}

int lgp_plan_cache(lgp_ctx* c, uint64_t topo_budget, uint64_t feat_budget, lgp_cache_plan* plan, void* stream) {
  if (!c) return LGP_EINVAL;
  if (!plan) return fail(c, LGP_EINVAL, "plan is null");
  LGP_HIP(c, hipSetDevice(c->di.device));
  if (c->plan.n_topo > 0 || c->plan.n_feat > 0)
    return fail(c, LGP_ESTATE, "lgp_plan_cache re-ranks the vertices; call it before lgp_build_cache");
  CachePlan p;
  int st = plan_core(c, topo_budget, feat_budget, &p, nullptr, static_cast<hipStream_t>(stream));
  if (st != LGP_OK) return st;
  plan->n_topo = p.n_topo;
  plan->topo_edges = p.topo_edges;
  plan->topo_bytes = p.topo_bytes;
  plan->n_feat = p.n_feat;
  plan->feat_bytes = p.feat_bytes;
  return LGP_OK;
}

int lgp_search_cache_plan(lgp_ctx* c, uint64_t total_budget, uint64_t n_tsum, uint32_t cls_bytes, int32_t n_alpha,
                          lgp_plan_point* points, int32_t* best, void* stream) {
  if (!c) return LGP_EINVAL;
  if (!best || cls_bytes < 1) return fail(c, LGP_EINVAL, "best is null or cls_bytes is 0");
  if (n_alpha < 2 || n_alpha > 1024) return fail(c, LGP_EINVAL, "n_alpha must be in [2, 1024]");
  if (!c->g.features) return fail(c, LGP_ESTATE, "the graph was created without a feature table");
  if (c->plan.n_topo > 0 || c->plan.n_feat > 0)
    return fail(c, LGP_ESTATE, "lgp_search_cache_plan re-ranks the vertices; call it before lgp_build_cache");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  const int64_t V = c->g.num_vertices;
  CachePlan unused;
  uint64_t* cost_scan = nullptr;
  int st = plan_core(c, 0, 0, &unused, &cost_scan, s);      // ranks both lists and scans the Eq. 3 cost
  if (st != LGP_OK) return st;
  std::vector<uint64_t> m_topo(n_alpha);
  for (int32_t i = 0; i < n_alpha; ++i)
    m_topo[i] = uint64_t((static_cast<unsigned __int128>(total_budget) * uint64_t(i)) / uint64_t(n_alpha - 1));
  uint64_t *hot_t = nullptr, *hot_f = nullptr, *d_m = nullptr;
  lgp_plan_point* d_points = nullptr;
  int32_t* d_best = nullptr;
  std::vector<lgp_plan_point> host_points(n_alpha);
  hipError_t e = dev_alloc(&hot_t, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&hot_f, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&d_m, size_t(n_alpha));
  if (e == hipSuccess) e = dev_alloc(&d_points, size_t(n_alpha));
  if (e == hipSuccess) e = dev_alloc(&d_best, 1);
  if (e == hipSuccess) e = scan_hotness(c->topo_hot, c->order_t, V, hot_t, s);
  if (e == hipSuccess) e = scan_hotness(c->feat_hot, c->order_f, V, hot_f, s);
  if (e == hipSuccess) e = hipMemcpyAsync(d_m, m_topo.data(), sizeof(uint64_t) * n_alpha, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) {
    const uint64_t per_row = (uint64_t(c->row_bytes) + cls_bytes - 1) / cls_bytes;
    launch_alpha_search(cost_scan, hot_t, hot_f, V, uint64_t(c->row_bytes), d_m, total_budget, n_tsum, per_row,
                        n_alpha, d_points, d_best, s);
    e = hipGetLastError();
  }
  if (e == hipSuccess)
    e = hipMemcpyAsync(host_points.data(), d_points, sizeof(lgp_plan_point) * n_alpha, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipMemcpyAsync(best, d_best, sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  for (void* p : {static_cast<void*>(hot_t), static_cast<void*>(hot_f), static_cast<void*>(d_m),
                  static_cast<void*>(d_points), static_cast<void*>(d_best), static_cast<void*>(cost_scan)})
    if (p) (void)hipFree(p);
  if (e != hipSuccess) return fail_hip(c, e, "cache plan search");
  if (points) std::memcpy(points, host_points.data(), sizeof(lgp_plan_point) * n_alpha);
  return LGP_OK;
}

int lgp_shuffle_tablet(int device, const int32_t* in, int32_t* out, int64_t n, uint64_t seed, uint32_t epoch,
                       void* stream) {
  if (n < 0 || (n > 0 && (!in || !out))) return LGP_EINVAL;
  if (n >= (int64_t(1) << 31)) return LGP_EUNSUPPORTED;   // positions are 32-bit counter words
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev || hipSetDevice(device) != hipSuccess) {
    (void)hipGetLastError();
    return LGP_EINVAL;
  }
  if (n == 0) return LGP_OK;
  DeviceInfo di;
  di.device = device;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) == hipSuccess) di.num_cus = prop.multiProcessorCount;
  hipError_t e = shuffle_by_key(di, in, out, n, seed, epoch, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? LGP_ENOMEM : LGP_EHIP;
  }
  return LGP_OK;
}

int lgp_cslp(int device, int32_t k_g, int64_t num_vertices, const uint32_t* hot, uint64_t* acc, int32_t* order,
             int32_t* owner, int32_t* queues, int64_t* queue_offsets, void* stream) {
  if (k_g < 1 || num_vertices < 1 || !hot || !acc || !order || !owner || !queues || !queue_offsets) return LGP_EINVAL;
  if (k_g > 64 || num_vertices >= (int64_t(1) << 31)) return LGP_EUNSUPPORTED;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev || hipSetDevice(device) != hipSuccess) {
    (void)hipGetLastError();
    return LGP_EINVAL;
  }
  DeviceInfo di;
  di.device = device;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) == hipSuccess) di.num_cus = prop.multiProcessorCount;
  unsigned long long* counts = nullptr;
  hipError_t e = dev_alloc(&counts, size_t(k_g));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (e == hipSuccess) e = cslp_rank(di, k_g, num_vertices, hot, acc, order, owner, queues, counts, s);
  unsigned long long host_counts[64] = {};
  if (e == hipSuccess) e = hipMemcpy(host_counts, counts, sizeof(unsigned long long) * size_t(k_g), hipMemcpyDeviceToHost);
  if (counts) (void)hipFree(counts);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? LGP_ENOMEM : LGP_EHIP;
  }
  queue_offsets[0] = 0;
  for (int32_t g = 0; g < k_g; ++g) queue_offsets[g + 1] = queue_offsets[g] + int64_t(host_counts[g]);
  return LGP_OK;
}

int lgp_build_cache(lgp_ctx* c, uint64_t topo_budget, uint64_t feat_budget, void* stream) {
  if (!c) return LGP_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  const int64_t V = c->g.num_vertices;
  if (!c->have_hot) return fail(c, LGP_ESTATE, "no hotness yet: call lgp_build_hotness or lgp_set_hotness first");
  // drop the old cache first: the remaps must not point into freed memory
  LGP_HIP(c, hipStreamSynchronize(s));
  LGP_HIP(c, hipStreamSynchronize(c->miss_stream));
  free_cache(c);
  launch_init_row_table(c->di, c->g.indptr, c->g.indptr_bytes, V, c->row_tab, s);
  launch_fill_i32(c->di, c->f_remap, V, -1, s);
  CachePlan p;
  uint64_t* scan = nullptr;
  int st = plan_core(c, topo_budget, feat_budget, &p, &scan, s);
  if (st != LGP_OK) return st;
  hipError_t e = dev_alloc(&c->t_indptr, size_t(p.n_topo + 1));
  if (e == hipSuccess) e = dev_alloc(&c->t_indices, size_t(p.topo_edges));
  if (e == hipSuccess && p.n_feat > 0) e = hipMalloc(&c->fc, size_t(p.feat_bytes));
  if (e == hipSuccess) {
    launch_topo_offsets(c->di, scan, p.n_topo, c->t_indptr, s);
    launch_fill_topo(c->di, c->g.indptr, c->g.indptr_bytes, c->g.indices, c->order_t, p.n_topo, c->t_indptr,
                     c->t_indices, s);
    launch_set_cached_rows(c->di, c->order_t, p.n_topo, c->t_indptr, c->row_tab, s);
    if (p.n_feat == V) {
      // the whole table fits: keep vertex order, so a cached row is found without any lookup
      launch_gather_rows(c->di, c->g.features, c->fc, c->row_bytes, nullptr, nullptr, V, nullptr, true, s);
      launch_iota_i32(c->di, c->f_remap, V, s);
    } else if (p.n_feat > 0) {
      launch_gather_rows(c->di, c->g.features, c->fc, c->row_bytes, nullptr, c->order_f, p.n_feat, nullptr, true, s);
      launch_scatter_rank(c->di, c->order_f, p.n_feat, c->f_remap, s);
    }
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(scan);
  if (e != hipSuccess) {
    st = fail_hip(c, e, "cache fill");
    free_cache(c);
    launch_init_row_table(c->di, c->g.indptr, c->g.indptr_bytes, V, c->row_tab, s);
    (void)hipStreamSynchronize(s);
    (void)hipMemset(c->f_remap, 0xff, sizeof(int32_t) * size_t(V));
    return st;
  }
  c->plan = p;
  c->fc_identity = (p.n_feat == V);
  return LGP_OK;
}

int lgp_build_clique_cache(lgp_ctx* c, int32_t k_g, const uint32_t* topo_hot, const uint32_t* feat_hot,
                           uint64_t topo_budget, uint64_t feat_budget, void* stream) {
  if (!c) return LGP_EINVAL;
  if (k_g < 1 || !topo_hot || !feat_hot) return fail(c, LGP_EINVAL, "k_g / topo_hot / feat_hot");
  if (k_g > LGP_MAX_CLIQUE) return fail(c, LGP_EUNSUPPORTED, "more than LGP_MAX_CLIQUE members");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  const int64_t V = c->g.num_vertices;
  LGP_HIP(c, hipStreamSynchronize(s));
  LGP_HIP(c, hipStreamSynchronize(c->miss_stream));
  free_cache(c);
  launch_init_row_table(c->di, c->g.indptr, c->g.indptr_bytes, V, c->row_tab, s);
  launch_fill_i32(c->di, c->f_remap, V, -1, s);
  if (!c->order_t) LGP_HIP(c, dev_alloc(&c->order_t, size_t(V)));
  if (!c->order_f) LGP_HIP(c, dev_alloc(&c->order_f, size_t(V)));

  uint64_t *acc = nullptr, *scan = nullptr, *result = nullptr;
  int32_t *order = nullptr, *owner = nullptr, *queues = nullptr, *deg = nullptr;
  unsigned long long* counts = nullptr;
  int64_t tn[LGP_MAX_CLIQUE + 1] = {}, te[LGP_MAX_CLIQUE + 1] = {}, fn[LGP_MAX_CLIQUE + 1] = {};
  unsigned long long host_counts[LGP_MAX_CLIQUE] = {};
  hipError_t e = dev_alloc(&acc, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&scan, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&result, 2);
  if (e == hipSuccess) e = dev_alloc(&order, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&owner, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&queues, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&deg, size_t(V));
  if (e == hipSuccess) e = dev_alloc(&counts, size_t(k_g));

  // topology: Algorithm 1 on H_T, then every member's queue is cut at its own budget (Eq. 3)
  if (e == hipSuccess) e = cslp_rank(c->di, k_g, V, topo_hot, acc, order, owner, queues, counts, s);
  if (e == hipSuccess) e = hipMemcpy(host_counts, counts, sizeof(unsigned long long) * size_t(k_g), hipMemcpyDeviceToHost);
  if (e == hipSuccess) launch_degrees(c->di, c->g.indptr, c->g.indptr_bytes, V, deg, s);
  int64_t q0 = 0;
  for (int32_t g = 0; g < k_g && e == hipSuccess; ++g) {
    const int64_t len = int64_t(host_counts[g]);
    uint64_t host_result[2] = {0, 0};
    if (len > 0) {
      e = scan_topo_cost(deg, queues + q0, len, scan, s);
      if (e == hipSuccess) {
        launch_prefix_within_budget(scan, len, topo_budget, result, s);
        e = hipMemcpyAsync(host_result, result, sizeof(host_result), hipMemcpyDeviceToHost, s);
      }
      if (e == hipSuccess) e = hipStreamSynchronize(s);
    }
    const int64_t n_g = int64_t(host_result[0]);
    if (e == hipSuccess && n_g > 0)
      e = hipMemcpyAsync(c->order_t + tn[g], queues + q0, sizeof(int32_t) * size_t(n_g), hipMemcpyDeviceToDevice, s);
    tn[g + 1] = tn[g] + n_g;
    te[g + 1] = te[g] + int64_t((host_result[1] - 8u * host_result[0]) / 4u);
    q0 += len;
  }
  const int64_t n_topo = tn[k_g], topo_edges = te[k_g];
  if (e == hipSuccess && n_topo > 0) e = scan_topo_cost(deg, c->order_t, n_topo, scan, s);
  if (e == hipSuccess) e = dev_alloc(&c->t_indptr, size_t(n_topo + 1));
  if (e == hipSuccess) e = dev_alloc(&c->t_indices, size_t(topo_edges));
  if (e == hipSuccess) {
    launch_topo_offsets(c->di, scan, n_topo, c->t_indptr, s);
    launch_fill_topo(c->di, c->g.indptr, c->g.indptr_bytes, c->g.indices, c->order_t, n_topo, c->t_indptr,
                     c->t_indices, s);
    launch_set_cached_rows(c->di, c->order_t, n_topo, c->t_indptr, c->row_tab, s);
    e = hipGetLastError();
  }

  // features: Algorithm 1 on H_F; every row costs the same (Eq. 6), so a member takes the head of its queue
  if (e == hipSuccess && c->g.features && c->row_bytes > 0) {
    e = cslp_rank(c->di, k_g, V, feat_hot, acc, order, owner, queues, counts, s);
    if (e == hipSuccess)
      e = hipMemcpy(host_counts, counts, sizeof(unsigned long long) * size_t(k_g), hipMemcpyDeviceToHost);
    q0 = 0;
    for (int32_t g = 0; g < k_g && e == hipSuccess; ++g) {
      const int64_t len = int64_t(host_counts[g]);
      const int64_t n_g = std::min<int64_t>(len, int64_t(feat_budget / uint64_t(c->row_bytes)));
      if (n_g > 0)
        e = hipMemcpyAsync(c->order_f + fn[g], queues + q0, sizeof(int32_t) * size_t(n_g), hipMemcpyDeviceToDevice, s);
      fn[g + 1] = fn[g] + n_g;
      q0 += len;
    }
    const int64_t n_feat = fn[k_g];
    if (e == hipSuccess && n_feat > 0) e = hipMalloc(&c->fc, size_t(n_feat) * size_t(c->row_bytes));
    if (e == hipSuccess && n_feat > 0) {
      launch_gather_rows(c->di, c->g.features, c->fc, c->row_bytes, nullptr, c->order_f, n_feat, nullptr, true, s);
      launch_scatter_rank(c->di, c->order_f, n_feat, c->f_remap, s);
      e = hipGetLastError();
    }
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  for (void* p : {static_cast<void*>(acc), static_cast<void*>(scan), static_cast<void*>(result),
                  static_cast<void*>(order), static_cast<void*>(owner), static_cast<void*>(queues),
                  static_cast<void*>(deg), static_cast<void*>(counts)})
    if (p) (void)hipFree(p);
  if (e != hipSuccess) {
    const int st = fail_hip(c, e, "clique cache fill");
    free_cache(c);
    launch_init_row_table(c->di, c->g.indptr, c->g.indptr_bytes, V, c->row_tab, s);
    (void)hipStreamSynchronize(s);
    (void)hipMemset(c->f_remap, 0xff, sizeof(int32_t) * size_t(V));
    return st;
  }
  c->plan.n_topo = n_topo;
  c->plan.topo_edges = topo_edges;
  c->plan.topo_bytes = uint64_t(topo_edges) * 4u + uint64_t(n_topo) * 8u;
  c->plan.n_feat = fn[k_g];
  c->plan.feat_bytes = uint64_t(fn[k_g]) * uint64_t(c->row_bytes);
  c->fc_identity = false;
  c->clique_k = k_g;
  for (int32_t g = 0; g <= k_g; ++g) {
    c->clique_tn[g] = tn[g];
    c->clique_te[g] = te[g];
    c->clique_fn[g] = fn[g];
  }
  return LGP_OK;
}

int lgp_get_clique_plan(lgp_ctx* c, int32_t member, lgp_cache_plan* plan) {
  if (!c) return LGP_EINVAL;
  if (!plan) return fail(c, LGP_EINVAL, "plan is null");
  if (c->clique_k == 0) return fail(c, LGP_ESTATE, "no clique cache: call lgp_build_clique_cache first");
  if (member < 0 || member >= c->clique_k) return fail(c, LGP_EINVAL, "member outside the clique");
  plan->n_topo = c->clique_tn[member + 1] - c->clique_tn[member];
  plan->topo_edges = c->clique_te[member + 1] - c->clique_te[member];
  plan->topo_bytes = uint64_t(plan->topo_edges) * 4u + uint64_t(plan->n_topo) * 8u;
  plan->n_feat = c->clique_fn[member + 1] - c->clique_fn[member];
  plan->feat_bytes = uint64_t(plan->n_feat) * uint64_t(c->row_bytes);
  return LGP_OK;
}

int lgp_get_cache_plan(lgp_ctx* c, lgp_cache_plan* plan) {
  if (!c) return LGP_EINVAL;
  if (!plan) return fail(c, LGP_EINVAL, "plan is null");
  plan->n_topo = c->plan.n_topo;
  plan->topo_edges = c->plan.topo_edges;
  plan->topo_bytes = c->plan.topo_bytes;
  plan->n_feat = c->plan.n_feat;
  plan->feat_bytes = c->plan.feat_bytes;
  return LGP_OK;
}

int lgp_get_cache(lgp_ctx* c, int32_t* topo_ids, int64_t* t_indptr, int32_t* t_indices, int32_t* feat_ids,
                  void* feat_rows) {
  if (!c) return LGP_EINVAL;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  const CachePlan& p = c->plan;
  if (topo_ids && p.n_topo)
    LGP_HIP(c, hipMemcpy(topo_ids, c->order_t, sizeof(int32_t) * size_t(p.n_topo), hipMemcpyDeviceToHost));
  if (t_indptr) {
    if (c->t_indptr)
      LGP_HIP(c, hipMemcpy(t_indptr, c->t_indptr, sizeof(int64_t) * size_t(p.n_topo + 1), hipMemcpyDeviceToHost));
    else
      t_indptr[0] = 0;
  }
  if (t_indices && p.topo_edges)
    LGP_HIP(c, hipMemcpy(t_indices, c->t_indices, sizeof(int32_t) * size_t(p.topo_edges), hipMemcpyDeviceToHost));
  if (feat_ids && p.n_feat)
    LGP_HIP(c, hipMemcpy(feat_ids, c->order_f, sizeof(int32_t) * size_t(p.n_feat), hipMemcpyDeviceToHost));
  if (feat_rows && p.n_feat) {
    const int st = lgp_get_cache_part(c, 1, 0, p.n_feat, feat_rows);
    if (st != LGP_OK) return st;
  }
  return LGP_OK;
}

int lgp_sample_khop(lgp_ctx* c, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                    uint64_t rng_seed, const lgp_sample_out* out, void* stream) {
  if (!c) return LGP_EINVAL;
  if (n_seeds < 0 || (n_seeds > 0 && !seeds) || !out) return fail(c, LGP_EINVAL, "seeds / n_seeds / out");
  int st = check_fanouts(c, fanouts, n_hops);
  if (st != LGP_OK) return st;
  if (!out->n_frontier || !out->n_gather) return fail(c, LGP_EINVAL, "out has null count pointers");
  int64_t need[LGP_MAX_HOPS + 1], gather_need;
  worst_case(c, n_seeds, fanouts, n_hops, need, &gather_need);
  for (int h = 0; h < n_hops; ++h) {
    if (need[h] > 0 && (!out->nbr[h] || !out->cnt[h] || (h > 0 && !out->frontier[h])))
      return fail(c, LGP_EINVAL, "out has a null hop buffer");
    if (out->cap[h] < need[h]) return fail(c, LGP_ECAPACITY, "out->cap[h] is below the worst-case frontier size");
  }
  if (out->frontier[n_hops] && out->cap[n_hops] < need[n_hops])
    return fail(c, LGP_ECAPACITY, "out->cap[n_hops] is below the worst-case size of the last frontier");
  if (out->gather_cap < gather_need) return fail(c, LGP_ECAPACITY, "out->gather_cap is below the worst case");
  if (gather_need > 0 && !out->gather_ids) return fail(c, LGP_EINVAL, "out->gather_ids is null");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  EvPair ev = prof_begin(c, PK_SAMPLE, s);
  st = sample_core(c, seeds, n_seeds, fanouts, n_hops, rng_seed, out, s);
  prof_end(c, ev, s);
  return st;
}

int lgp_sample_extract(lgp_ctx* c, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                       uint64_t rng_seed, const lgp_sample_out* out, void* rows, int32_t* groups, int32_t* stats,
                       void* stream) {
  if (!c) return LGP_EINVAL;
  if (n_seeds < 0 || (n_seeds > 0 && !seeds) || !out) return fail(c, LGP_EINVAL, "seeds / n_seeds / out");
  int st = check_fanouts(c, fanouts, n_hops);
  if (st != LGP_OK) return st;
  if (!c->g.features) return fail(c, LGP_ESTATE, "the graph was created without a feature table");
  if (!out->n_frontier || !out->n_gather) return fail(c, LGP_EINVAL, "out has null count pointers");
  int64_t need[LGP_MAX_HOPS + 1], gather_need;
  worst_case(c, n_seeds, fanouts, n_hops, need, &gather_need);
  for (int h = 0; h < n_hops; ++h) {
    if (need[h] > 0 && (!out->nbr[h] || !out->cnt[h] || (h > 0 && !out->frontier[h])))
      return fail(c, LGP_EINVAL, "out has a null hop buffer");
    if (out->cap[h] < need[h]) return fail(c, LGP_ECAPACITY, "out->cap[h] is below the worst-case frontier size");
  }
  if (out->frontier[n_hops] && out->cap[n_hops] < need[n_hops])
    return fail(c, LGP_ECAPACITY, "out->cap[n_hops] is below the worst-case size of the last frontier");
  // the seeds are listed as given, so a seed list with duplicates needs at least its own length
  if (out->gather_cap < std::max<int64_t>(gather_need, n_seeds))
    return fail(c, LGP_ECAPACITY, "out->gather_cap is below the worst case");
  if (gather_need > 0 && (!out->gather_ids || !rows)) return fail(c, LGP_EINVAL, "out->gather_ids / rows is null");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipStream_t x = c->extract_stream;
  LGP_HIP(c, hipSetDevice(c->di.device));
  if (0 < c->plan.n_feat && c->plan.n_feat < c->g.num_vertices) {   // the partition lists must exist before anything is enqueued
    st = ensure_lists(c, out->gather_cap, s);
    if (st != LGP_OK) return st;
  }
  const TopoView tv = topo_view(c);
  uint32_t* fbits32 = reinterpret_cast<uint32_t*>(c->fbits);
  uint32_t* gbits32 = reinterpret_cast<uint32_t*>(c->gbits);
  const int n_groups = n_hops + 1;
  // group 0: the seeds' rows, extracted while the first hop is being sampled
  launch_begin_listing(c->di, seeds, n_seeds, out->gather_ids, c->seg, c->seg_counters, n_groups * 3, s);
  LGP_HIP(c, hipEventRecord(c->ev_group[0], s));
  LGP_HIP(c, hipStreamWaitEvent(x, c->ev_group[0], 0));
  // from here on a failed step stops the enqueueing but not the clean-up below: the bitmaps must be clear and
  // `stream` must have joined the library's stream whatever the call returns
  st = gather_core(c, -1, out->gather_ids, out->gather_cap, nullptr, rows, c->seg_counters, x, nullptr, 0, c->seg,
                   std::max<int64_t>(n_seeds, 1));
  const int32_t* frontier = seeds;
  int64_t cap = n_seeds;
  for (int h = 0; h < n_hops && st == LGP_OK; ++h) {
    launch_sample_hop(c->di, tv, frontier, out->n_frontier + h, cap, fanouts[h], h, rng_seed, out->nbr[h], out->cnt[h],
                      fbits32, h == 0 ? gbits32 : nullptr, nullptr, c->d_err, s);
    // next frontier (if anyone needs it as a list) and the vertices this hop reached first, appended to the listing
    const bool want = (h + 1 < n_hops) || out->frontier[n_hops] != nullptr;
    int32_t* next = want ? out->frontier[h + 1] : nullptr;
    const bool last = h + 1 == n_hops;
    launch_compact_new(c->di, c->fbits, c->gbits, c->n_chunks, c->chunk_counts, c->new_counts, next,
                       next ? out->cap[h + 1] : 0, want ? out->n_frontier + h + 1 : nullptr, out->gather_ids,
                       out->gather_cap, c->seg + h + 1, last ? out->n_gather : nullptr, c->d_err, s);
    LGP_HIP(c, hipEventRecord(c->ev_group[h + 1], s));
    LGP_HIP(c, hipStreamWaitEvent(x, c->ev_group[h + 1], 0));
    st = gather_core(c, -1, out->gather_ids, out->gather_cap, nullptr, rows, c->seg_counters + 3 * (h + 1), x, nullptr, 0,
                     c->seg + h + 1, std::max<int64_t>(need[h + 1], 1));
    frontier = next;
    cap = next ? out->cap[h + 1] : 0;
  }
  // the "seen" bitmap of this batch is not compacted (the listing replaces the ascending list), so clear it whole
  launch_fill_i32(c->di, reinterpret_cast<int32_t*>(c->gbits), c->n_chunks * kChunkWords * 2, 0, s);
  if (st == LGP_OK && stats) launch_sum_stats(c->seg_counters, n_groups, stats, x);
  if (st == LGP_OK && groups) {
    LGP_HIP(c, hipMemcpyAsync(groups, c->seg, sizeof(int32_t) * size_t(n_hops + 2), hipMemcpyDeviceToDevice, x));
  }
  LGP_HIP(c, hipEventRecord(c->ev_extracted, x));
  LGP_HIP(c, hipStreamWaitEvent(s, c->ev_extracted, 0));
  if (st != LGP_OK) return st;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(c, e, "intra-batch pipeline launch");
  return LGP_OK;
}

int lgp_build_blocks(lgp_ctx* c, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                     const lgp_sample_out* sampled, const lgp_blocks_out* out, void* stream) {
  if (!c) return LGP_EINVAL;
  if (n_seeds < 0 || (n_seeds > 0 && !seeds) || !sampled || !out) return fail(c, LGP_EINVAL, "seeds / sampled / out");
  int st = check_fanouts(c, fanouts, n_hops);
  if (st != LGP_OK) return st;
  if (!sampled->n_frontier || !sampled->n_gather) return fail(c, LGP_EINVAL, "sampled has null count pointers");
  int64_t need[LGP_MAX_HOPS + 1], gather_need;
  worst_case(c, n_seeds, fanouts, n_hops, need, &gather_need);
  for (int h = 0; h <= n_hops; ++h) {
    if (h < n_hops && !out->blk_indptr[h]) return fail(c, LGP_EINVAL, "out->blk_indptr[h] is null");
    if (need[h] == 0) continue;
    if (sampled->cap[h] < need[h]) return fail(c, LGP_ECAPACITY, "sampled->cap[h] is below the worst case");
    if (h > 0 && !sampled->frontier[h])
      return fail(c, LGP_EINVAL, "sampled->frontier[h] is null (the last frontier is needed too)");
    if (!out->feat_row[h]) return fail(c, LGP_EINVAL, "out->feat_row[h] is null");
    if (h < n_hops && (!sampled->nbr[h] || !sampled->cnt[h] || !out->blk_indptr[h] || !out->blk_src[h]))
      return fail(c, LGP_EINVAL, "a hop buffer is null");
  }
  if (gather_need > 0 && !sampled->gather_ids) return fail(c, LGP_EINVAL, "sampled->gather_ids is null");
  hipStream_t s = static_cast<hipStream_t>(stream);
  LGP_HIP(c, hipSetDevice(c->di.device));
  BlocksArgs a = {};
  a.n_hops = n_hops;
  a.num_vertices = c->g.num_vertices;
  a.n_frontier = sampled->n_frontier;
  a.gather_ids = sampled->gather_ids;
  a.n_gather = sampled->n_gather;
  a.gather_cap = gather_need > 0 ? sampled->gather_cap : 0;
  int64_t tiles = 0;
  for (int h = 0; h <= n_hops; ++h) {
    a.frontier[h] = h == 0 ? seeds : sampled->frontier[h];
    a.cap[h] = need[h] ? sampled->cap[h] : 0;
    a.feat_row[h] = out->feat_row[h];
    if (h == n_hops) break;
    a.nbr[h] = sampled->nbr[h];
    a.cnt[h] = sampled->cnt[h];
    a.fanout[h] = fanouts[h];
    a.blk_indptr[h] = out->blk_indptr[h];
    a.blk_src[h] = out->blk_src[h];
    a.tile_base[h] = tiles;
    tiles += a.cap[h] / kScanTile + 1;
  }
  // scratch: one position table per list (the extracted ids and every frontier after the seeds) and the scan tiles
  st = ensure_block_scratch(c, n_hops + 1, tiles, s);
  if (st != LGP_OK) return st;
  a.table = c->pos_table;
  a.tile_sums = c->tile_sums;
  launch_build_blocks(c->di, a, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(c, e, "graph constructor launch");
  return LGP_OK;
}

int lgp_gather_features(lgp_ctx* c, const int32_t* ids, int64_t n_max, const int32_t* n_dev, void* out,
                        int32_t* stats, void* stream) {
  if (!c) return LGP_EINVAL;
  return gather_core(c, -1, ids, n_max, n_dev, out, stats, stream);
}

int lgp_gather_features_static(lgp_ctx* c, const int32_t* ids, int64_t n_max, const int32_t* n_dev, void* out,
                               int32_t* stats, void* stream) {
  if (!c) return LGP_EINVAL;
  if (n_max > kStaticMaxIds) return fail(c, LGP_ECAPACITY, "n_max exceeds LGP_STATIC_GATHER_MAX_IDS");
  int32_t* const block = (c->di.device >= 0 && c->di.device < kMaxDevices) ? g_scratch[c->di.device] : nullptr;
  if (!block) return fail(c, LGP_EUNSUPPORTED, "no static scratch was set up for this device");
  return gather_core(c, -1, ids, n_max, n_dev, out, stats, stream, block, kStaticMaxIds);
}

int lgp_gather_features_clique(lgp_ctx* c, int32_t member, const int32_t* ids, int64_t n_max, const int32_t* n_dev,
                               void* out, int32_t* stats, void* stream) {
  if (!c) return LGP_EINVAL;
  if (c->clique_k == 0) return fail(c, LGP_ESTATE, "no clique cache: call lgp_build_clique_cache first");
  if (member < 0 || member >= c->clique_k) return fail(c, LGP_EINVAL, "member outside the clique");
  return gather_core(c, member, ids, n_max, n_dev, out, stats, stream);
}

int lgp_reserve(lgp_ctx* c, int32_t max_seeds, const int32_t* fanouts, int32_t n_hops) {
  if (!c) return LGP_EINVAL;
  if (max_seeds < 0) return fail(c, LGP_EINVAL, "max_seeds is negative");
  int st = check_fanouts(c, fanouts, n_hops);
  if (st != LGP_OK) return st;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  int64_t need[LGP_MAX_HOPS + 1], gather_need;
  worst_case(c, max_seeds, fanouts, n_hops, need, &gather_need);
  c->reserved = false;
  if ((st = ensure_lists(c, gather_need, nullptr)) != LGP_OK) return st;
  if ((st = ensure_block_scratch(c, n_hops + 1, scan_tiles(need, n_hops), nullptr)) != LGP_OK) return st;
  if ((st = ensure_presample_frontiers(c, need, n_hops, nullptr)) != LGP_OK) return st;
  c->reserved = true;
  return LGP_OK;
}

int lgp_get_cache_part(lgp_ctx* c, int32_t which, int64_t first, int64_t count, void* dst) {
  if (!c) return LGP_EINVAL;
  if (first < 0 || count < 0 || (count > 0 && !dst)) return fail(c, LGP_EINVAL, "first / count / dst");
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipDeviceSynchronize());
  const CachePlan& p = c->plan;
  if (count == 0) return LGP_OK;
  if (which == 0) {
    if (first + count > p.topo_edges) return fail(c, LGP_EINVAL, "range beyond the cached column ids");
    LGP_HIP(c, hipMemcpy(dst, c->t_indices + first, sizeof(int32_t) * size_t(count), hipMemcpyDeviceToHost));
    return LGP_OK;
  }
  if (which != 1) return fail(c, LGP_EINVAL, "which must be 0 (column ids) or 1 (feature rows)");
  if (first + count > p.n_feat) return fail(c, LGP_EINVAL, "range beyond the cached feature rows");
  if (!c->fc_identity) {
    LGP_HIP(c, hipMemcpy(dst, static_cast<const char*>(c->fc) + first * c->row_bytes, size_t(count * c->row_bytes),
                         hipMemcpyDeviceToHost));
    return LGP_OK;
  }
  // the cache sits in vertex order; hand the rows out in rank order like any other cache
  const int64_t chunk = std::max<int64_t>(1, std::min<int64_t>(count, (int64_t(256) << 20) / c->row_bytes));
  void* tmp = nullptr;
  LGP_HIP(c, hipMalloc(&tmp, size_t(chunk * c->row_bytes)));
  hipError_t e = hipSuccess;
  for (int64_t lo = 0; lo < count && e == hipSuccess; lo += chunk) {
    const int64_t n = std::min(chunk, count - lo);
    launch_gather_rows(c->di, c->fc, tmp, c->row_bytes, nullptr, c->order_f + first + lo, n, nullptr, false, nullptr);
    e = hipGetLastError();
    if (e == hipSuccess)
      e = hipMemcpy(static_cast<char*>(dst) + lo * c->row_bytes, tmp, size_t(n * c->row_bytes), hipMemcpyDeviceToHost);
  }
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail_hip(c, e, "reading the feature cache back");
  return LGP_OK;
}

int lgp_workspace_bytes(const lgp_ctx* c, int32_t max_seeds, const int32_t* fanouts, int32_t n_hops, size_t* fixed,
                        size_t* scratch) {
  if (!c || max_seeds < 0) return LGP_EINVAL;
  if (!fanouts || n_hops < 1) return LGP_EINVAL;
  if (n_hops > LGP_MAX_HOPS) return LGP_EUNSUPPORTED;
  for (int h = 0; h < n_hops; ++h) {
    if (fanouts[h] < 1) return LGP_EINVAL;
    if (fanouts[h] > LGP_MAX_FANOUT) return LGP_EUNSUPPORTED;
  }
  const size_t V = size_t(c->g.num_vertices);
  if (fixed) {
    const size_t bitmap = size_t(c->n_chunks) * size_t(kChunkWords) * 8;
    // row table 8 + remap 4 + two hotness vectors 4 + 4 + two rankings 4 + 4 bytes per vertex
    *fixed = V * 28 + 2 * bitmap + size_t(c->n_chunks) * 4 + 64;
  }
  if (scratch) {
    int64_t need[LGP_MAX_HOPS + 1], gather_need;
    worst_case(c, max_seeds, fanouts, n_hops, need, &gather_need);
    size_t total = size_t(gather_need) * 6 * 4;                 // hit / miss / peer lists
    total += size_t(n_hops + 1) * V * 4;                        // graph constructor: one position table per list
    for (int h = 0; h < n_hops; ++h) total += (size_t(need[h]) / kScanTile + 1) * 8;
    for (int h = 1; h < n_hops; ++h) total += size_t(need[h]) * 4;   // pre-sampling frontiers
    *scratch = total;
  }
  return LGP_OK;
}

int lgp_check(lgp_ctx* c, void* stream) {
  if (!c) return LGP_EINVAL;
  LGP_HIP(c, hipSetDevice(c->di.device));
  LGP_HIP(c, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  LGP_HIP(c, hipStreamSynchronize(c->miss_stream));
  uint32_t flag = 0;
  LGP_HIP(c, hipMemcpy(&flag, c->d_err, sizeof(flag), hipMemcpyDeviceToHost));
  if (flag) {
    LGP_HIP(c, hipMemset(c->d_err, 0, sizeof(uint32_t)));
    char buf[96];
    std::snprintf(buf, sizeof(buf), "device error flag 0x%x (1 = invalid vertex id, 2 = output overrun)", flag);
    return fail(c, LGP_EDEVICE, buf);
  }
  return LGP_OK;
}

int lgp_set_overlap(lgp_ctx* c, int enable) {
  if (!c) return LGP_EINVAL;
  c->overlap = enable != 0;
  return LGP_OK;
}

int lgp_set_profiling(lgp_ctx* c, int enable) {
  if (!c) return LGP_EINVAL;
  c->profiling = enable == 2 ? 2 : (enable != 0 ? 1 : 0);
  return LGP_OK;
}

int lgp_get_profile(lgp_ctx* c, lgp_profile* out) {
  if (!c) return LGP_EINVAL;
  if (!out) return fail(c, LGP_EINVAL, "out is null");
  LGP_HIP(c, hipSetDevice(c->di.device));
  std::memset(out, 0, sizeof(*out));
  int64_t* counts[PK_COUNT] = {&out->n_sample, &out->n_partition, &out->n_hit, &out->n_miss};
  double* sums[PK_COUNT] = {&out->ms_sample, &out->ms_partition, &out->ms_hit, &out->ms_miss};
  // a pair leaves ev_used before it enters ev_free, so that an error in the middle of the loop
  // leaves every pair in exactly one of the two lists (lgp_destroy destroys both)
  hipError_t e = hipSuccess;
  while (!c->ev_used.empty()) {
    const EvPair p = c->ev_used.back();
    c->ev_used.pop_back();
    c->ev_free.push_back(p);
    if (e != hipSuccess) continue;
    float ms = 0.f;
    e = hipEventSynchronize(p.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.a, p.b);
    if (e != hipSuccess) continue;
    *counts[p.kind] += 1;
    *sums[p.kind] += double(ms);
  }
  if (e != hipSuccess) return fail_hip(c, e, "reading the profiling events");
  return LGP_OK;
}

}  // extern "C"
