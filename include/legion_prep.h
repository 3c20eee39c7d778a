/*
 * legion_prep -- per-mini-batch data preparation for cache-based GNN training
 * on one MI355X: pre-sampling hotness, hotness-ranked topology / feature
 * caches in HBM, k-hop uniform neighbour sampling and feature extraction.
 *
 * C ABI.  Every function returns 0 (LGP_OK) or a negative lgp_status; no C++
 * exception crosses this boundary.  Unless stated otherwise a call only
 * enqueues work on `stream` (a hipStream_t passed as void*, NULL = the default
 * stream) and returns without waiting for it.
 *
 * Pointer kinds used below
 *   [host]    ordinary host memory, read or written before the call returns
 *   [pinned]  host memory that the GPU can address (lgp_host_alloc,
 *             hipHostMalloc, or a pinned torch tensor); kernels read it in
 *             place over PCIe.  A device pointer is accepted in its place.
 *   [device]  memory of the GPU the context was created on
 * The caller owns every buffer it passes and keeps it alive until the work
 * that uses it has finished (graph arrays: until lgp_destroy).  The library
 * owns the context, the caches, the hotness vectors and its scratch memory.
 * A context is driven from one host thread.  lgp_sample_khop, lgp_build_blocks and
 * lgp_gather_features (or lgp_gather_features_clique) use disjoint scratch memory, so one
 * call of each may be in flight at the same time on different streams -- the pipelines of
 * Sec. 5: within a batch the graph constructor beside the feature extractor, across
 * batches the sampling of batch i+1 beside both (the caller orders what depends on what:
 * both consumers wait for the sampling of their batch, and a sample buffer is reused only
 * after its consumers finished).  Any other pair of calls must be ordered by the caller,
 * e.g. by issuing them on one stream.
 */
#ifndef LEGION_PREP_H
#define LEGION_PREP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LGP_OK = 0,
  LGP_EINVAL = -1,       /* null pointer, negative size, id out of range, bad dtype width        */
  LGP_ESTATE = -2,       /* call order: e.g. build_cache before any hotness exists                */
  LGP_ECAPACITY = -3,    /* a caller buffer is smaller than the worst case for this call          */
  LGP_EUNSUPPORTED = -4, /* fanout > LGP_MAX_FANOUT, hops > LGP_MAX_HOPS, V >= 2^31, E >= 2^39, row too wide */
  LGP_EHIP = -5,         /* a HIP runtime call failed; lgp_last_error has the text                */
  LGP_ENOMEM = -6,       /* device or pinned allocation failed                                    */
  LGP_EDEVICE = -7       /* a kernel met an invalid vertex id or overran a buffer (sticky flag)   */
} lgp_status;

#define LGP_MAX_HOPS 8
#define LGP_MAX_FANOUT 64

typedef struct lgp_ctx lgp_ctx; /* opaque */

/* Graph and feature table as they sit in CPU memory (Sec. 4.2: the full graph lives in
 * CPU memory; topology is CSR, Eq. 3; features are a V x D array, Eq. 6). */
typedef struct {
  int64_t num_vertices;      /* V, 1 <= V < 2^31                                              */
  int64_t num_edges;         /* E = indptr[V]                                                 */
  const void* indptr;        /* [pinned] V + 1 row offsets, int32 or int64                    */
  int32_t indptr_bytes;      /* 4 or 8                                                        */
  const int32_t* indices;    /* [pinned] E column ids (out-neighbours), each in [0, V)        */
  const void* features;      /* [pinned] row-major V x D table; may be NULL (no gather then)   */
  int32_t feat_dim;          /* D                                                             */
  int32_t elem_bytes;        /* bytes per element: 4 (fp32) or 2 (fp16); rows are opaque bytes */
} lgp_graph;

/* What lgp_plan_cache / lgp_get_cache_plan report (Eq. 3 and Eq. 6 evaluated on the ranking). */
typedef struct {
  int64_t n_topo;            /* vertices whose adjacency is cached                             */
  int64_t topo_edges;        /* column ids held by the topology cache                          */
  uint64_t topo_bytes;       /* sum over cached vertices of deg * 4 + 8  (<= topology budget)  */
  int64_t n_feat;            /* vertices whose feature row is cached                           */
  uint64_t feat_bytes;       /* n_feat * D * elem_bytes (<= feature budget)                    */
} lgp_cache_plan;

/* Destination buffers of one lgp_sample_khop call.  Hop h (0-based) expands frontier h
 * with fan-out fanouts[h]; frontier 0 is the seed list itself; frontier n_hops is the set
 * reached by the last hop (never expanded).
 * Worst-case sizes: need[0] = n_seeds, need[h] = min(V, need[h-1] * fanouts[h-1]). */
typedef struct {
  int32_t* frontier[LGP_MAX_HOPS + 1]; /* [device] frontier[h], 1 <= h <= n_hops: cap[h] ids, ascending, unique;
                                          [0] unused; frontier[n_hops] may be NULL (last set not wanted)        */
  int32_t* nbr[LGP_MAX_HOPS];      /* [device] nbr[h]: cap[h] * fanouts[h]; row i = samples of frontier[h][i],
                                      -1 padded; rows past n_frontier[h] are left untouched                     */
  int32_t* cnt[LGP_MAX_HOPS];      /* [device] cnt[h]: cap[h]; valid entries in row i = min(deg, fanout)        */
  int64_t cap[LGP_MAX_HOPS + 1];   /* capacities in vertices; cap[h] >= need[h] or LGP_ECAPACITY                */
  int32_t* n_frontier;             /* [device] int32[n_hops + 1]: actual frontier sizes (n_frontier[0] = n_seeds;
                                      the last entry is written only if frontier[n_hops] is given)              */
  int32_t* gather_ids;             /* [device] ascending unique union of seeds and all sampled neighbours       */
  int64_t gather_cap;              /* >= min(V, n_seeds + sum_h need[h] * fanouts[h]) or LGP_ECAPACITY          */
  int32_t* n_gather;               /* [device] int32[1]: number of ids written to gather_ids                    */
} lgp_sample_out;

/* Destination buffers of lgp_build_blocks: the sampled sub-graph as one bipartite CSR block
 * per hop, in local numbering (what a GNN layer consumes). */
typedef struct {
  int64_t* blk_indptr[LGP_MAX_HOPS];   /* [device] cap[h] + 1: blk_indptr[h][i] = sampled edges of the destinations
                                          before frontier[h][i]                                                  */
  int32_t* blk_src[LGP_MAX_HOPS];      /* [device] cap[h] * fanouts[h]: position of each sampled neighbour inside
                                          frontier[h + 1], destination by destination, in slot order             */
  int32_t* feat_row[LGP_MAX_HOPS + 1]; /* [device] cap[h]: position of frontier[h][i] inside gather_ids = its row
                                          in the matrix lgp_gather_features(gather_ids) returns; 0 <= h <= n_hops */
} lgp_blocks_out;

/* Accumulated HIP-event timings of the per-batch kernels (see lgp_set_profiling). */
typedef struct {
  int64_t n_sample, n_partition, n_hit, n_miss; /* launches / calls timed          */
  double ms_sample;     /* whole lgp_sample_khop calls (all hops + dedup)          */
  double ms_partition;  /* cache lookup + hit/miss partition kernel                */
  double ms_hit;        /* row gather of cache hits (HBM -> HBM)                   */
  double ms_miss;       /* row gather of misses (pinned host -> HBM over PCIe)     */
} lgp_profile;

/* Pinned, GPU-addressable host memory for the graph arrays (plain hipHostMalloc /
 * hipHostFree; synchronous).  lgp_host_alloc returns LGP_ENOMEM on failure. */
int lgp_host_alloc(size_t bytes, void** out);
int lgp_host_free(void* ptr);

/* Create a context for `g` on GPU `device`.  Validates sizes and pointer kinds
 * (LGP_EINVAL if an array is not GPU-addressable) and allocates the per-vertex
 * lookup state in HBM: a row table (offset + degree + "cached" flag, 8 bytes per
 * vertex, filled from indptr), the feature remap, two hotness vectors and the dedup
 * bitmaps -- about 20.3 bytes per vertex, outside the cache budgets.  It starts with
 * empty caches, so sampling and gathering already work, with every column id and
 * feature row read from CPU memory (Sec. 3.2's mode with the topology kept in CPU memory).
 * Synchronous. */
int lgp_create(const lgp_graph* g, int device, lgp_ctx** out);
int lgp_destroy(lgp_ctx* ctx);

/* Batch generator (Sec. 5, the first operator of the sampling server: a per-epoch shuffle of
 * this GPU's training vertices, cut into mini-batches of seeds).  out[j] = in[pi(j)] where pi orders the positions 0 .. n-1 by the
 * 64-bit Philox4x32-10 draw keyed (seed, position, epoch, 0), ascending, ties by position:
 * a reproducible permutation per epoch.  in / out are [device], n ids each, and must not
 * overlap.  Needs no context; runs on `device`; allocates sort scratch; synchronous. */
int lgp_shuffle_tablet(int device, const int32_t* in, int32_t* out, int64_t n, uint64_t seed, uint32_t epoch,
                       void* stream);

/* Pre-sampling (Sec. 4.2.2, step S1).  The tablet train_ids [device, n_train ids,
 * already in epoch order] is cut into consecutive mini-batches of `batch` seeds (the
 * last may be short); batch b is sampled with rng seed base_seed + b; column ids come
 * from CPU memory unless a topology cache was built before.  For every expanded vertex its topology hotness grows by
 * the number of edges sampled out of it; for every distinct vertex of a batch's
 * result (seeds included) its feature hotness grows by one.  Both vectors are reset
 * first.  max_batches < 0 processes the whole tablet once.  fanouts is [host]. */
int lgp_build_hotness(lgp_ctx* ctx, const int32_t* train_ids, int64_t n_train, int32_t batch,
                      const int32_t* fanouts, int32_t n_hops, uint64_t base_seed, int64_t max_batches,
                      void* stream);

/* What the last lgp_build_hotness did: mini-batches processed and vertex expansions performed
 * (the sum of all frontier sizes).  During pre-sampling every expansion reads its column ids
 * from CPU memory, so n_expansions is the exact count of row reads over PCIe -- on this GPU one
 * 128-byte line each for all but very long rows -- and serves as N_TSUM for
 * lgp_search_cache_plan (with cls_bytes = 128).  Synchronous. */
int lgp_get_presample_stats(lgp_ctx* ctx, int64_t* n_batches, int64_t* n_expansions);

/* Copy the hotness vectors (uint32[V] each) to / from [host] memory; either pointer
 * may be NULL.  Synchronous.  lgp_set_hotness lets a saved ranking be reused. */
int lgp_get_hotness(lgp_ctx* ctx, uint32_t* topo_hot, uint32_t* feat_hot);
int lgp_set_hotness(lgp_ctx* ctx, const uint32_t* topo_hot, const uint32_t* feat_hot);

/* Cache candidate selection and fill-up (Sec. 4.2.2 steps S2-S3; Algorithm 1 with one
 * GPU per clique reduces to ranking vertices by descending hotness, ties by ascending
 * id).  The topology cache takes the longest prefix of the topology ranking whose
 * cost sum(deg * 4 + 8) stays within topo_budget (Eq. 3); the feature cache takes
 * min(V, feat_budget / (D * elem_bytes)) rows of the feature ranking (Eq. 6).  Rows
 * are copied from CPU memory in rank order; cache slot = rank (one exception, invisible
 * through this interface: a feature cache that holds every vertex is laid out in vertex
 * order, so that no lookup is needed to find a row).  Replaces any earlier cache.  Needs hotness (LGP_ESTATE otherwise).  Allocates device memory and
 * synchronises `stream`.  lgp_plan_cache only reports the sizes. */
int lgp_plan_cache(lgp_ctx* ctx, uint64_t topo_budget, uint64_t feat_budget, lgp_cache_plan* plan, void* stream);
int lgp_build_cache(lgp_ctx* ctx, uint64_t topo_budget, uint64_t feat_budget, void* stream);
int lgp_get_cache_plan(lgp_ctx* ctx, lgp_cache_plan* plan);

/* One candidate of the cache-plan search: what alpha = index / (n_alpha - 1) would cache. */
typedef struct {
  uint64_t m_topo, m_feat;        /* bytes for the two caches: m_topo = floor(B * alpha), m_feat = B - m_topo */
  int64_t n_topo, n_feat;         /* cached vertices under Eq. 3 / Eq. 6                                      */
  uint64_t uncached_topo_hot;     /* sum of topology hotness outside the cache; N_T = N_TSUM * this / total   */
  uint64_t uncached_feat_hot;     /* U_F of Eq. 7; N_F = ceil(row_bytes / CLS) * this                          */
} lgp_plan_point;

/* Automatic cache management (Sec. 4.3): evaluate the cost model N_total = N_T + N_F
 * (Eq. 2-8) for alpha = 0, 1/(n_alpha-1), ..., 1 with inclusive scans along the two
 * rankings and one binary search per candidate (Sec. 4.3.3), and return the index of the
 * smallest N_total in *best (ties: smallest alpha; plans are compared exactly, by cross
 * multiplication).  total_budget is B in bytes, n_tsum the number of PCIe transactions
 * that topology reads caused during pre-sampling (N_TSUM; the sum of topology hotness is
 * a software stand-in: one transaction per traversed edge), cls_bytes the transfer
 * granularity CLS of Eq. 8.  points [host, n_alpha entries, may be NULL] receives every
 * candidate.  2 <= n_alpha <= 1024.  Needs hotness; must be called before lgp_build_cache
 * (LGP_ESTATE otherwise).  Synchronous. */
int lgp_search_cache_plan(lgp_ctx* ctx, uint64_t total_budget, uint64_t n_tsum, uint32_t cls_bytes, int32_t n_alpha,
                          lgp_plan_point* points, int32_t* best, void* stream);

/* Cache candidate selection for a clique of k_g GPUs (Algorithm 1, "Complete Sharing with
 * Local Preference").  hot [device] is the k_g x V hotness matrix, row-major, one row per
 * GPU of the clique.  Outputs, all [device] unless noted: acc[V] = column sums (step 1);
 * order[V] = vertex ids by descending acc, ties by ascending id (step 2); owner[V] = the GPU
 * with the largest local hotness of each vertex, ties to the lowest GPU index (step 3's
 * arg-max); queues[V] = the k_g per-GPU queues laid end to end, each in `order` order;
 * queue_offsets [host, k_g + 1] delimits them.  1 <= k_g <= 64.  With k_g = 1 this is the
 * plain ranking lgp_build_cache uses.  Needs no context; runs on `device`; synchronous. */
int lgp_cslp(int device, int32_t k_g, int64_t num_vertices, const uint32_t* hot, uint64_t* acc, int32_t* order,
             int32_t* owner, int32_t* queues, int64_t* queue_offsets, void* stream);

/* Unified cache of a whole clique of k_g GPUs, held by this one device (Sec. 4.2.2, S2 and
 * S3, for K_g > 1; Sec. 3.1, O1: GPUs of a clique read one another's caches).  The k_g
 * member GPUs are simulated: each member's cache is a region of its own in this device's HBM,
 * so a "peer" read is a read of another region.  topo_hot and feat_hot [device] are the
 * k_g x V hotness matrices H_T and H_F, row-major (one row per member; lgp_build_hotness on
 * the member's tablet followed by lgp_get_hotness yields a row).  Algorithm 1 turns each
 * matrix into k_g queues; member g then fills its topology cache with the longest prefix of
 * its queue G_T[g] whose Eq. 3 cost fits topo_budget bytes, and its feature cache with the
 * first floor(feat_budget / row_bytes) entries of G_F[g] -- both budgets are per member.  No
 * vertex is cached twice.  Replaces any earlier cache; afterwards lgp_sample_khop reads
 * every member's cached rows from HBM, lgp_gather_features counts a row cached by any
 * member as a hit, lgp_get_cache returns the members' parts end to end (member 0 first, each
 * in fill order) and lgp_get_cache_plan their totals.  1 <= k_g <= LGP_MAX_CLIQUE.
 * Synchronous. */
#define LGP_MAX_CLIQUE 8
int lgp_build_clique_cache(lgp_ctx* ctx, int32_t k_g, const uint32_t* topo_hot, const uint32_t* feat_hot,
                           uint64_t topo_budget, uint64_t feat_budget, void* stream);

/* What member `member` of the clique cache holds (its share of lgp_get_cache's arrays starts
 * where the shares of the members before it end).  LGP_ESTATE without a clique cache. */
int lgp_get_clique_plan(lgp_ctx* ctx, int32_t member, lgp_cache_plan* plan);

/* Feature extraction as member `member` of the clique sees it: like lgp_gather_features, but
 * the ids are split three ways -- rows in the member's own cache, rows in a peer's cache (both
 * HBM reads here, gathered by separate launches) and rows in no cache (read in place from CPU
 * memory).  stats [device int32[3], may be NULL] receives {n_local, n_miss, n_peer}.
 * LGP_ESTATE without a clique cache. */
int lgp_gather_features_clique(lgp_ctx* ctx, int32_t member, const int32_t* ids, int64_t n_max, const int32_t* n_dev,
                               void* out, int32_t* stats, void* stream);

/* Copy the cache to [host] memory for inspection; any pointer may be NULL.
 * topo_ids[n_topo], t_indptr[n_topo + 1], t_indices[topo_edges], feat_ids[n_feat],
 * feat_rows[n_feat * D * elem_bytes].  Synchronous. */
int lgp_get_cache(lgp_ctx* ctx, int32_t* topo_ids, int64_t* t_indptr, int32_t* t_indices, int32_t* feat_ids,
                  void* feat_rows);

/* A slice of the cache contents, for inspecting caches too large to copy in one piece.  which = 0:
 * t_indices[first .. first + count), int32 entries; which = 1: the feature rows of ranks first ..
 * first + count - 1, row_bytes each (rank order, as lgp_get_cache returns them).  dst is [host].
 * LGP_EINVAL if the range leaves the cache.  Synchronous. */
int lgp_get_cache_part(lgp_ctx* ctx, int32_t which, int64_t first, int64_t count, void* dst);

/* k-hop uniform neighbour sampling of one mini-batch (Sec. 2.2 step 2; the neighbour
 * sampler of Sec. 5).  seeds is [device], n_seeds distinct ids; fanouts is [host],
 * 1 <= fanouts[h] <= LGP_MAX_FANOUT, 1 <= n_hops <= LGP_MAX_HOPS.  A vertex of degree
 * d <= fanout yields all its neighbours in CSR order; otherwise `fanout` distinct
 * positions are chosen by Floyd's subset algorithm from Philox4x32-10 draws keyed by
 * (rng_seed, vertex, hop, slot).  Adjacency comes from the topology cache when the
 * vertex is cached, from CPU memory otherwise; the result does not depend on which.
 * Frontier h + 1 is the ascending unique set of hop h's samples.  No host
 * synchronisation: sizes stay on the device (out->n_frontier, out->n_gather). */
int lgp_sample_khop(lgp_ctx* ctx, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                    uint64_t rng_seed, const lgp_sample_out* out, void* stream);

/* One mini-batch through the intra-batch pipeline of Sec. 5 (one batch's sampling runs beside its own
 * feature extraction): lgp_sample_khop and lgp_gather_features in one call, with the
 * extraction running on a stream of the library's own beside the sampling.  That is only possible if rows are
 * extracted in the order in which the sampler reaches their vertices, so out->gather_ids is not the ascending
 * list here but the listing
 *     seeds as given | vertices first reached by hop 0, ascending | ... | first reached by hop n_hops-1, ascending
 * (a vertex is "first reached" by a hop if it is among that hop's samples and is neither a seed nor among the
 * samples of an earlier hop; as a set the listing equals lgp_sample_khop's gather_ids).  The seeds' rows are
 * extracted while hop 0 is sampled, hop h's group while hop h+1 is sampled, the last group after the last hop.
 * Everything else in `out` is what lgp_sample_khop writes (frontiers, nbr, cnt, counts; *out->n_gather = length
 * of the listing).  rows [device] receives the feature row of gather_ids[i] at row i, like lgp_gather_features;
 * groups [device int32[n_hops + 2], may be NULL] receives the group bounds (groups[0] = 0, groups[1] = n_seeds,
 * group g = [groups[g], groups[g+1])); stats [device int32[2], may be NULL] = {n_hit, n_miss} over all groups.
 * Seeds must be distinct (a repeated seed is listed, and its row extracted, once per occurrence;
 * out->gather_cap must also be >= n_seeds).  `stream` waits for the extraction before later work on it runs.
 * lgp_build_blocks accepts the result (its feat_row then points into this listing).  Not to be overlapped with
 * lgp_sample_khop, lgp_gather_features or another lgp_sample_extract on the same context. */
int lgp_sample_extract(lgp_ctx* ctx, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                       uint64_t rng_seed, const lgp_sample_out* out, void* rows, int32_t* groups, int32_t* stats,
                       void* stream);

/* Graph constructor (Sec. 5, the fourth operator: it turns the sampled neighbour lists into the
 * per-hop subgraph).  Takes the buffers a finished lgp_sample_khop call filled (same seeds, fanouts
 * and `sampled`, with sampled->frontier[n_hops] given) and writes, per hop h, a bipartite
 * block in CSR form whose destinations are frontier h and whose sources are frontier h+1,
 * plus for every frontier the rows of its vertices in the extracted feature matrix.
 * Everything is read from device memory; no host synchronisation.  Unless lgp_reserve sized
 * the scratch beforehand, the first call (and a later one with more hops) allocates n_hops + 1
 * lookup tables of V 4-byte entries and a small scan scratch, and synchronises once. */
int lgp_build_blocks(lgp_ctx* ctx, const int32_t* seeds, int32_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                     const lgp_sample_out* sampled, const lgp_blocks_out* out, void* stream);

/* Feature extraction (Sec. 2.2 step 3; the feature extractor of Sec. 5):
 * out[i, :] = features[ids[i], :] for i < n, byte for byte.  ids is [device] (any
 * order, duplicates allowed); n = *n_dev if n_dev [device int32] is given, else n_max;
 * out is [device] with room for n_max rows.  Ids are split into cache hits (rows read
 * from the HBM feature cache) and misses (rows read in place from CPU memory over
 * PCIe); stats [device int32[2], may be NULL] receives {n_hit, n_miss} (unspecified if
 * lgp_check then reports an invalid id).  When every row is cached, or none, the split is
 * skipped and one gather looks the ids up itself.  Otherwise scratch for the two lists
 * grows on demand (a growth step allocates and synchronises) unless lgp_reserve sized it
 * beforehand; lgp_gather_features_static needs neither. */
int lgp_gather_features(lgp_ctx* ctx, const int32_t* ids, int64_t n_max, const int32_t* n_dev, void* out,
                        int32_t* stats, void* stream);

/* For callers that cannot allocate device memory -- code under HIP-graph capture without a warm-up call,
 * tight serving loops, harnesses that forbid hipMalloc: lgp_gather_features with the same arguments, results
 * and errors, but its scratch (the hit / miss counters and the four partition lists) lives in a fixed
 * 64 MiB block of device memory that is part of the library image, so the call allocates and frees nothing,
 * creates no events (it is never timed by lgp_set_profiling) and never synchronises.  n_max above
 * LGP_STATIC_GATHER_MAX_IDS is refused with LGP_ECAPACITY before anything is launched.  Every call on a GPU,
 * from any context, uses that GPU's one block: calls that overlap in time on one GPU race; order them on one
 * stream or with events.  The block keeps the last call's contents; the call clears the counters itself with
 * a small kernel (no memset node, so it may be captured) and never reads list entries it did not write. */
#define LGP_STATIC_GATHER_MAX_IDS (1 << 22)
int lgp_gather_features_static(lgp_ctx* ctx, const int32_t* ids, int64_t n_max, const int32_t* n_dev, void* out,
                               int32_t* stats, void* stream);

/* By default lgp_gather_features runs the hit gather and then the miss gather on
 * `stream`.  With overlap enabled the miss gather runs on a stream of the library's own
 * beside the hit gather, which is then launched a quarter as wide so that its requests do
 * not crowd the PCIe reads, and `stream` waits for both.  Measured on MI355X with misses
 * dominating (2.4 M vertices, 400-byte rows, 30 % of them cached): 2.49 ms per step instead
 * of 2.56 ms.  The hit gather itself takes many times longer that way (PCIe reads queued
 * ahead of it throttle it), so per-kernel timings are only meaningful with overlap off,
 * which is the default.  A process has a few hardware queues (four by default) and HIP
 * spreads streams over them: if the library's stream and `stream` happen to share one, the
 * result is the same but the two gathers run one after the other.  The same holds for
 * lgp_sample_extract's stream. */
int lgp_set_overlap(lgp_ctx* ctx, int enable);

/* HBM the library holds or will allocate on its own for calls of one shape, in bytes, so that a
 * caller can budget device memory before building caches (Sec. 4.3.1: B is what is left after
 * everything else is reserved).  fixed [host] = the per-context tables that exist since
 * lgp_create (row table, feature remap, hotness vectors, dedup bitmaps, rankings once a plan
 * was made); scratch [host] = what pre-sampling, lgp_gather_features(_clique) with up to the
 * worst-case number of ids and lgp_build_blocks allocate on first use for batches of up to
 * max_seeds seeds with these fan-outs.  The caches themselves are reported by lgp_plan_cache /
 * lgp_get_cache_plan.  Either pointer may be NULL.  Nothing is allocated or launched. */
int lgp_workspace_bytes(const lgp_ctx* ctx, int32_t max_seeds, const int32_t* fanouts, int32_t n_hops, size_t* fixed,
                        size_t* scratch);

/* Allocate, now, every scratch buffer that lgp_sample_khop, lgp_build_blocks, lgp_gather_features(_clique)
 * and lgp_build_hotness use for batches of up to max_seeds seeds with these fan-outs (the amount
 * lgp_workspace_bytes reports as `scratch`).  Afterwards those per-batch calls never allocate, free or
 * synchronise -- they may be captured into a HIP graph without a warm-up call -- and a call whose shape
 * exceeds the reservation returns LGP_ECAPACITY instead of growing the scratch.  May be called again with a
 * larger shape.  Without it the scratch grows on demand, as described at each call.  fanouts is [host].
 * Synchronous. */
int lgp_reserve(lgp_ctx* ctx, int32_t max_seeds, const int32_t* fanouts, int32_t n_hops);

/* Sticky device-side error flag (invalid vertex id met by a kernel, output overrun).
 * Synchronises `stream`, returns LGP_EDEVICE if set, and clears it. */
int lgp_check(lgp_ctx* ctx, void* stream);

/* HIP-event timing of the per-batch kernels, recorded on the streams they run on.
 * mode 0 = off, 1 = every kernel group of lgp_profile, 2 = only the two row gathers
 * (hits, misses).  The gather launches record their own start and stop times; the groups
 * of several launches (sampling, partition) are bracketed by two recorded events, each of
 * which costs a few microseconds of stream time -- visible in steps that take a fraction of
 * a millisecond, hence mode 2.  Keep profiling off while calls are captured into a HIP
 * graph: timed launches are not capturable.  lgp_get_profile waits for the recorded events, adds
 * them up and resets. */
int lgp_set_profiling(lgp_ctx* ctx, int mode);
int lgp_get_profile(lgp_ctx* ctx, lgp_profile* out);

const char* lgp_strerror(int status);
const char* lgp_last_error(const lgp_ctx* ctx); /* text of the last failure on this context */

#ifdef __cplusplus
}
#endif
#endif /* LEGION_PREP_H */
