// CPU oracle for the mini-batch data-preparation path of a cache-based GNN
// training system (pre-sampling hotness, hotness-ranked topology/feature
// caches, k-hop uniform neighbour sampling, feature extraction).
//
// THIS IS TEST INFRASTRUCTURE.  It is a plain, single-threaded, deliberately
// slow definition of what the path computes.  Only the tests, the smoke check
// and the bench's cpu_baseline leg may load it; the product library shares no
// code with it and never calls it.
//
// What the paper fixes, and what this file adds where the paper is silent:
//   * workflow (Sec. 2.2): pick a mini-batch, uniformly sample several hops of
//     fixed-size neighbour sets, extract the features of seeds and samples.
//   * hotness (Sec. 4.2.2, step S1): topology hotness of a vertex grows by one
//     for every edge traversed out of it; feature hotness grows by one for
//     every vertex present in a mini-batch's sample result.
//   * ranking (Algorithm 1 with one GPU per clique): vertices ordered by
//     descending hotness.  Tie-break (paper silent): ascending vertex id.
//   * cache size rule (Eq. 3 and Eq. 6): a cached topology row costs
//     4 bytes per neighbour plus 8 bytes; a cached feature row costs
//     D * element size.  The cached set is the longest prefix of the ranking
//     whose total cost does not exceed the budget (the paper fills the cache
//     up to size m; read as <=).
//   * cache layout (Sec. 4.2.1): topology cache = CSR over the cached rows in
//     rank order; feature cache = 2-D array, one row per cached vertex in rank
//     order.
//   * RNG (paper silent): Philox4x32-10 (Salmon et al., SC'11), one call per
//     (seed, vertex, hop, slot).
//   * subset selection (the paper only asks for a uniform sample of fixed size): rows with
//     degree <= fanout are returned whole; otherwise Floyd's subset algorithm.
//   * frontier semantics (paper silent): the next frontier is the ascending
//     sorted set of the current hop's sampled neighbours; the set of vertices
//     whose features are extracted is the ascending sorted union of the seeds
//     and all sampled neighbours.
//
//   * extraction order of the intra-batch pipeline (Sec. 5; order not stated): seeds as
//     given, then per hop the vertices first reached by that hop, ascending.
//
//   * cache plan search (Sec. 4.3): for alpha = 0, 1/(n-1), ..., 1 the topology cache gets
//     m_T = floor(B * alpha) bytes and the feature cache B - m_T; N_total = N_T + N_F with
//     Eq. 3-8, the plan with the smallest N_total wins (paper silent on ties: smallest
//     alpha).  N_T is a ratio of integers, so plans are compared exactly by cross
//     multiplication instead of in floating point.
//
//   * clique of several GPUs (Algorithm 1 in full; Sec. 4.2.2 S2-S3; Sec. 3.1 O1): column sums,
//     ranking, arg-max owner (ties, paper silent: lowest GPU index), per-GPU queues; each GPU
//     caches the longest prefix of its own queue that fits its own budget; a GPU's extraction
//     finds a row in its own cache, in a peer's, or in CPU memory.
//   * batch generator and graph constructor (Sec. 5): a Philox-keyed shuffle of the tablet per
//     epoch; per hop a bipartite block in CSR form over local numbering (format: paper silent).
//
// Every function has a pin in tests/ (known-answer vectors, brute force,
// closed forms or library routines); none is "parity unpinned".

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

struct Graph {
  int64_t num_vertices;
  const void* indptr;     // num_vertices + 1 offsets
  int32_t indptr_bytes;   // 4 or 8
  const int32_t* indices; // column ids
};

inline int64_t row_begin(const Graph& g, int64_t v) {
  if (g.indptr_bytes == 8) return static_cast<const int64_t*>(g.indptr)[v];
  return static_cast<const int32_t*>(g.indptr)[v];
}

// ---------------------------------------------------------------------------
// Philox4x32-10.  Counter c[4], key k[2], ten rounds; the key is bumped by the
// Weyl constants before every round but the first.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += W0; k1 += W1; }
    const uint64_t p0 = M0 * c0;
    const uint64_t p1 = M1 * c2;
    const uint32_t hi0 = static_cast<uint32_t>(p0 >> 32), lo0 = static_cast<uint32_t>(p0);
    const uint32_t hi1 = static_cast<uint32_t>(p1 >> 32), lo1 = static_cast<uint32_t>(p1);
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// One 64-bit draw for (rng_seed, vertex, hop, slot): counter = (vertex low
// word, vertex high word, hop, slot), key = (seed low word, seed high word);
// the draw is output word 0 (low half) and word 1 (high half).
uint64_t draw64(uint64_t rng_seed, int64_t v, int32_t hop, int32_t slot) {
  const uint32_t ctr[4] = {static_cast<uint32_t>(static_cast<uint64_t>(v)),
                           static_cast<uint32_t>(static_cast<uint64_t>(v) >> 32),
                           static_cast<uint32_t>(hop), static_cast<uint32_t>(slot)};
  const uint32_t key[2] = {static_cast<uint32_t>(rng_seed), static_cast<uint32_t>(rng_seed >> 32)};
  uint32_t out[4];
  philox4x32_10(ctr, key, out);
  return static_cast<uint64_t>(out[0]) | (static_cast<uint64_t>(out[1]) << 32);
}

// Map a 64-bit draw onto {0, ..., n-1}: floor(r * n / 2^64).
inline uint64_t scale_draw(uint64_t r, uint64_t n) {
  return static_cast<uint64_t>((static_cast<unsigned __int128>(r) * n) >> 64);
}

// ---------------------------------------------------------------------------
// Uniform fixed-size neighbour sample of one vertex (Sec. 2.2, step 2).
// Returns the number of valid entries; out[] has f entries, -1 padded.
// ---------------------------------------------------------------------------
int32_t sample_row(const Graph& g, int64_t v, int32_t hop, int32_t f, uint64_t rng_seed, int32_t* out) {
  const int64_t s = row_begin(g, v);
  const int64_t d = row_begin(g, v + 1) - s;
  for (int32_t i = 0; i < f; ++i) out[i] = -1;
  if (d <= f) {
    for (int64_t i = 0; i < d; ++i) out[i] = g.indices[s + i];
    return static_cast<int32_t>(d);
  }
  // Floyd: for j = d-f .. d-1 pick t uniform in [0, j]; take t unless already
  // taken, in which case take j.
  std::vector<int64_t> pos;
  pos.reserve(f);
  for (int32_t i = 0; i < f; ++i) {
    const int64_t j = d - f + i;
    const int64_t t = static_cast<int64_t>(scale_draw(draw64(rng_seed, v, hop, i), static_cast<uint64_t>(j) + 1));
    const bool taken = std::find(pos.begin(), pos.end(), t) != pos.end();
    const int64_t p = taken ? j : t;
    pos.push_back(p);
    out[i] = g.indices[s + p];
  }
  return f;
}

struct Batch {
  int32_t n_hops = 0;
  std::vector<std::vector<int32_t>> frontier; // frontier[h], h = 0..n_hops (the last one is never expanded)
  std::vector<std::vector<int32_t>> nbr;      // nbr[h]: frontier[h].size() * fanouts[h]
  std::vector<std::vector<int32_t>> cnt;      // cnt[h]: frontier[h].size()
  std::vector<int32_t> gather_ids;
};

void sorted_unique(std::vector<int32_t>& a) {
  std::sort(a.begin(), a.end());
  a.erase(std::unique(a.begin(), a.end()), a.end());
}

// k-hop sampling of one mini-batch.
void sample_khop(const Graph& g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                 uint64_t rng_seed, Batch& b) {
  b.n_hops = n_hops;
  b.frontier.assign(n_hops + 1, {});
  b.nbr.assign(n_hops, {});
  b.cnt.assign(n_hops, {});
  std::vector<int32_t> all(seeds, seeds + n_seeds);
  std::vector<int32_t> cur(seeds, seeds + n_seeds);
  for (int32_t h = 0; h < n_hops; ++h) {
    const int32_t f = fanouts[h];
    b.frontier[h] = cur;
    b.nbr[h].assign(cur.size() * static_cast<size_t>(f), -1);
    b.cnt[h].assign(cur.size(), 0);
    std::vector<int32_t> next;
    for (size_t i = 0; i < cur.size(); ++i) {
      int32_t* row = b.nbr[h].data() + i * static_cast<size_t>(f);
      const int32_t c = sample_row(g, cur[i], h, f, rng_seed, row);
      b.cnt[h][i] = c;
      for (int32_t k = 0; k < f; ++k)
        if (row[k] >= 0) next.push_back(row[k]);
    }
    all.insert(all.end(), next.begin(), next.end());
    sorted_unique(next);
    cur.swap(next);
  }
  b.frontier[n_hops] = cur;
  sorted_unique(all);
  b.gather_ids.swap(all);
}

} // namespace

extern "C" {

struct orc_graph {
  int64_t num_vertices;
  const void* indptr;
  int32_t indptr_bytes;
  const int32_t* indices;
};

static Graph to_graph(const orc_graph* g) { return Graph{g->num_vertices, g->indptr, g->indptr_bytes, g->indices}; }

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox4x32_10(ctr, key, out); }

uint64_t orc_draw64(uint64_t rng_seed, int64_t v, int32_t hop, int32_t slot) { return draw64(rng_seed, v, hop, slot); }

int32_t orc_sample_row(const orc_graph* g, int64_t v, int32_t hop, int32_t f, uint64_t rng_seed, int32_t* out) {
  return sample_row(to_graph(g), v, hop, f, rng_seed, out);
}

// --- k-hop sampling: result handle + accessors -----------------------------
void* orc_sample_khop(const orc_graph* g, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts,
                      int32_t n_hops, uint64_t rng_seed) {
  Batch* b = new Batch();
  sample_khop(to_graph(g), seeds, n_seeds, fanouts, n_hops, rng_seed, *b);
  return b;
}
int64_t orc_batch_frontier_size(const void* h, int32_t hop) { return (int64_t) static_cast<const Batch*>(h)->frontier[hop].size(); }
const int32_t* orc_batch_frontier(const void* h, int32_t hop) { return static_cast<const Batch*>(h)->frontier[hop].data(); }
const int32_t* orc_batch_nbr(const void* h, int32_t hop) { return static_cast<const Batch*>(h)->nbr[hop].data(); }
const int32_t* orc_batch_cnt(const void* h, int32_t hop) { return static_cast<const Batch*>(h)->cnt[hop].data(); }
int64_t orc_batch_gather_size(const void* h) { return (int64_t) static_cast<const Batch*>(h)->gather_ids.size(); }
const int32_t* orc_batch_gather_ids(const void* h) { return static_cast<const Batch*>(h)->gather_ids.data(); }
void orc_batch_free(void* h) { delete static_cast<Batch*>(h); }

// --- batch generator (Sec. 5, operator 1) -------------------------------------
// The operator reorders this GPU's training vertices once per epoch and cuts the order into
// mini-batches of seeds.  The paper names no particular shuffle; here position i of the tablet gets the 64-bit key draw64(seed, i, epoch, 0) and
// the tablet is reordered by ascending key (ties by position), so every epoch has its own
// reproducible order.
void orc_shuffle_tablet(const int32_t* in, int32_t* out, int64_t n, uint64_t seed, uint32_t epoch) {
  std::vector<std::pair<uint64_t, int64_t>> keyed(n);
  for (int64_t i = 0; i < n; ++i) keyed[i] = {draw64(seed, i, static_cast<int32_t>(epoch), 0), i};
  std::sort(keyed.begin(), keyed.end());
  for (int64_t i = 0; i < n; ++i) out[i] = in[keyed[i].second];
}

// --- graph constructor (Sec. 5, operator 4) ----------------------------------
// The paper only says that the constructor builds the subgraph from the sampler's
// output.  Reading used here: hop h becomes a bipartite block in CSR form whose
// destinations are frontier h (in order) and whose sources are frontier h+1;
// blk_indptr[i] = number of sampled edges of destinations before i, blk_src[e] = position of
// the e-th sampled neighbour inside frontier h+1; feat_row[i] = position of frontier h's i-th
// vertex inside gather_ids, i.e. its row in the extracted feature matrix.
void orc_block_of_hop(const void* handle, int32_t hop, int32_t fanout, int64_t* blk_indptr, int32_t* blk_src) {
  const Batch& b = *static_cast<const Batch*>(handle);
  const std::vector<int32_t>& src_set = b.frontier[hop + 1];
  int64_t e = 0;
  blk_indptr[0] = 0;
  for (size_t i = 0; i < b.frontier[hop].size(); ++i) {
    for (int32_t k = 0; k < fanout; ++k) {
      const int32_t u = b.nbr[hop][i * static_cast<size_t>(fanout) + k];
      if (u < 0) continue;
      blk_src[e++] = static_cast<int32_t>(std::lower_bound(src_set.begin(), src_set.end(), u) - src_set.begin());
    }
    blk_indptr[i + 1] = e;
  }
}
void orc_feature_rows(const void* handle, int32_t hop, int32_t* feat_row) {
  const Batch& b = *static_cast<const Batch*>(handle);
  for (size_t i = 0; i < b.frontier[hop].size(); ++i)
    feat_row[i] = static_cast<int32_t>(std::lower_bound(b.gather_ids.begin(), b.gather_ids.end(), b.frontier[hop][i]) -
                                       b.gather_ids.begin());
}

// --- extraction order of the intra-batch pipeline (Sec. 5) ------------------
// Sec. 5: within one batch, sampling and graph construction can run beside feature
// extraction.  The extractor can only run ahead of the sampler if it takes the vertices in
// the order in which the sampler reaches them (paper silent on that order; reading): first
// the seeds as given, then, hop after hop, the vertices that hop reaches for the first time
// -- the members of frontier h (h = 1 .. n_hops) that are neither seeds nor members of an
// earlier frontier -- each group in ascending order.  seg (n_hops + 2 entries) delimits the
// groups: seg[0] = 0, seg[1] = number of seeds, seg[h + 1] = end of hop h's group.  Returns
// the total; call with out == nullptr to learn it.
int64_t orc_hop_order(const void* handle, int64_t num_vertices, int32_t* out, int64_t* seg) {
  const Batch& b = *static_cast<const Batch*>(handle);
  std::vector<uint8_t> seen(static_cast<size_t>(num_vertices), 0);
  int64_t at = 0;
  seg[0] = 0;
  for (int32_t v : b.frontier[0]) {            // the seed list, duplicates and all
    if (out) out[at] = v;
    ++at;
    seen[v] = 1;
  }
  seg[1] = at;
  for (int32_t h = 1; h <= b.n_hops; ++h) {
    for (int32_t v : b.frontier[h]) {          // ascending by construction
      if (seen[v]) continue;
      seen[v] = 1;
      if (out) out[at] = v;
      ++at;
    }
    seg[h + 1] = at;
  }
  return at;
}

// --- pre-sampling hotness (Sec. 4.2.2, S1) ---------------------------------
// The tablet is consumed in consecutive slices of `batch` ids (last slice may
// be short); slice b is sampled with rng seed base_seed + b.  max_batches < 0
// means the whole tablet once.  Returns the number of batches processed.
int64_t orc_build_hotness(const orc_graph* g, const int32_t* train_ids, int64_t n_train, int32_t batch,
                          const int32_t* fanouts, int32_t n_hops, uint64_t base_seed, int64_t max_batches,
                          uint32_t* topo_hot, uint32_t* feat_hot) {
  const Graph G = to_graph(g);
  std::memset(topo_hot, 0, sizeof(uint32_t) * G.num_vertices);
  std::memset(feat_hot, 0, sizeof(uint32_t) * G.num_vertices);
  int64_t n_batches = (n_train + batch - 1) / batch;
  if (max_batches >= 0 && max_batches < n_batches) n_batches = max_batches;
  for (int64_t b = 0; b < n_batches; ++b) {
    const int64_t lo = b * batch;
    const int64_t hi = std::min<int64_t>(n_train, lo + batch);
    Batch res;
    sample_khop(G, train_ids + lo, hi - lo, fanouts, n_hops, base_seed + static_cast<uint64_t>(b), res);
    for (int32_t h = 0; h < n_hops; ++h)
      for (size_t i = 0; i < res.frontier[h].size(); ++i)
        topo_hot[res.frontier[h][i]] += static_cast<uint32_t>(res.cnt[h][i]); // one per traversed edge
    for (int32_t u : res.gather_ids) feat_hot[u] += 1;
  }
  return n_batches;
}

// --- ranking (Algorithm 1, one GPU): descending hotness, ascending id -------
void orc_rank_by_hotness(const uint32_t* hot, int64_t num_vertices, int32_t* order) {
  for (int64_t v = 0; v < num_vertices; ++v) order[v] = static_cast<int32_t>(v);
  std::stable_sort(order, order + num_vertices, [hot](int32_t a, int32_t b) { return hot[a] > hot[b]; });
}

// --- Eq. 3: longest prefix of the topology ranking within the byte budget ---
int64_t orc_plan_topo(const orc_graph* g, const int32_t* order, uint64_t topo_budget) {
  const Graph G = to_graph(g);
  uint64_t used = 0;
  int64_t n = 0;
  for (; n < G.num_vertices; ++n) {
    const int64_t v = order[n];
    const uint64_t cost = static_cast<uint64_t>(row_begin(G, v + 1) - row_begin(G, v)) * 4u + 8u;
    if (used + cost > topo_budget) break;
    used += cost;
  }
  return n;
}

// --- Eq. 6: number of feature rows within the byte budget -------------------
int64_t orc_plan_feat(int64_t num_vertices, int64_t row_bytes, uint64_t feat_budget) {
  uint64_t used = 0;
  int64_t n = 0;
  for (; n < num_vertices; ++n) {
    if (used + static_cast<uint64_t>(row_bytes) > feat_budget) break;
    used += static_cast<uint64_t>(row_bytes);
  }
  return n;
}

// --- cache fill-up (Sec. 4.2.2, S3) -----------------------------------------
// Topology cache: CSR over the first n ranked vertices.  t_indptr has n + 1
// entries; t_indices must hold t_indptr[n] entries (call once with
// t_indices == nullptr to learn the size).
int64_t orc_fill_topo(const orc_graph* g, const int32_t* order, int64_t n, int64_t* t_indptr, int32_t* t_indices) {
  const Graph G = to_graph(g);
  int64_t at = 0;
  t_indptr[0] = 0;
  for (int64_t r = 0; r < n; ++r) {
    const int64_t v = order[r];
    const int64_t s = row_begin(G, v), e = row_begin(G, v + 1);
    if (t_indices)
      for (int64_t k = s; k < e; ++k) t_indices[at + (k - s)] = G.indices[k];
    at += e - s;
    t_indptr[r + 1] = at;
  }
  return at;
}

// Feature cache: row r is the feature row of the r-th ranked vertex.
void orc_fill_feat(const uint8_t* features, int64_t row_bytes, const int32_t* order, int64_t n, uint8_t* cache) {
  for (int64_t r = 0; r < n; ++r)
    std::memcpy(cache + r * row_bytes, features + static_cast<int64_t>(order[r]) * row_bytes, row_bytes);
}

// --- feature extraction (Sec. 5, feature extractor) -------------------------
void orc_gather(const uint8_t* features, int64_t row_bytes, const int32_t* ids, int64_t n, uint8_t* out) {
  for (int64_t i = 0; i < n; ++i)
    std::memcpy(out + i * row_bytes, features + static_cast<int64_t>(ids[i]) * row_bytes, row_bytes);
}

// Number of ids whose feature row is in the cache holding the first n_cached
// ranked vertices.
int64_t orc_count_hits(const int32_t* ids, int64_t n, const int32_t* order, int64_t n_cached, int64_t num_vertices) {
  std::vector<uint8_t> cached(num_vertices, 0);
  for (int64_t r = 0; r < n_cached; ++r) cached[order[r]] = 1;
  int64_t hits = 0;
  for (int64_t i = 0; i < n; ++i) hits += cached[ids[i]];
  return hits;
}

// --- Algorithm 1 (CSLP) for a clique of k_g GPUs -----------------------------
// hot is a k_g x V row-major matrix (one hotness row per GPU).  acc = column sums (step 1),
// order = vertices by descending acc, ties by ascending id (step 2), owner[v] = GPU with the
// largest local hotness of v (paper silent on ties: lowest GPU index), queues = the k_g
// per-GPU queues of step 3 laid end to end, queue g being [offsets[g], offsets[g+1]).
void orc_cslp(int32_t k_g, int64_t num_vertices, const uint32_t* hot, uint64_t* acc, int32_t* order, int32_t* owner,
              int32_t* queues, int64_t* offsets) {
  const int64_t V = num_vertices;
  for (int64_t v = 0; v < V; ++v) {
    uint64_t sum = 0;
    int32_t arg = 0;
    for (int32_t g = 0; g < k_g; ++g) {
      const uint32_t h = hot[static_cast<int64_t>(g) * V + v];
      sum += h;
      if (h > hot[static_cast<int64_t>(arg) * V + v]) arg = g;
    }
    acc[v] = sum;
    owner[v] = arg;
    order[v] = static_cast<int32_t>(v);
  }
  std::stable_sort(order, order + V, [acc](int32_t a, int32_t b) { return acc[a] > acc[b]; });
  std::vector<std::vector<int32_t>> G(k_g);
  for (int64_t r = 0; r < V; ++r) G[owner[order[r]]].push_back(order[r]);
  int64_t at = 0;
  for (int32_t g = 0; g < k_g; ++g) {
    offsets[g] = at;
    for (int32_t v : G[g]) queues[at++] = v;
  }
  offsets[k_g] = at;
}

// --- cache of a clique of k_g GPUs (Sec. 4.2.2: the queues of S2 drive the fill-up of S3) ---
// GPU g fills its own cache in the order of its own queue until its budget is used up.  The
// paper does not say where a queue is cut: as for one GPU (Eq. 3), the longest prefix whose
// rows (4 bytes per neighbour + 8 per row) fit.  Returns the number of queue entries taken.
int64_t orc_queue_prefix_topo(const orc_graph* g, const int32_t* queue, int64_t len, uint64_t topo_budget) {
  const Graph G = to_graph(g);
  uint64_t used = 0;
  int64_t n = 0;
  for (; n < len; ++n) {
    const int64_t v = queue[n];
    const uint64_t cost = static_cast<uint64_t>(row_begin(G, v + 1) - row_begin(G, v)) * 4u + 8u;
    if (used + cost > topo_budget) break;
    used += cost;
  }
  return n;
}

// Feature rows all cost the same (Eq. 6): the first floor(budget / row_bytes) entries of the queue.
int64_t orc_queue_prefix_feat(int64_t len, int64_t row_bytes, uint64_t feat_budget) {
  uint64_t used = 0;
  int64_t n = 0;
  for (; n < len; ++n) {
    if (used + static_cast<uint64_t>(row_bytes) > feat_budget) break;
    used += static_cast<uint64_t>(row_bytes);
  }
  return n;
}

// Feature extraction as GPU `member` of the clique sees it (Sec. 3.1, O1: a GPU reads its
// clique peers' caches over the fast links).  cached_by[v] = GPU whose cache holds v's row, or
// -1.  counts[0] = rows found in the member's own cache, counts[1] = rows in no cache of the
// clique (read from CPU memory), counts[2] = rows found in a peer's cache.
void orc_count_three_way(const int32_t* ids, int64_t n, const int32_t* cached_by, int32_t member, int64_t* counts) {
  counts[0] = counts[1] = counts[2] = 0;
  for (int64_t i = 0; i < n; ++i) {
    const int32_t where = cached_by[ids[i]];
    if (where < 0) ++counts[1];
    else if (where == member) ++counts[0];
    else ++counts[2];
  }
}

// --- cost model and alpha search (Sec. 4.3.2 Eq. 2-8, Sec. 4.3.3) -----------
struct orc_plan_point {
  uint64_t m_topo, m_feat;          // bytes given to the two caches at this alpha
  int64_t n_topo, n_feat;           // cached vertices (Eq. 3, Eq. 6)
  uint64_t uncached_topo_hot;       // sum of a_T over vertices outside the topology cache
  uint64_t uncached_feat_hot;       // U_F of Eq. 7
};

// Evaluates every candidate plan and returns the index of the best one.  n_tsum is
// N_TSUM (PCIe transactions the pre-sampling caused for topology); cls is the transfer
// granularity of Eq. 8.  N_T = n_tsum * uncached_topo_hot / total_topo_hot (Eq. 4-5),
// N_F = ceil(row_bytes / cls) * uncached_feat_hot (Eq. 8).
int32_t orc_search_cache_plan(const orc_graph* g, const uint32_t* topo_hot, const uint32_t* feat_hot,
                              const int32_t* order_t, const int32_t* order_f, int64_t row_bytes,
                              uint64_t total_budget, uint64_t n_tsum, uint32_t cls, int32_t n_alpha,
                              orc_plan_point* points) {
  const Graph G = to_graph(g);
  const int64_t V = G.num_vertices;
  uint64_t all_t = 0, all_f = 0;
  for (int64_t v = 0; v < V; ++v) { all_t += topo_hot[v]; all_f += feat_hot[v]; }
  const uint64_t per_row = (static_cast<uint64_t>(row_bytes) + cls - 1) / cls;
  int32_t best = 0;
  unsigned __int128 best_key = 0;
  for (int32_t i = 0; i < n_alpha; ++i) {
    orc_plan_point& p = points[i];
    p.m_topo = n_alpha > 1 ? static_cast<uint64_t>((static_cast<unsigned __int128>(total_budget) * i) / (n_alpha - 1))
                           : 0;
    p.m_feat = total_budget - p.m_topo;
    // Eq. 3: grow the topology cache along Q_T while it fits
    uint64_t used = 0, cached_t = 0;
    int64_t n = 0;
    for (; n < V; ++n) {
      const int64_t v = order_t[n];
      const uint64_t cost = static_cast<uint64_t>(row_begin(G, v + 1) - row_begin(G, v)) * 4u + 8u;
      if (used + cost > p.m_topo) break;
      used += cost;
      cached_t += topo_hot[v];
    }
    p.n_topo = n;
    p.uncached_topo_hot = all_t - cached_t;
    // Eq. 6: feature rows along Q_F while they fit
    uint64_t used_f = 0, cached_f = 0;
    int64_t m = 0;
    for (; m < V; ++m) {
      if (used_f + static_cast<uint64_t>(row_bytes) > p.m_feat) break;
      used_f += static_cast<uint64_t>(row_bytes);
      cached_f += feat_hot[order_f[m]];
    }
    p.n_feat = m;
    p.uncached_feat_hot = all_f - cached_f;
    // N_total * all_t = n_tsum * uncached_t + N_F * all_t   (all_t == 0: no topology traffic at all)
    const unsigned __int128 scale = all_t ? all_t : 1;
    const unsigned __int128 key = (all_t ? static_cast<unsigned __int128>(n_tsum) * p.uncached_topo_hot : 0) +
                                  static_cast<unsigned __int128>(per_row) * p.uncached_feat_hot * scale;
    if (i == 0 || key < best_key) { best = i; best_key = key; }
  }
  return best;
}

} // extern "C"
