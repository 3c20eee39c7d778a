// Sanitizer driver for the CPU oracle (test infrastructure).  It includes the oracle's source, so the whole
// thing is one translation unit built with -fsanitize=address,undefined, and calls every exported function on a
// small random graph (int32 and int64 offsets, empty rows, rows longer than the fan-out, empty inputs).  It
// checks nothing about values -- the pins do that -- only that the run is clean: exit code 0 and no report.
#include "legion_oracle.cpp"

#include <cstdio>
#include <random>

int main() {
  std::mt19937_64 rng(7);
  const int64_t V = 500;
  std::vector<int64_t> indptr64(V + 1, 0);
  std::vector<int32_t> indptr32(V + 1, 0), indices;
  for (int64_t v = 0; v < V; ++v) {
    int d = (v % 17 == 0) ? 0 : int(rng() % 40);
    if (v == 3) d = 200;
    std::vector<int32_t> row;
    for (int k = 0; k < d; ++k) row.push_back(int32_t(rng() % V));
    std::sort(row.begin(), row.end());
    row.erase(std::unique(row.begin(), row.end()), row.end());
    indices.insert(indices.end(), row.begin(), row.end());
    indptr64[v + 1] = int64_t(indices.size());
    indptr32[v + 1] = int32_t(indices.size());
  }
  const int64_t row_bytes = 24;
  std::vector<uint8_t> feats(V * row_bytes);
  for (auto& x : feats) x = uint8_t(rng());
  std::vector<int32_t> tablet(V);
  for (int64_t v = 0; v < V; ++v) tablet[v] = int32_t(v);
  std::vector<int32_t> shuffled(V);
  orc_shuffle_tablet(tablet.data(), shuffled.data(), V, 99, 3);
  orc_shuffle_tablet(tablet.data(), shuffled.data(), 0, 99, 3);

  uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, outw[4];
  orc_philox4x32_10(ctr, key, outw);
  (void)orc_draw64(~0ull, V - 1, 7, 63);

  for (int wide = 0; wide < 2; ++wide) {
    orc_graph g{V, wide ? static_cast<const void*>(indptr64.data()) : static_cast<const void*>(indptr32.data()),
                wide ? 8 : 4, indices.data()};
    std::vector<int32_t> row(64);
    for (int64_t v : {int64_t(0), int64_t(3), V - 1}) (void)orc_sample_row(&g, v, 1, 64, 11, row.data());
    (void)orc_sample_row(&g, 3, 0, 5, 11, row.data());
    const int32_t fan[3] = {7, 3, 2};
    for (int64_t n_seeds : {int64_t(0), int64_t(1), int64_t(130)}) {
      void* h = orc_sample_khop(&g, shuffled.data(), n_seeds, fan, 3, 42);
      for (int hop = 0; hop <= 3; ++hop) {
        const int64_t n = orc_batch_frontier_size(h, hop);
        (void)orc_batch_frontier(h, hop);
        std::vector<int32_t> fr(n + 1);
        orc_feature_rows(h, hop, fr.data());
        if (hop < 3) {
          (void)orc_batch_nbr(h, hop);
          const int32_t* cnt = orc_batch_cnt(h, hop);
          int64_t edges = 0;
          for (int64_t i = 0; i < n; ++i) edges += cnt[i];
          std::vector<int64_t> bi(n + 1);
          std::vector<int32_t> bs(edges + 1);
          orc_block_of_hop(h, hop, fan[hop], bi.data(), bs.data());
        }
      }
      const int64_t ng = orc_batch_gather_size(h);
      const int32_t* gids = orc_batch_gather_ids(h);
      std::vector<int64_t> seg(5);
      const int64_t total = orc_hop_order(h, V, nullptr, seg.data());
      std::vector<int32_t> order(total + 1);
      (void)orc_hop_order(h, V, order.data(), seg.data());
      std::vector<uint8_t> gathered(ng * row_bytes + 1);
      orc_gather(feats.data(), row_bytes, gids, ng, gathered.data());
      orc_batch_free(h);
    }
    std::vector<uint32_t> topo_hot(V), feat_hot(V);
    (void)orc_build_hotness(&g, shuffled.data(), V, 64, fan, 3, 1000, -1, topo_hot.data(), feat_hot.data());
    (void)orc_build_hotness(&g, shuffled.data(), V, 64, fan, 3, 1000, 2, topo_hot.data(), feat_hot.data());
    std::vector<int32_t> qt(V), qf(V);
    orc_rank_by_hotness(topo_hot.data(), V, qt.data());
    orc_rank_by_hotness(feat_hot.data(), V, qf.data());
    for (uint64_t budget : {uint64_t(0), uint64_t(5000), ~uint64_t(0) >> 1}) {
      const int64_t n_t = orc_plan_topo(&g, qt.data(), budget);
      const int64_t n_f = orc_plan_feat(V, row_bytes, budget);
      std::vector<int64_t> ti(n_t + 1);
      const int64_t edges = orc_fill_topo(&g, qt.data(), n_t, ti.data(), nullptr);
      std::vector<int32_t> tx(edges + 1);
      (void)orc_fill_topo(&g, qt.data(), n_t, ti.data(), tx.data());
      std::vector<uint8_t> fc(n_f * row_bytes + 1);
      orc_fill_feat(feats.data(), row_bytes, qf.data(), n_f, fc.data());
      (void)orc_count_hits(shuffled.data(), 200, qf.data(), n_f, V);
      (void)orc_queue_prefix_topo(&g, qt.data(), V / 2, budget);
      (void)orc_queue_prefix_feat(V / 2, row_bytes, budget);
    }
    std::vector<orc_plan_point> pts(11);
    (void)orc_search_cache_plan(&g, topo_hot.data(), feat_hot.data(), qt.data(), qf.data(), row_bytes, 20000, 12345, 64,
                                11, pts.data());
    const int32_t k_g = 3;
    std::vector<uint32_t> hot(k_g * V);
    for (auto& x : hot) x = uint32_t(rng() % 5);
    std::vector<uint64_t> acc(V);
    std::vector<int32_t> order(V), owner(V), queues(V);
    std::vector<int64_t> offsets(k_g + 1);
    orc_cslp(k_g, V, hot.data(), acc.data(), order.data(), owner.data(), queues.data(), offsets.data());
    int64_t counts[3];
    orc_count_three_way(shuffled.data(), 100, owner.data(), 1, counts);
  }
  std::puts("oracle sanitizer run clean");
  return 0;
}
