// Host-side sanitizer driver for the C ABI (no GPU needed): every entry point is called with null handles and
// malformed arguments, which must come back as a negative status from the host-side checks, with the
// library's own host code (api.hip) built under -fsanitize=address,undefined.
#include <cstdio>
#include <cstring>

#include "legion_prep.h"

#define EXPECT(cond)                                              \
  do {                                                            \
    if (!(cond)) {                                                \
      std::printf("FAILED: %s (line %d)\n", #cond, __LINE__);     \
      return 1;                                                   \
    }                                                             \
  } while (0)

int main() {
  for (int st = -9; st <= 1; ++st) EXPECT(std::strlen(lgp_strerror(st)) > 0);
  EXPECT(std::strcmp(lgp_last_error(nullptr), "") == 0);
  lgp_ctx* ctx = nullptr;
  lgp_graph g;
  std::memset(&g, 0, sizeof(g));
  EXPECT(lgp_create(nullptr, 0, &ctx) == LGP_EINVAL);
  EXPECT(lgp_create(&g, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_create(&g, 0, &ctx) == LGP_EINVAL && ctx == nullptr);            // V = 0
  int32_t indptr[3] = {0, 1, 2}, indices[2] = {1, 0};
  g.num_vertices = 2; g.num_edges = 2; g.indptr = indptr; g.indices = indices; g.indptr_bytes = 3;
  EXPECT(lgp_create(&g, 0, &ctx) == LGP_EINVAL);                              // offset width
  g.indptr_bytes = 4; g.num_vertices = int64_t(1) << 31;
  EXPECT(lgp_create(&g, 0, &ctx) == LGP_EUNSUPPORTED);
  g.num_vertices = 2; g.features = indices; g.feat_dim = 0; g.elem_bytes = 4;
  EXPECT(lgp_create(&g, 0, &ctx) == LGP_EINVAL);                              // feature width
  g.features = nullptr;
  EXPECT(lgp_create(&g, -1, &ctx) == LGP_EINVAL);                             // no such device
  EXPECT(lgp_destroy(nullptr) == LGP_OK);
  EXPECT(lgp_host_alloc(16, nullptr) == LGP_EINVAL);
  EXPECT(lgp_host_free(nullptr) == LGP_OK);
  const int32_t fan[2] = {10, 5};
  lgp_sample_out so;
  std::memset(&so, 0, sizeof(so));
  lgp_blocks_out bo;
  std::memset(&bo, 0, sizeof(bo));
  lgp_cache_plan plan;
  lgp_profile prof;
  int64_t a = 0, b = 0;
  size_t fixed = 0, scratch = 0;
  int32_t best = 0;
  EXPECT(lgp_build_hotness(nullptr, indices, 2, 1, fan, 2, 1, -1, nullptr) == LGP_EINVAL);
  EXPECT(lgp_get_presample_stats(nullptr, &a, &b) == LGP_EINVAL);
  EXPECT(lgp_get_hotness(nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_set_hotness(nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_plan_cache(nullptr, 0, 0, &plan, nullptr) == LGP_EINVAL);
  EXPECT(lgp_build_cache(nullptr, 0, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_get_cache_plan(nullptr, &plan) == LGP_EINVAL);
  EXPECT(lgp_search_cache_plan(nullptr, 1, 1, 64, 11, nullptr, &best, nullptr) == LGP_EINVAL);
  EXPECT(lgp_get_cache(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_get_cache_part(nullptr, 0, 0, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_build_clique_cache(nullptr, 2, nullptr, nullptr, 0, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_get_clique_plan(nullptr, 0, &plan) == LGP_EINVAL);
  EXPECT(lgp_sample_khop(nullptr, indices, 2, fan, 2, 1, &so, nullptr) == LGP_EINVAL);
  EXPECT(lgp_sample_extract(nullptr, indices, 2, fan, 2, 1, &so, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_build_blocks(nullptr, indices, 2, fan, 2, &so, &bo, nullptr) == LGP_EINVAL);
  EXPECT(lgp_gather_features(nullptr, indices, 2, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_gather_features_static(nullptr, indices, 2, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_gather_features_clique(nullptr, 0, indices, 2, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_reserve(nullptr, 16, fan, 2) == LGP_EINVAL);
  EXPECT(lgp_workspace_bytes(nullptr, 16, fan, 2, &fixed, &scratch) == LGP_EINVAL);
  EXPECT(lgp_check(nullptr, nullptr) == LGP_EINVAL);
  EXPECT(lgp_set_overlap(nullptr, 1) == LGP_EINVAL);
  EXPECT(lgp_set_profiling(nullptr, 1) == LGP_EINVAL);
  EXPECT(lgp_get_profile(nullptr, &prof) == LGP_EINVAL);
  // calls that need no context check their arguments before they touch a device
  EXPECT(lgp_shuffle_tablet(0, nullptr, nullptr, 5, 1, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_shuffle_tablet(0, indices, indices, -1, 1, 0, nullptr) == LGP_EINVAL);
  EXPECT(lgp_cslp(0, 0, 2, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == LGP_EINVAL);
  std::puts("abi sanitizer run clean");
  return 0;
}
