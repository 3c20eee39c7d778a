"""MI355X-native mini-batch data preparation for cache-based GNN training:
hotness pre-sampling, HBM topology / feature caches, k-hop neighbour sampling
and feature extraction (hand-written HIP behind a C ABI, see include/legion_prep.h)."""
from .binding import (BlockBuffers, CachePlan, Context, LegionPrepError, PlanPoint, Profile, SampleBuffers, concurrent_streams, cslp, load_library, shuffle_tablet, pinned_copy,
                      pinned_empty, worst_case_sizes)

__all__ = ["BlockBuffers", "CachePlan", "Context", "LegionPrepError", "PlanPoint", "Profile", "SampleBuffers", "concurrent_streams", "cslp", "load_library", "shuffle_tablet", "pinned_copy",
           "pinned_empty", "worst_case_sizes"]
