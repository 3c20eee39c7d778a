"""One epoch of mini-batch data preparation, end to end, on a synthetic workload.

    python -m paper_2305_16588_amd.example_epoch [--workload mid] [--cache-gb 0.4]

Shows the call sequence a training loop would use: pre-sampling, automatic split of one
cache budget between topology and features, cache build, then per batch: epoch shuffle,
k-hop sampling, graph construction and feature extraction on three streams -- the graph
constructor beside the feature extractor of the same batch, the sampling of the next batch
beside both -- with the miss gather overlapping the hit gather.  The feature matrix and
the per-hop blocks of every batch are what a GNN layer stack would consume.
"""
from __future__ import annotations

import argparse
import time

import numpy as np
import torch

import datagen
import paper_2305_16588_amd as lgp


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="mid")
    ap.add_argument("--cache-gb", type=float, default=0.4, help="total HBM budget for both caches")
    ap.add_argument("--epochs", type=int, default=1)
    args = ap.parse_args()
    spec = datagen.WORKLOADS[args.workload]

    indptr = lgp.pinned_empty(spec.num_vertices + 1, np.int64 if spec.index64 else np.int32)
    _, indices = datagen.make_graph(spec, device="cuda", indptr_out=indptr,
                                    indices_alloc=lambda n: lgp.pinned_empty(n, np.int32))
    feats = lgp.pinned_empty((spec.num_vertices, spec.feat_dim),
                             np.float32 if spec.feat_dtype == "float32" else np.float16)
    datagen.make_features(spec, device="cuda", out=feats)
    tablet = torch.from_numpy(datagen.make_tablet(spec, device="cuda")).cuda()
    ctx = lgp.Context(indptr, indices, feats)

    # cache construction: pre-sampling -> cost model picks alpha -> fill
    ctx.build_hotness(tablet, spec.batch, spec.fanouts, spec.base_seed)
    _, n_row_reads = ctx.get_presample_stats()          # N_TSUM: one 128-byte line per expansion on this GPU
    budget = int(args.cache_gb * 1e9)
    best, pts = ctx.search_cache_plan(budget, n_tsum=n_row_reads, cls_bytes=128)
    plan = ctx.build_cache(int(pts["m_topo"][best]), int(pts["m_feat"][best]))
    print(f"cache plan: alpha = {best / 100:.2f} -> {plan.n_topo} topology rows ({plan.topo_bytes / 1e6:.0f} MB), "
          f"{plan.n_feat} feature rows ({plan.feat_bytes / 1e6:.0f} MB)")

    ctx.set_overlap(0 < plan.n_feat < spec.num_vertices)        # both gathers have work: run them side by side
    n_batches = tablet.numel() // spec.batch
    # streams that share a hardware queue would run one after the other, so pick three that do not
    (s_sample, s_gather, s_blocks), _ = lgp.concurrent_streams(3)
    bufs = [lgp.SampleBuffers(spec.num_vertices, spec.batch, spec.fanouts, last_frontier=True) for _ in range(2)]
    blks = [lgp.BlockBuffers(b) for b in bufs]
    rows = [torch.empty((bufs[0].gather_cap, spec.feat_dim), dtype=ctx.feat_torch_dtype, device="cuda") for _ in range(2)]
    stats = torch.zeros((n_batches, 2), dtype=torch.int32, device="cuda")
    sampled = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    built = [torch.cuda.Event() for _ in range(2)]
    for epoch in range(args.epochs):
        order = lgp.shuffle_tablet(tablet, seed=spec.split_seed, epoch=epoch)       # batch generator
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for b in range(n_batches):
            k = b % 2
            seeds = order[b * spec.batch:(b + 1) * spec.batch]
            if b >= 2:
                s_sample.wait_event(consumed[k])
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + epoch * n_batches + b, out=bufs[k], stream=s_sample)
            sampled[k].record(s_sample)
            s_blocks.wait_event(sampled[k])
            ctx.build_blocks(seeds, spec.fanouts, bufs[k], out=blks[k], stream=s_blocks)
            built[k].record(s_blocks)
            s_gather.wait_event(sampled[k])
            ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=rows[k], stats=stats[b], stream=s_gather)
            s_gather.wait_event(built[k])
            # ... a training step would consume rows[k] and blks[k] here, on s_gather ...
            consumed[k].record(s_gather)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.check()
        st = stats.cpu().numpy().astype(np.int64)
        print(f"epoch {epoch}: {n_batches} batches of {spec.batch} seeds in {dt * 1e3:.1f} ms "
              f"({n_batches * spec.batch / dt / 1e6:.2f} M seeds/s), {st.sum() / n_batches:.0f} rows per batch, "
              f"feature-cache hit rate {st[:, 0].sum() / st.sum():.3f}")


if __name__ == "__main__":
    main()
