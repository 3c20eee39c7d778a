#!/usr/bin/env python3
"""Benchmark of the mini-batch data-preparation hot path on one MI355X.

One step = sample_khop + gather_features for one mini-batch of the workload's
training tablet (all per-batch stages; the caches are built beforehand from a
pre-sampling epoch, whose time is reported separately).  Inputs are seeded and
synthetic (see datagen) and are resident -- graph and feature table in pinned CPU
memory, caches in HBM -- before the timed region starts.

Prints ONE JSON line.  `roofline` covers the cache-hit row gather (HBM -> HBM),
`roofline_pcie` the miss row gather (CPU memory -> HBM); both use HIP events
recorded by the library on the streams the kernels run on.  `cpu_baseline` is
the single-threaded CPU oracle timed on a bounded sample of the same batches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
PCIE_PEAK_GBS = 63.0           # PCIe Gen5 x16, one direction: 32 GT/s * 16 * 128/130 / 8
# HBM bytes per hit row measured with rocprofv3 --pmc (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors a plain
# 1 GiB copy gives; see profiles/bench_{mid,large,share,wide}_workload.md), keyed by row width in bytes.
MEASURED_HBM_BYTES_PER_HIT_ROW = {256: 516.3, 400: 931.7, 512: 1028.1, 2048: 4105.0}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mid", help="tiny | mid | wide | large | share (optionally name@scale)")
    ap.add_argument("--feat-frac", type=float, default=None, help="override the feature-cache ratio")
    ap.add_argument("--topo-frac", type=float, default=None, help="override the topology-cache ratio")
    ap.add_argument("--cache-bytes", type=int, default=0,
                    help="one total cache budget B instead of the two ratios; split by --alpha, or by the cost model")
    ap.add_argument("--alpha", type=float, default=None, help="topology share of --cache-bytes (default: cost-model search)")
    ap.add_argument("--clique", type=int, default=0, metavar="K",
                    help="also time the step as member 0 of a simulated clique of K GPUs (each member with the "
                         "workload's cache budgets; secondary figure, replaces the cache at the end of the run)")
    ap.add_argument("--overlap", action="store_true", help="miss gather on a second stream beside the hit gather")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="skip the secondary measurement (sampling of batch i+1 beside feature extraction of batch i)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--features-on-device", action="store_true",
                    help="keep the source feature table in HBM (for tables beyond the box's 64 GiB pinned-memory limit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=0, help="oracle batches to time (0 = pick for ~15 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the work; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from dataclasses import replace

    import datagen
    import paper_2305_16588_amd as lgp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3

    name, _, scale = args.workload.partition("@")
    spec = datagen.WORKLOADS[name]
    if scale:
        spec = datagen.scaled(spec, float(scale))
    if args.feat_frac is not None:
        spec = replace(spec, feat_frac=args.feat_frac)
    if args.topo_frac is not None:
        spec = replace(spec, topo_frac=args.topo_frac)

    t0 = time.time()
    indptr = lgp.pinned_empty(spec.num_vertices + 1, np.int64 if spec.index64 else np.int32)
    _, indices = datagen.make_graph(spec, device="cuda", indptr_out=indptr,
                                    indices_alloc=lambda n: lgp.pinned_empty(n, np.int32))
    npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
    if args.features_on_device:
        feats = np.empty((spec.num_vertices, spec.feat_dim), npdt)
    else:
        feats = lgp.pinned_empty((spec.num_vertices, spec.feat_dim), npdt)
    datagen.make_features(spec, device="cuda", out=feats)
    feats_src = feats
    if args.features_on_device:
        feats_src = torch.empty(feats.shape, device="cuda",
                                dtype=torch.float32 if spec.feat_dtype == "float32" else torch.float16)
        for lo in range(0, spec.num_vertices, 1 << 22):
            feats_src[lo:lo + (1 << 22)].copy_(torch.from_numpy(feats[lo:lo + (1 << 22)]))
    tablet = datagen.make_tablet(spec)
    t_gen = time.time() - t0
    V, E, D = spec.num_vertices, int(indices.size), spec.feat_dim
    row_bytes = D * feats.dtype.itemsize

    ctx = lgp.Context(indptr, indices, feats_src)
    ctx.set_overlap(args.overlap)
    tablet_dev = torch.from_numpy(tablet).cuda()
    torch.cuda.synchronize()
    t0 = time.time()
    ctx.build_hotness(tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    torch.cuda.synchronize()
    t_hot = time.time() - t0
    topo_b, feat_b = datagen.budgets(spec, E)
    auto_plan = None
    if args.cache_bytes:
        topo_hot, _ = ctx.get_hotness()
        # N_TSUM: pre-sampling reads one 128-byte line of column ids per vertex expansion; CLS = that line size
        _, n_tsum = ctx.get_presample_stats()
        best, pts = ctx.search_cache_plan(args.cache_bytes, n_tsum, cls_bytes=128)
        pick = best if args.alpha is None else int(round(args.alpha * 100))
        topo_b, feat_b = int(pts["m_topo"][pick]), int(pts["m_feat"][pick])
        per_row = -(-row_bytes // 128)
        all_t = max(int(topo_hot.sum()), 1)
        auto_plan = {"B": args.cache_bytes, "alpha": pick / 100, "alpha_by_cost_model": best / 100,
                     "predicted_N_total": round(n_tsum * int(pts["uncached_topo_hot"][pick]) / all_t
                                                + per_row * int(pts["uncached_feat_hot"][pick]))}
    t0 = time.time()
    plan = ctx.build_cache(topo_b, feat_b)
    t_cache = time.time() - t0

    n_batches = (tablet.size + spec.batch - 1) // spec.batch
    full_batches = max(1, tablet.size // spec.batch)     # timed steps use full batches only
    buf = lgp.SampleBuffers(V, spec.batch, spec.fanouts)
    rows = torch.empty((buf.gather_cap, D), dtype=ctx.feat_torch_dtype, device="cuda")
    stats = torch.zeros((args.steps + args.warmup, 2), dtype=torch.int32, device="cuda")

    def step(i: int):
        b = i % full_batches
        seeds = tablet_dev[b * spec.batch:(b + 1) * spec.batch]
        ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=buf)
        ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats[i])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ctx.check()
    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    # Timed region: K steps, HIP events only around the two row gathers (hits: the kernel of `roofline`; misses:
    # `roofline_pcie`).  An event pair costs a few microseconds of stream time, so the full breakdown of `per_step`
    # comes from an untimed second pass over the same K steps with events around every kernel group.
    ctx.set_profiling(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof_g = ctx.get_profile()
    ctx.check()
    ctx.set_profiling(1)
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    ctx.set_profiling(0)
    prof = ctx.get_profile()
    ctx.check()

    elapsed = t1 - t0
    ms_per_step = elapsed * 1e3 / args.steps
    seeds_per_s = args.steps * spec.batch / elapsed
    st = stats[args.warmup:].cpu().numpy().astype(np.int64)
    hit_rows, miss_rows = int(st[:, 0].sum()), int(st[:, 1].sum())
    gathered = hit_rows + miss_rows

    # algorithmic bytes of one hit-gather launch: each hit row is read once and written once,
    # plus its (row, slot) list entry
    hit_bytes_per_row = 2 * row_bytes + 8
    # kernel names as rocprofv3 lists them (16-byte chunks; lane groups of the next power of two >= chunks per row)
    cpr = row_bytes // 16
    grp = next(g for g in (4, 8, 16, 32, 64) if g >= min(cpr, 64))
    hit_kernel = (f"gather_rows_group_kernel<u32x4, {grp}, 1, true>" if row_bytes % 128 and cpr <= 32
                  else f"gather_rows_flat_kernel<u32x4, 4, {'true' if row_bytes % 128 == 0 else 'false'}>")
    miss_kernel = f"gather_rows_group_kernel<u32x4, {grp}, 4, false>"
    roofline = None
    if prof_g.n_hit and hit_rows:
        ach = hit_rows * hit_bytes_per_row / (prof_g.ms_hit * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": hit_kernel + " (cache hits, HBM->HBM)", "achieved": round(ach, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                    # measured on the launch shape of the profiled workload: the 400-byte figure is for a
                    # hit list, not for the direct launch of a cache that holds every vertex
                    "traffic": (round(MEASURED_HBM_BYTES_PER_HIT_ROW[row_bytes] * hit_rows / prof_g.n_hit)
                                if row_bytes in MEASURED_HBM_BYTES_PER_HIT_ROW
                                and not (row_bytes == 400 and plan.n_feat == V) else None),
                    "avg_launch_ms": round(prof_g.ms_hit / prof_g.n_hit, 4),
                    "rows_per_launch": round(hit_rows / prof_g.n_hit, 1), "bytes_per_row": hit_bytes_per_row}
    roofline_pcie = None
    if prof_g.n_miss and miss_rows:
        ach = miss_rows * row_bytes / (prof_g.ms_miss * 1e-3) / 1e9
        roofline_pcie = {"bound": "pcie", "kernel": miss_kernel + " (cache misses, CPU memory->HBM)",
                         "achieved": round(ach, 2), "peak": PCIE_PEAK_GBS, "unit": "GB/s",
                         "frac": round(ach / PCIE_PEAK_GBS, 4), "avg_launch_ms": round(prof_g.ms_miss / prof_g.n_miss, 4),
                         "rows_per_launch": round(miss_rows / prof_g.n_miss, 1), "bytes_per_row": row_bytes}

    # Secondary figure: the same K steps with the library's hit / miss overlap switched on (the miss gather on a
    # stream of its own beside a narrower hit gather).  Faster whenever both gathers have work, but the hit gather's
    # own duration then says nothing about the kernel, so the headline and the rooflines stay with overlap off.
    overlapped = None
    if not args.no_pipeline and not args.overlap and 0 < plan.n_feat < V:
        ctx.set_overlap(True)
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        o0 = time.perf_counter()
        for i in range(args.warmup, args.warmup + args.steps):
            step(i)
        torch.cuda.synchronize()
        o1 = time.perf_counter()
        ctx.set_overlap(False)
        ctx.check()
        overlapped = {"value": round(args.steps * spec.batch / (o1 - o0), 1), "unit": "seeds/s",
                      "ms_per_step": round((o1 - o0) * 1e3 / args.steps, 4),
                      "how": "lgp_set_overlap(1): miss gather on its own stream beside a narrower hit gather"}

    # Secondary figure: the same K steps with sampling of batch i+1 running on a second stream
    # beside the feature extraction of batch i (double-buffered outputs).  Not the headline.
    pipelined = None
    # the secondary pipelines below use the hit / miss overlap too where it paid above
    both_gathers = overlapped is not None and overlapped["ms_per_step"] < ms_per_step
    if not args.no_pipeline:
        ctx.set_overlap(args.overlap or both_gathers)
        sA, sB = torch.cuda.Stream(), torch.cuda.Stream()
        bufs = [buf, lgp.SampleBuffers(V, spec.batch, spec.fanouts)]
        outs = [rows, torch.empty_like(rows)]
        ev_sampled = [torch.cuda.Event(), torch.cuda.Event()]
        ev_gathered = [torch.cuda.Event(), torch.cuda.Event()]
        pstats = torch.zeros((args.steps + args.warmup, 2), dtype=torch.int32, device="cuda")

        def pstep(i: int):
            k = i % 2
            b = i % full_batches
            seeds = tablet_dev[b * spec.batch:(b + 1) * spec.batch]
            if i >= 2:
                sA.wait_event(ev_gathered[k])              # buffer k is free again
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=bufs[k], stream=sA)
            ev_sampled[k].record(sA)
            sB.wait_event(ev_sampled[k])
            ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=outs[k], stats=pstats[i], stream=sB)
            ev_gathered[k].record(sB)

        torch.cuda.synchronize()
        for i in range(args.warmup):
            pstep(i)
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for i in range(args.warmup, args.warmup + args.steps):
            pstep(i)
        torch.cuda.synchronize()
        p1 = time.perf_counter()
        ctx.check()
        assert torch.equal(pstats[args.warmup:].cpu(), stats[args.warmup:].cpu()), "pipelined run diverged"
        pipelined = {"value": round(args.steps * spec.batch / (p1 - p0), 1), "unit": "seeds/s",
                     "ms_per_step": round((p1 - p0) * 1e3 / args.steps, 4),
                     "how": "sample_khop of batch i+1 on a second stream beside gather_features of batch i"
                            + (", hit / miss overlap on" if both_gathers else "")}
        del bufs, outs
        ctx.set_overlap(args.overlap)

    # Secondary figure: the whole sampling server of Sec. 5 -- neighbour sampler, graph constructor and feature
    # extractor per batch -- serial on one stream, and as the two pipelines the section describes: within a batch
    # the graph constructor beside the feature extractor, across batches the sampling of batch i+1 beside both.
    server = None
    if not args.no_pipeline:
        sA, sB, sC = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        bufs = [lgp.SampleBuffers(V, spec.batch, spec.fanouts, last_frontier=True) for _ in range(2)]
        blks = [lgp.BlockBuffers(b) for b in bufs]
        outs = [rows, torch.empty_like(rows)]
        ev_s = [torch.cuda.Event(), torch.cuda.Event()]
        ev_g = [torch.cuda.Event(), torch.cuda.Event()]
        ev_b = [torch.cuda.Event(), torch.cuda.Event()]
        sstats = torch.zeros((args.steps + args.warmup, 2), dtype=torch.int32, device="cuda")

        def serial_step(i: int):
            b = i % full_batches
            seeds = tablet_dev[b * spec.batch:(b + 1) * spec.batch]
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=bufs[0])
            ctx.build_blocks(seeds, spec.fanouts, bufs[0], out=blks[0])
            ctx.gather_features(bufs[0].gather_ids, n_dev=bufs[0].n_gather, out=outs[0], stats=sstats[i])

        def piped_step(i: int):
            k = i % 2
            b = i % full_batches
            seeds = tablet_dev[b * spec.batch:(b + 1) * spec.batch]
            if i >= 2:
                sA.wait_event(ev_g[k])                      # buffer k is free again
                sA.wait_event(ev_b[k])
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=bufs[k], stream=sA)
            ev_s[k].record(sA)
            sB.wait_event(ev_s[k])
            sC.wait_event(ev_s[k])
            ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=outs[k], stats=sstats[i], stream=sB)
            ev_g[k].record(sB)
            ctx.build_blocks(seeds, spec.fanouts, bufs[k], out=blks[k], stream=sC)
            ev_b[k].record(sC)

        times = []
        for fn in (serial_step, piped_step):
            ctx.set_overlap(args.overlap or (both_gathers and fn is piped_step))
            torch.cuda.synchronize()
            for i in range(args.warmup):
                fn(i)
            torch.cuda.synchronize()
            q0 = time.perf_counter()
            for i in range(args.warmup, args.warmup + args.steps):
                fn(i)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - q0)
            ctx.check()
            assert torch.equal(sstats[args.warmup:].cpu(), stats[args.warmup:].cpu()), "sampling-server run diverged"
        server = {"serial": {"value": round(args.steps * spec.batch / times[0], 1), "unit": "seeds/s",
                             "ms_per_step": round(times[0] * 1e3 / args.steps, 4)},
                  "pipelined": {"value": round(args.steps * spec.batch / times[1], 1), "unit": "seeds/s",
                                "ms_per_step": round(times[1] * 1e3 / args.steps, 4)},
                  "how": "step = sample_khop + build_blocks + gather_features; pipelined = three streams: build_blocks "
                         "beside gather_features of the same batch, sample_khop of the next batch beside both"
                         + (", hit / miss overlap on" if both_gathers else "")}
        del bufs, blks, outs
        ctx.set_overlap(args.overlap)

    # Secondary figure: the same step captured once into a HIP graph (sampling, dedup, partition, gathers: about a
    # dozen launches) and replayed; seeds change per replay, the rng seed is the captured one.
    graph_replay = None
    if not args.no_pipeline:
        seeds_buf = tablet_dev[:spec.batch].clone()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            ctx.sample_khop(seeds_buf, spec.fanouts, spec.base_seed, out=buf)
            ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats[0])
        for i in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(args.warmup, args.warmup + args.steps):
            b = i % full_batches
            seeds_buf.copy_(tablet_dev[b * spec.batch:(b + 1) * spec.batch], non_blocking=True)
            g.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        ctx.check()
        graph_replay = {"value": round(args.steps * spec.batch / (g1 - g0), 1), "unit": "seeds/s",
                        "ms_per_step": round((g1 - g0) * 1e3 / args.steps, 4),
                        "how": "one captured HIP graph per step, replayed; seeds copied in before each replay"}
        del g

    # Graph constructor (a widening row, not part of the headline step): time it on the same batches.
    blocks_ms = None
    if not args.no_pipeline:
        bbuf = lgp.SampleBuffers(V, spec.batch, spec.fanouts, last_frontier=True)
        blk = lgp.BlockBuffers(bbuf)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        total = 0.0
        reps = min(args.steps, 20)
        for i in range(args.warmup, args.warmup + reps + 2):
            b = i % full_batches
            seeds = tablet_dev[b * spec.batch:(b + 1) * spec.batch]
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=bbuf)
            e0.record()
            ctx.build_blocks(seeds, spec.fanouts, bbuf, out=blk)
            e1.record()
            torch.cuda.synchronize()
            if i >= args.warmup + 2:
                total += e0.elapsed_time(e1)
        blocks_ms = round(total / reps, 4)
        ctx.check()
        del bbuf, blk

    # Secondary figure: the same step as member 0 of a simulated clique of K GPUs.  Every member pre-samples its own
    # hash share of the tablet and contributes a cache of the workload's budgets; rows a peer caches are read from
    # the peer's region of this device's HBM, so the time says nothing about a real inter-GPU link -- the split
    # {own cache, peer's cache, CPU memory} is the result.
    clique = None
    if args.clique > 0:
        K = args.clique
        HT = torch.empty((K, V), dtype=torch.int32, device="cuda")
        HF = torch.empty((K, V), dtype=torch.int32, device="cuda")
        tabs = []
        sum_t, sum_f, n_tsum_c = np.zeros(V, np.uint64), np.zeros(V, np.uint64), 0
        for g in range(K):
            tabs.append(tablet_dev[g::K].contiguous())
            ctx.build_hotness(tabs[g], spec.batch, spec.fanouts, spec.base_seed + 1000 * g)
            th, fh = ctx.get_hotness()
            HT[g].copy_(torch.from_numpy(th.view(np.int32)))
            HF[g].copy_(torch.from_numpy(fh.view(np.int32)))
            sum_t += th
            sum_f += fh
            n_tsum_c += ctx.get_presample_stats()[1]
        ctopo_b, cfeat_b, clique_plan = topo_b, feat_b, None
        if args.cache_bytes:
            # Sec. 4.3 at clique granularity: the cost model runs on the clique's summed hotness (A_T, A_F) with the
            # clique's budget K * B and the clique's N_TSUM; every member then gets 1/K of each share.
            ctx.build_cache(0, 0)                                   # drop the cache: the search re-ranks the vertices
            ctx.set_hotness(np.minimum(sum_t, 2**32 - 1).astype(np.uint32), np.minimum(sum_f, 2**32 - 1).astype(np.uint32))
            cbest, cpts = ctx.search_cache_plan(K * args.cache_bytes, n_tsum_c, cls_bytes=128)
            ctopo_b, cfeat_b = int(cpts["m_topo"][cbest]) // K, int(cpts["m_feat"][cbest]) // K
            clique_plan = {"B_per_member": args.cache_bytes, "alpha_by_cost_model": cbest / 100}
        plans = ctx.build_clique_cache(HT, HF, ctopo_b, cfeat_b)
        del HT, HF
        my_batches = max(1, tabs[0].numel() // spec.batch)
        cstats = torch.zeros((args.steps + args.warmup, 3), dtype=torch.int32, device="cuda")

        def cstep(i: int):
            b = i % my_batches
            seeds = tabs[0][b * spec.batch:(b + 1) * spec.batch]
            ctx.sample_khop(seeds, spec.fanouts, spec.base_seed + i, out=buf)
            ctx.gather_features_clique(0, buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=cstats[i])

        for i in range(args.warmup):
            cstep(i)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for i in range(args.warmup, args.warmup + args.steps):
            cstep(i)
        torch.cuda.synchronize()
        c1 = time.perf_counter()
        ctx.check()
        n_seeds = min(spec.batch, tabs[0].numel())
        tot = cstats[args.warmup:].sum(dim=0).tolist()
        clique = {"k_g": K, "member": 0, "value": round(args.steps * n_seeds / (c1 - c0), 1), "unit": "seeds/s",
                  "ms_per_step": round((c1 - c0) * 1e3 / args.steps, 4),
                  "cache_plan": clique_plan,
                  "cached_topo_rows": [p.n_topo for p in plans], "cached_feat_rows": [p.n_feat for p in plans],
                  "rows_per_step": {"own_cache": round(tot[0] / args.steps, 1), "peer_cache": round(tot[2] / args.steps, 1),
                                    "cpu_memory": round(tot[1] / args.steps, 1)},
                  "how": "hash split of the tablet; every member caches "
                         + ("1/K of the clique budget K * B, split by the cost model on the clique's summed hotness"
                            if clique_plan else "the workload's budgets") + "; peers simulated in local HBM"}
        del tabs, cstats

    cpu = None
    cpu_all = None
    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Oracle(indptr, indices, feats)
        nb = args.cpu_batches
        t_cpu = 0.0
        done = 0
        i = args.warmup
        while True:
            b = i % full_batches
            seeds = tablet[b * spec.batch:(b + 1) * spec.batch]
            c0 = time.perf_counter()
            res = orc.sample_khop(seeds, spec.fanouts, spec.base_seed + i)
            out = orc.gather(res.gather_ids)
            t_cpu += time.perf_counter() - c0
            done += 1
            i += 1
            del out
            if (nb and done >= nb) or (not nb and (t_cpu > 15.0 or done >= args.steps)):
                break
        cpu = {"value": round(done * spec.batch / t_cpu, 1), "unit": "seeds/s", "cores": 1, "kind": "oracle",
               "sample": f"{done} of the timed mini-batches (sample_khop + gather, same seeds and rng seeds)",
               "ms_per_step": round(t_cpu * 1e3 / done, 2)}
        # The same unchanged oracle on all host cores: independent instances on disjoint batches (threads; the
        # oracle calls run outside the interpreter lock).
        from concurrent.futures import ThreadPoolExecutor
        cores = len(os.sched_getaffinity(0))
        per_thread = max(1, min(done, 3))

        def work(t: int) -> int:
            for j in range(per_thread):
                i = args.warmup + t * per_thread + j
                b = i % full_batches
                res = orc.sample_khop(tablet[b * spec.batch:(b + 1) * spec.batch], spec.fanouts, spec.base_seed + i)
                orc.gather(res.gather_ids)
            return per_thread

        c0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as ex:
            total_batches = sum(ex.map(work, range(cores)))
        t_all = time.perf_counter() - c0
        cpu_all = {"value": round(total_batches * spec.batch / t_all, 1), "unit": "seeds/s", "cores": cores,
                   "kind": "oracle", "sample": f"{cores} independent oracle instances x {per_thread} mini-batches each"}

    line = {
        "metric": "seeds/sec through sample+gather; feature-gather GB/s vs HBM & PCIe peak",
        "value": round(seeds_per_s, 1), "unit": "seeds/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / opaque feature bytes", "data": "synthetic",
        "config": {"workload": f"{spec.name}: V={V} E={E} D={D} {spec.feat_dtype} fanouts={list(spec.fanouts)} "
                               f"batch={spec.batch} topo_cache={spec.topo_frac:g} feat_cache={spec.feat_frac:g}"
                               + (" (source feature table in HBM)" if args.features_on_device else ""),
                   "cached_topo_rows": plan.n_topo, "cached_feat_rows": plan.n_feat, "cache_plan": auto_plan,
                   "batches_in_tablet": n_batches},
        "roofline": roofline, "roofline_pcie": roofline_pcie, "cpu_baseline": cpu, "cpu_baseline_all_cores": cpu_all,
        "overlapped": overlapped, "pipelined": pipelined, "sampling_server": server, "graph_replay": graph_replay,
        "graph_constructor_ms": blocks_ms, "clique": clique,
        "per_step": {"gather_rows": round(gathered / args.steps, 1), "hit_rate": round(hit_rows / max(gathered, 1), 4),
                     "ms_sample": round(prof.ms_sample / max(prof.n_sample, 1), 4),
                     "ms_partition": round(prof.ms_partition / max(prof.n_partition, 1), 4),
                     "ms_hit_gather": round(prof.ms_hit / max(prof.n_hit, 1), 4),
                     "ms_miss_gather": round(prof.ms_miss / max(prof.n_miss, 1), 4)},
        "setup_s": {"generate": round(t_gen, 2), "build_hotness": round(t_hot, 3), "build_cache": round(t_cache, 3)},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
