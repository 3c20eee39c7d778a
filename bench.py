#!/usr/bin/env python3
"""Benchmark of the mini-batch data-preparation hot path on one MI355X.

One step = sample_khop + gather_features for one mini-batch of the workload's
training tablet (all per-batch stages; the caches are built beforehand from a
pre-sampling epoch, whose time is reported separately; the timed steps use other
rng seeds than that epoch, so cache hit rates are those of a later epoch).  Inputs are seeded and
synthetic (see datagen) and are resident -- graph and feature table in pinned CPU
memory (or HBM where the table exceeds what a process may pin), caches in HBM --
before the timed region starts.

The headline is the largest single-GPU workload ("share": one GPU's share of a
billion-scale graph).  The timed region of K steps is run R times (--reps; by
default as often as it takes to time at least half a second of work, and at
least five times); `value` / `ms_per_step` are the mean over all R x K steps,
the median, minimum and maximum of the R regions are reported beside it.  `configs` holds one shorter record per other
workload (tiny, mid, large, and the wide-feature sweep over the feature-cache
ratio), each with its own rooflines.

Prints ONE JSON line.  `roofline` covers the cache-hit row gather (HBM -> HBM),
`roofline_pcie` the miss row gather (CPU memory -> HBM), `roofline_sampler` the
whole lgp_sample_khop call; all use HIP events recorded by the library on the
streams the kernels run on.  `cpu_baseline` is the single-threaded CPU oracle
timed on a bounded sample of the headline's batches.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
PCIE_PEAK_GBS = 63.0           # PCIe Gen5 x16, one direction: 32 GT/s * 16 * 128/130 / 8
PINNED_LIMIT = 60 << 30        # a process on the GPU machines can pin at most 64 GiB of host memory
# Measured HBM traffic per launch shape, written by the profile summariser from the rocprofv3 --pmc passes whose
# text summaries sit next to it (FETCH_SIZE and WRITE_SIZE scaled by what a plain 1 GiB copy reads).
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(key: str):
    """The profile record of one launch shape ("share@topo1,feat1", "wide@topo1,feat0.25", ...), or (None, why)."""
    try:
        with open(TRAFFIC_JSON) as f:
            table = json.load(f)
    except (OSError, ValueError) as e:
        return None, f"no {os.path.relpath(TRAFFIC_JSON, ROOT)} ({type(e).__name__})"
    rec = table.get("launch_shapes", {}).get(key)
    if rec is None:
        return None, f"no profile of launch shape '{key}' in {os.path.relpath(TRAFFIC_JSON, ROOT)}"
    return rec, None


class Inputs:
    """One workload resident on the machine: arrays, context, pre-sampled hotness."""

    def __init__(self, spec, on_device_features: bool | None = None):
        import numpy as np
        import torch

        import datagen
        import paper_2305_16588_amd as lgp

        self.spec = spec
        elem = 4 if spec.feat_dtype == "float32" else 2
        host_bytes = 4 * spec.num_edges + 8 * spec.num_vertices + spec.num_vertices * spec.feat_dim * elem
        self.on_device = host_bytes > PINNED_LIMIT if on_device_features is None else on_device_features
        t0 = time.time()
        self.indptr = lgp.pinned_empty(spec.num_vertices + 1, np.int64 if spec.index64 else np.int32)
        _, self.indices = datagen.make_graph(spec, device="cuda", indptr_out=self.indptr,
                                             indices_alloc=lambda n: lgp.pinned_empty(n, np.int32))
        npdt = np.float32 if spec.feat_dtype == "float32" else np.float16
        if self.on_device:
            self.feats = np.empty((spec.num_vertices, spec.feat_dim), npdt)
        else:
            self.feats = lgp.pinned_empty((spec.num_vertices, spec.feat_dim), npdt)
        datagen.make_features(spec, device="cuda", out=self.feats)
        self.feats_src = self.feats
        if self.on_device:
            self.feats_src = torch.empty(self.feats.shape, device="cuda",
                                         dtype=torch.float32 if spec.feat_dtype == "float32" else torch.float16)
            for lo in range(0, spec.num_vertices, 1 << 22):
                self.feats_src[lo:lo + (1 << 22)].copy_(torch.from_numpy(self.feats[lo:lo + (1 << 22)]))
        self.tablet = datagen.make_tablet(spec, device="cuda")
        self.t_gen = time.time() - t0
        self.V, self.E, self.D = spec.num_vertices, int(self.indices.size), spec.feat_dim
        self.row_bytes = self.D * self.feats.dtype.itemsize
        self.ctx = lgp.Context(self.indptr, self.indices, self.feats_src)
        self.tablet_dev = torch.from_numpy(self.tablet).cuda()
        torch.cuda.synchronize()
        t0 = time.time()
        self.ctx.build_hotness(self.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
        torch.cuda.synchronize()
        self.t_hot = time.time() - t0
        self.full_batches = max(1, self.tablet.size // spec.batch)   # timed steps use full batches only
        self.n_batches = (self.tablet.size + spec.batch - 1) // spec.batch

    def seeds(self, i: int):
        b = i % self.full_batches
        return self.tablet_dev[b * self.spec.batch:(b + 1) * self.spec.batch]

    def close(self):
        import torch
        self.ctx.close()
        for name in ("indptr", "indices", "feats", "feats_src", "tablet_dev", "ctx"):
            setattr(self, name, None)
        gc.collect()
        torch.cuda.empty_cache()


def step_seed(spec, i: int) -> int:
    """rng seed of timed step i.  Pre-sampling used base_seed + b for batch b, so the timed steps draw other
    samples than the ones the caches were ranked on -- as later epochs of a training job do."""
    return spec.base_seed + (1 << 20) + i


def timed_regions(fn, first: int, steps: int, reps: int):
    """R back-to-back timed regions of K calls fn(i), each bracketed by a device synchronisation."""
    import torch
    out = []
    for r in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(first + r * steps, first + (r + 1) * steps):
            fn(i)
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def measure(inp: Inputs, steps: int, warmup: int, reps: int, topo_frac=None, feat_frac=None, cache_bytes: int = 0,
            alpha=None, overlap: bool = False, extras: bool = False, intra: bool = True, clique_k: int = 0,
            copy_calibration: bool = False):
    """Build the caches for the given ratios and time the step.  Returns one record."""
    import numpy as np
    import torch
    from dataclasses import replace

    import datagen
    import paper_2305_16588_amd as lgp

    spec = inp.spec
    if topo_frac is not None:
        spec = replace(spec, topo_frac=topo_frac)
    if feat_frac is not None:
        spec = replace(spec, feat_frac=feat_frac)
    ctx, V, E, D, row_bytes = inp.ctx, inp.V, inp.E, inp.D, inp.row_bytes
    ctx.set_overlap(overlap)
    topo_b, feat_b = datagen.budgets(spec, E)
    auto_plan = None
    if cache_bytes:
        ctx.build_cache(0, 0)                               # drop any earlier cache: the search re-ranks the vertices
        topo_hot, _ = ctx.get_hotness()
        # N_TSUM: pre-sampling reads one 128-byte line of column ids per vertex expansion; CLS = that line size
        _, n_tsum = ctx.get_presample_stats()
        best, pts = ctx.search_cache_plan(cache_bytes, n_tsum, cls_bytes=128)
        pick = best if alpha is None else int(round(alpha * 100))
        topo_b, feat_b = int(pts["m_topo"][pick]), int(pts["m_feat"][pick])
        per_row = -(-row_bytes // 128)
        all_t = max(int(topo_hot.sum()), 1)
        auto_plan = {"B": cache_bytes, "alpha": pick / 100, "alpha_by_cost_model": best / 100,
                     "predicted_N_total": round(n_tsum * int(pts["uncached_topo_hot"][pick]) / all_t
                                                + per_row * int(pts["uncached_feat_hot"][pick]))}
    t0 = time.time()
    plan = ctx.build_cache(topo_b, feat_b)
    t_cache = time.time() - t0

    L = len(spec.fanouts)
    total = warmup + max(reps, 5) * steps
    buf = lgp.SampleBuffers(V, spec.batch, spec.fanouts)
    rows = torch.empty((buf.gather_cap, D), dtype=ctx.feat_torch_dtype, device="cuda")
    stats = torch.zeros((total, 2), dtype=torch.int32, device="cuda")

    def step(i: int):
        ctx.sample_khop(inp.seeds(i), spec.fanouts, step_seed(spec, i), out=buf)
        ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats[i])

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ctx.check()
    if copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    # Timed regions: R x K steps, HIP events only on the two row gathers (hits: the kernel of `roofline`; misses:
    # `roofline_pcie`), which those launches record themselves.  The full breakdown of `per_step` and the sampler's
    # work counts come from an untimed pass over the first region's K steps with events around every kernel group.
    ctx.set_profiling(2)
    if reps <= 0:                                       # auto: at least 0.5 s of timed work, at least 5 regions
        probe = timed_regions(step, warmup, steps, 1)[0]
        reps = max(5, min(400, int(0.5 / max(probe, 1e-6)) + 1))
        ctx.get_profile()                               # the probe region's events are not part of the figures
        if warmup + reps * steps > stats.shape[0]:
            stats = torch.zeros((warmup + reps * steps, 2), dtype=torch.int32, device="cuda")
            for i in range(warmup):                     # `step` writes into the new tensor from here on
                step(i)
            torch.cuda.synchronize()
    regions = timed_regions(step, warmup, steps, reps)
    prof_g = ctx.get_profile()
    ctx.check()
    ctx.set_profiling(1)
    n_front = np.zeros(L, np.int64)        # frontier vertices expanded per hop, summed over the K steps
    n_edges = np.zeros(L, np.int64)        # column ids sampled per hop
    n_lists = 0                            # ids written by the compactions (frontiers 1 .. L-1 and the gather set)
    for i in range(warmup, warmup + steps):
        step(i)
        nf = buf.n_frontier.cpu().numpy()
        for h in range(L):
            n_front[h] += int(nf[h])
            n_edges[h] += int(buf.cnt[h][:int(nf[h])].sum().item())
            if h:
                n_lists += int(nf[h])
        n_lists += int(buf.n_gather.item())
    torch.cuda.synchronize()
    ctx.set_profiling(0)
    prof = ctx.get_profile()
    ctx.check()

    n_steps = reps * steps
    elapsed = sum(regions)
    ms_per_step = elapsed * 1e3 / n_steps
    per_region = [t * 1e3 / steps for t in regions]
    st = stats[warmup:].cpu().numpy().astype(np.int64)
    hit_rows, miss_rows = int(st[:, 0].sum()), int(st[:, 1].sum())
    gathered = hit_rows + miss_rows
    shape_key = (f"{inp.spec.name}@B{cache_bytes}" if cache_bytes
                 else f"{inp.spec.name}@topo{spec.topo_frac:g},feat{spec.feat_frac:g}")
    prof_rec, prof_why = measured_traffic(shape_key)

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
        per_row = (prof_rec or {}).get("hit_gather_hbm_bytes_per_row")
        roofline = {"bound": "hbm", "kernel": hit_kernel + " (cache hits, HBM->HBM)", "achieved": round(ach, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": round(per_row * hit_rows / prof_g.n_hit) if per_row else None,
                    "traffic_source": (prof_rec or {}).get("source") if per_row else prof_why or "no hit-gather figure",
                    "avg_launch_ms": round(prof_g.ms_hit / prof_g.n_hit, 4),
                    "rows_per_launch": round(hit_rows / prof_g.n_hit, 1), "bytes_per_row": hit_bytes_per_row}
    roofline_pcie = None
    if prof_g.n_miss and miss_rows:
        ach = miss_rows * row_bytes / (prof_g.ms_miss * 1e-3) / 1e9
        roofline_pcie = {"bound": "pcie", "kernel": miss_kernel + " (cache misses, CPU memory->HBM)",
                         "achieved": round(ach, 2), "peak": PCIE_PEAK_GBS, "unit": "GB/s",
                         "frac": round(ach / PCIE_PEAK_GBS, 4), "avg_launch_ms": round(prof_g.ms_miss / prof_g.n_miss, 4),
                         "rows_per_launch": round(miss_rows / prof_g.n_miss, 1), "bytes_per_row": row_bytes}
    # The sampler (whole lgp_sample_khop call: hop kernels + dedup compactions).  Algorithmic bytes per call:
    # per expanded vertex its id (4), its row-table entry (8) and the sampled column ids (4 each) are read, its
    # nbr row (4 f) and cnt (4) written; every sample sets one bit of the dedup bitmap (an atomic, not counted as
    # bytes); each of the L compactions reads the V/8-byte bitmap once and writes its id list (4 per id).
    roofline_sampler = None
    if prof.n_sample:
        f = np.asarray(spec.fanouts, np.int64)
        sampler_bytes = int((n_front * (4 + 8 + 4 + 4 * f)).sum() + 4 * n_edges.sum() + 4 * n_lists) + steps * L * (V // 8)
        ms_call = prof.ms_sample / prof.n_sample
        ach = sampler_bytes / steps / (ms_call * 1e-3) / 1e9
        s_traffic = (prof_rec or {}).get("sampler_hbm_bytes_per_call")
        roofline_sampler = {"bound": "hbm", "kernel": "lgp_sample_khop (sample_hop_kernel per hop, count_bits_kernel + "
                                                      "emit_bits_kernel per dedup)",
                            "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": s_traffic,
                            "traffic_source": (prof_rec or {}).get("source") if s_traffic else prof_why or "no sampler figure",
                            "occupancy_percent": (prof_rec or {}).get("sampler_occupancy_percent"),
                            "avg_call_ms": round(ms_call, 4), "bytes_per_call": round(sampler_bytes / steps),
                            "expanded_vertices_per_call": round(float(n_front.sum()) / steps, 1),
                            "bitmap_atomics_per_call": round(float(n_edges.sum()) / steps + spec.batch, 1)}

    rec = {
        "value": round(n_steps * spec.batch / elapsed, 1), "unit": "seeds/s", "steps": steps, "warmup": warmup,
        "reps": reps, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(statistics.median(per_region), 4),
        "ms_per_step_min": round(min(per_region), 4), "ms_per_step_max": round(max(per_region), 4),
        "timed_s": round(elapsed, 4),
        "config": {"workload": f"{inp.spec.name}: V={V} E={E} D={D} {spec.feat_dtype} fanouts={list(spec.fanouts)} "
                               f"batch={spec.batch} topo_cache={spec.topo_frac:g} feat_cache={spec.feat_frac:g}"
                               + (" (source feature table in HBM: the box pins at most 64 GiB of host memory)"
                                  if inp.on_device else ""),
                   "cached_topo_rows": plan.n_topo, "cached_feat_rows": plan.n_feat, "cache_plan": auto_plan,
                   "batches_in_tablet": inp.n_batches},
        "roofline": roofline, "roofline_pcie": roofline_pcie, "roofline_sampler": roofline_sampler,
        "per_step": {"gather_rows": round(gathered / n_steps, 1), "hit_rate": round(hit_rows / max(gathered, 1), 4),
                     "ms_sample": round(prof.ms_sample / max(prof.n_sample, 1), 4),
                     "ms_partition": round(prof.ms_partition / max(prof.n_partition, 1), 4),
                     "ms_hit_gather": round(prof.ms_hit / max(prof.n_hit, 1), 4),
                     "ms_miss_gather": round(prof.ms_miss / max(prof.n_miss, 1), 4)},
        "setup_s": {"generate": round(inp.t_gen, 2), "build_hotness": round(inp.t_hot, 3),
                    "build_cache": round(t_cache, 3)},
    }
    # Secondary figure: the intra-batch pipeline of Sec. 5 -- the same batches through lgp_sample_extract, which
    # extracts the seeds' rows while hop 0 is sampled and every hop's newly reached rows while the next hop is
    # sampled (rows come out in first-reach order instead of ascending id order).
    if intra:
        groups = torch.zeros(L + 2, dtype=torch.int32, device="cuda")
        istats = torch.zeros((warmup + steps, 2), dtype=torch.int32, device="cuda")

        def istep(i: int):
            ctx.sample_extract(inp.seeds(i), spec.fanouts, step_seed(spec, i), buf, rows, groups, istats[i])

        for i in range(warmup):
            istep(i)
        t_intra = timed_regions(istep, warmup, steps, 1)[0]
        ctx.check()
        assert torch.equal(istats[warmup:].cpu(), stats[warmup:warmup + steps].cpu()), "intra-batch pipeline diverged"
        rec["intra_batch_pipeline"] = {
            "value": round(steps * spec.batch / t_intra, 1), "unit": "seeds/s",
            "ms_per_step": round(t_intra * 1e3 / steps, 4),
            "how": "lgp_sample_extract: extraction of the seeds' rows beside hop 0, of each hop's newly reached rows "
                   "beside the next hop, on a second stream"}
    if extras:
        rec.update(secondary_figures(inp, spec, plan, buf, rows, stats, steps, warmup, ms_per_step, overlap, step))
    if clique_k > 0:
        rec["clique"] = clique_figure(inp, spec, buf, rows, steps, warmup, clique_k, topo_b, feat_b, cache_bytes)
    del buf, rows, stats
    return rec


def secondary_figures(inp, spec, plan, buf, rows, stats, steps, warmup, ms_per_step, overlap, step):
    """The pipelines of Sec. 5 and a HIP-graph replay over the same K steps (never the headline)."""
    import torch

    import paper_2305_16588_amd as lgp

    ctx, V = inp.ctx, inp.V
    ref_stats = stats[warmup:warmup + steps].cpu()

    def timed(fn):
        for i in range(warmup):
            fn(i)
        t = timed_regions(fn, warmup, steps, 1)[0]
        ctx.check()
        return {"value": round(steps * spec.batch / t, 1), "unit": "seeds/s", "ms_per_step": round(t * 1e3 / steps, 4)}

    # the library's hit / miss overlap (the miss gather on a stream of its own beside a narrower hit gather):
    # faster whenever both gathers have work, but the hit gather's own duration then says nothing about the
    # kernel, so the headline and the rooflines stay with overlap off
    overlapped = None
    if not overlap and 0 < plan.n_feat < V:
        ctx.set_overlap(True)
        overlapped = timed(step)
        overlapped["how"] = "lgp_set_overlap(1): miss gather on its own stream beside a narrower hit gather"
        ctx.set_overlap(False)
    both_gathers = overlapped is not None and overlapped["ms_per_step"] < ms_per_step

    # inter-batch pipeline: sampling of batch i+1 on a second stream beside the feature extraction of batch i
    ctx.set_overlap(overlap or both_gathers)
    (sA, sB, sC), streams_concurrent = lgp.concurrent_streams(3)
    bufs = [buf, lgp.SampleBuffers(V, spec.batch, spec.fanouts)]
    outs = [rows, torch.empty_like(rows)]
    ev_sampled = [torch.cuda.Event(), torch.cuda.Event()]
    ev_gathered = [torch.cuda.Event(), torch.cuda.Event()]
    pstats = torch.zeros((steps + warmup, 2), dtype=torch.int32, device="cuda")

    def pstep(i: int):
        k = i % 2
        if i >= 2:
            sA.wait_event(ev_gathered[k])              # buffer k is free again
        ctx.sample_khop(inp.seeds(i), spec.fanouts, step_seed(spec, i), out=bufs[k], stream=sA)
        ev_sampled[k].record(sA)
        sB.wait_event(ev_sampled[k])
        ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=outs[k], stats=pstats[i], stream=sB)
        ev_gathered[k].record(sB)

    torch.cuda.synchronize()
    pipelined = timed(pstep)
    assert torch.equal(pstats[warmup:].cpu(), ref_stats), "pipelined run diverged"
    pipelined["how"] = ("sample_khop of batch i+1 on a second stream beside gather_features of batch i"
                        + (", hit / miss overlap on" if both_gathers else "")
                        + ("" if streams_concurrent else "; no three streams on hardware queues of their own found"))
    del bufs, outs

    # the whole sampling server of Sec. 5 -- neighbour sampler, graph constructor and feature extractor per batch --
    # serial on one stream, and as the two pipelines the section describes
    bufs = [lgp.SampleBuffers(V, spec.batch, spec.fanouts, last_frontier=True) for _ in range(2)]
    blks = [lgp.BlockBuffers(b) for b in bufs]
    outs = [rows, torch.empty_like(rows)]
    ev_s = [torch.cuda.Event(), torch.cuda.Event()]
    ev_g = [torch.cuda.Event(), torch.cuda.Event()]
    ev_b = [torch.cuda.Event(), torch.cuda.Event()]
    sstats = torch.zeros((steps + warmup, 2), dtype=torch.int32, device="cuda")

    def serial_step(i: int):
        seeds = inp.seeds(i)
        ctx.sample_khop(seeds, spec.fanouts, step_seed(spec, i), out=bufs[0])
        ctx.build_blocks(seeds, spec.fanouts, bufs[0], out=blks[0])
        ctx.gather_features(bufs[0].gather_ids, n_dev=bufs[0].n_gather, out=outs[0], stats=sstats[i])

    def piped_step(i: int):
        k = i % 2
        seeds = inp.seeds(i)
        if i >= 2:
            sA.wait_event(ev_g[k])                      # buffer k is free again
            sA.wait_event(ev_b[k])
        ctx.sample_khop(seeds, spec.fanouts, step_seed(spec, i), out=bufs[k], stream=sA)
        ev_s[k].record(sA)
        sB.wait_event(ev_s[k])
        sC.wait_event(ev_s[k])
        ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=outs[k], stats=sstats[i], stream=sB)
        ev_g[k].record(sB)
        ctx.build_blocks(seeds, spec.fanouts, bufs[k], out=blks[k], stream=sC)
        ev_b[k].record(sC)

    server = {}
    for name, fn in (("serial", serial_step), ("pipelined", piped_step)):
        ctx.set_overlap(overlap or (both_gathers and fn is piped_step))
        torch.cuda.synchronize()
        server[name] = timed(fn)
        assert torch.equal(sstats[warmup:].cpu(), ref_stats), "sampling-server run diverged"
    server["how"] = ("step = sample_khop + build_blocks + gather_features; pipelined = three streams: build_blocks "
                     "beside gather_features of the same batch, sample_khop of the next batch beside both"
                     + (", hit / miss overlap on" if both_gathers else ""))
    ctx.set_overlap(overlap)

    # graph constructor alone, on the same batches
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total_ms, n_timed = 0.0, min(steps, 20)
    for i in range(warmup, warmup + n_timed + 2):
        seeds = inp.seeds(i)
        ctx.sample_khop(seeds, spec.fanouts, step_seed(spec, i), out=bufs[0])
        e0.record()
        ctx.build_blocks(seeds, spec.fanouts, bufs[0], out=blks[0])
        e1.record()
        torch.cuda.synchronize()
        if i >= warmup + 2:
            total_ms += e0.elapsed_time(e1)
    blocks_ms = round(total_ms / n_timed, 4)
    ctx.check()
    del bufs, blks, outs

    # the same step captured once into a HIP graph (sampling, dedup, partition, gathers: about a dozen launches) and
    # replayed; seeds change per replay, the rng seed is the captured one
    seeds_buf = inp.tablet_dev[:spec.batch].clone()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        ctx.sample_khop(seeds_buf, spec.fanouts, step_seed(spec, 0), out=buf)
        ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats[0])

    def replay(i: int):
        seeds_buf.copy_(inp.seeds(i), non_blocking=True)
        g.replay()

    graph_replay = timed(replay)
    graph_replay["how"] = "one captured HIP graph per step, replayed; seeds copied in before each replay"
    del g
    return {"overlapped": overlapped, "pipelined": pipelined, "sampling_server": server, "graph_replay": graph_replay,
            "graph_constructor_ms": blocks_ms}


def clique_figure(inp, spec, buf, rows, steps, warmup, K, topo_b, feat_b, cache_bytes):
    """The step as member 0 of a simulated clique of K GPUs.  Every member pre-samples its own hash share of the
    tablet and contributes a cache; rows a peer caches are read from the peer's region of this device's HBM, so the
    time says nothing about a real inter-GPU link -- the split {own cache, peer's cache, CPU memory} is the result.
    Replaces the context's cache and hotness."""
    import numpy as np
    import torch

    ctx, V = inp.ctx, inp.V
    HT = torch.empty((K, V), dtype=torch.int32, device="cuda")
    HF = torch.empty((K, V), dtype=torch.int32, device="cuda")
    tabs = []
    sum_t, sum_f, n_tsum_c = np.zeros(V, np.uint64), np.zeros(V, np.uint64), 0
    for g in range(K):
        tabs.append(inp.tablet_dev[g::K].contiguous())
        ctx.build_hotness(tabs[g], spec.batch, spec.fanouts, spec.base_seed + 1000 * g)
        th, fh = ctx.get_hotness()
        HT[g].copy_(torch.from_numpy(th.view(np.int32)))
        HF[g].copy_(torch.from_numpy(fh.view(np.int32)))
        sum_t += th
        sum_f += fh
        n_tsum_c += ctx.get_presample_stats()[1]
    ctopo_b, cfeat_b, clique_plan = topo_b, feat_b, None
    if cache_bytes:
        # Sec. 4.3 at clique granularity: the cost model runs on the clique's summed hotness (A_T, A_F) with the
        # clique's budget K * B and the clique's N_TSUM; every member then gets 1/K of each share.
        ctx.build_cache(0, 0)                                   # drop the cache: the search re-ranks the vertices
        ctx.set_hotness(np.minimum(sum_t, 2**32 - 1).astype(np.uint32), np.minimum(sum_f, 2**32 - 1).astype(np.uint32))
        cbest, cpts = ctx.search_cache_plan(K * cache_bytes, n_tsum_c, cls_bytes=128)
        ctopo_b, cfeat_b = int(cpts["m_topo"][cbest]) // K, int(cpts["m_feat"][cbest]) // K
        clique_plan = {"B_per_member": cache_bytes, "alpha_by_cost_model": cbest / 100}
    plans = ctx.build_clique_cache(HT, HF, ctopo_b, cfeat_b)
    del HT, HF
    my_batches = max(1, tabs[0].numel() // spec.batch)
    cstats = torch.zeros((steps + warmup, 3), dtype=torch.int32, device="cuda")

    def cstep(i: int):
        b = i % my_batches
        seeds = tabs[0][b * spec.batch:(b + 1) * spec.batch]
        ctx.sample_khop(seeds, spec.fanouts, step_seed(spec, i), out=buf)
        ctx.gather_features_clique(0, buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=cstats[i])

    for i in range(warmup):
        cstep(i)
    t = timed_regions(cstep, warmup, steps, 1)[0]
    ctx.check()
    n_seeds = min(spec.batch, tabs[0].numel())
    tot = cstats[warmup:].sum(dim=0).tolist()
    return {"k_g": K, "member": 0, "value": round(steps * n_seeds / t, 1), "unit": "seeds/s",
            "ms_per_step": round(t * 1e3 / steps, 4), "cache_plan": clique_plan,
            "cached_topo_rows": [p.n_topo for p in plans], "cached_feat_rows": [p.n_feat for p in plans],
            "rows_per_step": {"own_cache": round(tot[0] / steps, 1), "peer_cache": round(tot[2] / steps, 1),
                              "cpu_memory": round(tot[1] / steps, 1)},
            "how": "hash split of the tablet; every member caches "
                   + ("1/K of the clique budget K * B, split by the cost model on the clique's summed hotness"
                      if clique_plan else "the workload's budgets") + "; peers simulated in local HBM"}


def cpu_baseline(inp: Inputs, first: int, max_batches: int, budget_s: float = 15.0):
    """The CPU oracle as it stands on a bounded sample of the same batches: one core, then every host core."""
    import oracle
    spec = inp.spec
    orc = oracle.Oracle(inp.indptr, inp.indices, inp.feats)

    def one(i: int):
        b = i % inp.full_batches
        res = orc.sample_khop(inp.tablet[b * spec.batch:(b + 1) * spec.batch], spec.fanouts, step_seed(spec, i))
        orc.gather(res.gather_ids)

    t_cpu, done = 0.0, 0
    while done < max_batches and t_cpu < budget_s:
        c0 = time.perf_counter()
        one(first + done)
        t_cpu += time.perf_counter() - c0
        done += 1
    cpu = {"value": round(done * spec.batch / t_cpu, 1), "unit": "seeds/s", "cores": 1, "kind": "oracle",
           "sample": f"{done} of the timed mini-batches of the headline workload (sample_khop + gather, same seeds "
                     "and rng seeds)",
           "ms_per_step": round(t_cpu * 1e3 / done, 2)}
    # The same unchanged oracle on all host cores: independent instances on disjoint batches (threads; the
    # oracle calls run outside the interpreter lock).
    from concurrent.futures import ThreadPoolExecutor
    cores = len(os.sched_getaffinity(0))
    per_thread = max(1, min(done, 3))

    def work(t: int) -> int:
        for j in range(per_thread):
            one(first + t * per_thread + j)
        return per_thread

    c0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        total_batches = sum(ex.map(work, range(cores)))
    t_all = time.perf_counter() - c0
    cpu_all = {"value": round(total_batches * spec.batch / t_all, 1), "unit": "seeds/s", "cores": cores,
               "kind": "oracle", "sample": f"{cores} independent oracle instances x {per_thread} mini-batches each"}
    return cpu, cpu_all


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--reps", type=int, default=0,
                    help="timed regions of --steps steps each (mean, median, min and max reported); 0 = as many as it "
                         "takes to time at least 0.5 s of work, at least 5")
    ap.add_argument("--workload", default="share",
                    help="headline workload: tiny | mid | wide | large | share (optionally name@scale); the default "
                         "is the largest single-GPU one")
    ap.add_argument("--configs", default="all",
                    help="'all' = also one short record per other workload (tiny, mid, large, wide-feature sweep) "
                         "under `configs`; 'none' = headline only")
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
                    help="skip the secondary figures (hit / miss overlap, pipelines of Sec. 5, HIP-graph replay)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--features-on-device", action="store_true",
                    help="keep the source feature table in HBM even if it could be pinned")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=0, help="oracle batches to time (0 = as many as fit ~15 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the work; --gpus must be 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        return 2

    import torch

    import datagen
    import paper_2305_16588_amd  # noqa: F401  (fails loudly if the HIP library is missing)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3

    def spec_of(text: str):
        name, _, scale = text.partition("@")
        spec = datagen.WORKLOADS[name]
        return datagen.scaled(spec, float(scale)) if scale else spec

    t_start = time.time()
    head_spec = spec_of(args.workload)
    fallback = None
    try:
        inp = Inputs(head_spec, on_device_features=True if args.features_on_device else None)
    except Exception as e:                         # the box cannot hold the largest workload: say so, take the next
        if args.workload != "share":
            raise
        fallback = f"share did not fit this box ({type(e).__name__}: {e}); headline is the large workload instead"
        print("bench.py: " + fallback, file=sys.stderr)
        gc.collect()
        torch.cuda.empty_cache()
        head_spec = datagen.WORKLOADS["large"]
        inp = Inputs(head_spec)
    head = measure(inp, args.steps, args.warmup, args.reps, topo_frac=args.topo_frac, feat_frac=args.feat_frac,
                   cache_bytes=args.cache_bytes, alpha=args.alpha, overlap=args.overlap,
                   extras=not args.no_pipeline, intra=not args.no_pipeline, clique_k=args.clique,
                   copy_calibration=args.copy_calibration)
    cpu = cpu_all = None
    if not args.no_cpu_baseline:
        cpu, cpu_all = cpu_baseline(inp, args.warmup, args.cpu_batches or args.steps)
    inp.close()
    del inp

    configs = {}
    if args.configs == "all":
        k, w, r = min(args.steps, 10), min(args.warmup, 3), 3
        for name in ("tiny", "mid", "large", "share"):
            if name == head_spec.name:
                continue
            try:
                other = Inputs(datagen.WORKLOADS[name])
                configs[name] = measure(other, k, w, r, intra=not args.no_pipeline)
                other.close()
                del other
            except Exception as e:
                configs[name] = {"error": f"{type(e).__name__}: {e}"}
                gc.collect()
                torch.cuda.empty_cache()
        if head_spec.name != "wide":
            try:
                other = Inputs(datagen.WORKLOADS["wide"])
                for frac in (0.0, 0.10, 0.25, 0.50, 1.0):
                    configs[f"wide@feat{frac:g}"] = measure(other, k, w, r, feat_frac=frac, intra=not args.no_pipeline)
                other.close()
                del other
            except Exception as e:
                configs["wide"] = {"error": f"{type(e).__name__}: {e}"}

    line = {
        "metric": "seeds/sec through sample+gather; feature-gather GB/s vs HBM & PCIe peak",
        "value": head["value"], "unit": "seeds/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "reps": head["reps"], "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"],
        "ms_per_step_min": head["ms_per_step_min"], "ms_per_step_max": head["ms_per_step_max"],
        "timed_s": head["timed_s"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / opaque feature bytes", "data": "synthetic",
        "config": dict(head["config"], headline_choice=fallback or (
            "share is the largest single-GPU workload of the five (250 M vertices, 8 B edges); the others are "
            "under `configs`" if head_spec.name == "share" else "chosen with --workload")),
        "roofline": head["roofline"], "roofline_pcie": head["roofline_pcie"],
        "roofline_sampler": head["roofline_sampler"], "cpu_baseline": cpu, "cpu_baseline_all_cores": cpu_all,
        "per_step": head["per_step"], "setup_s": head["setup_s"],
    }
    for key in ("intra_batch_pipeline", "overlapped", "pipelined", "sampling_server", "graph_replay",
                "graph_constructor_ms", "clique"):
        line[key] = head.get(key)
    line["configs"] = configs
    line["bench_wall_s"] = round(time.time() - t_start, 1)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
