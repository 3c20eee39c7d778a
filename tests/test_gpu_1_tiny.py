"""GPU parity on the tiny workload (config 1) and on edge cases: every output of the
HIP path is compared bit for bit with the CPU oracle on the same seeded inputs."""
import os

import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def W():
    from gpu_common import Workload
    return Workload(datagen.TINY)


def test_sampling_every_batch_of_the_epoch(W):
    from gpu_common import assert_batch_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
    n_batches = (W.tablet.size + spec.batch - 1) // spec.batch
    assert n_batches == 10
    for b in range(n_batches):
        seeds, seeds_dev = W.batch(b)
        W.ctx.sample_khop(seeds_dev, spec.fanouts, spec.base_seed + b, out=buf)
        got = buf.to_host(seeds_dev)
        ref = W.orc.sample_khop(seeds, spec.fanouts, spec.base_seed + b)
        assert_batch_equal(ref, got, f"batch {b}")
    W.ctx.check()


@pytest.mark.parametrize("fanouts", [(1,), (64,), (3, 2, 2, 2), (25, 10), (15, 10, 5), (16, 8), (33, 2), (2,) * 8,
                                     (64, 64)])
def test_sampling_fanout_shapes(W, fanouts):
    from gpu_common import assert_batch_equal
    seeds, seeds_dev = W.tablet[:300], W.tablet_dev[:300]
    buf = W.ctx.sample_khop(seeds_dev, fanouts, 777)
    assert_batch_equal(W.orc.sample_khop(seeds, fanouts, 777), buf.to_host(seeds_dev), str(fanouts))
    W.ctx.check()


def test_sampling_degenerate_inputs(W):
    from gpu_common import assert_batch_equal
    deg = np.diff(W.indptr)
    iso = np.flatnonzero(deg == 0)[:3].astype(np.int32)
    hub = np.array([int(np.argmax(deg))], dtype=np.int32)
    for seeds in (np.empty(0, np.int32), iso, hub, np.concatenate([iso, hub])):
        dev = torch.from_numpy(seeds).cuda()
        buf = W.ctx.sample_khop(dev, (10, 5), 2**63 + 11)      # seed with the high word in use
        assert_batch_equal(W.orc.sample_khop(seeds, (10, 5), 2**63 + 11), buf.to_host(dev), f"seeds {seeds}")
    W.ctx.check()


def test_hotness_whole_epoch(W):
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    topo, feat = W.ctx.get_hotness()
    rt, rf, nb = W.orc.build_hotness(W.tablet, spec.batch, spec.fanouts, spec.base_seed)
    assert nb == 10 and (topo == rt).all() and (feat == rf).all()
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed, max_batches=3)
    topo, feat = W.ctx.get_hotness()
    rt, rf, nb = W.orc.build_hotness(W.tablet, spec.batch, spec.fanouts, spec.base_seed, max_batches=3)
    assert nb == 3 and (topo == rt).all() and (feat == rf).all()
    expansions = 0                                             # sum of all frontier sizes = row reads over PCIe
    for b in range(3):
        res = W.orc.sample_khop(W.batch(b)[0], spec.fanouts, spec.base_seed + b)
        expansions += sum(res.frontier[h].size for h in range(len(spec.fanouts)))
    assert W.ctx.get_presample_stats() == (3, expansions)
    W.ctx.check()


def _check_cache(W, topo_budget, feat_budget):
    plan = W.ctx.build_cache(topo_budget, feat_budget)
    topo_hot, feat_hot = W.ctx.get_hotness()
    qt, qf = W.orc.rank_by_hotness(topo_hot), W.orc.rank_by_hotness(feat_hot)
    n_t, n_f = W.orc.plan_topo(qt, topo_budget), W.orc.plan_feat(feat_budget)
    assert (plan.n_topo, plan.n_feat) == (n_t, n_f)
    topo_ids, t_indptr, t_indices, feat_ids, feat_rows = W.ctx.get_cache()
    r_indptr, r_indices = W.orc.fill_topo(qt, n_t)
    assert (topo_ids == qt[:n_t]).all() and (feat_ids == qf[:n_f]).all()
    assert (t_indptr == r_indptr).all() and (t_indices == r_indices).all()
    assert plan.topo_edges == r_indices.size and plan.topo_bytes == 4 * r_indices.size + 8 * n_t
    assert feat_rows.tobytes() == W.orc.fill_feat(qf, n_f).tobytes()
    return plan, qf


def test_cache_selection_and_contents(W):
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    total_t = 4 * W.E + 8 * W.V
    tb, fb = datagen.budgets(spec, W.E)
    for topo_budget, feat_budget in [(tb, fb), (0, 0), (total_t, W.V * 512), (total_t - 1, W.V * 512 - 1), (8, 511),
                                     (total_t * 3, 10**12), (tb, 0), (0, fb)]:
        _check_cache(W, topo_budget, feat_budget)
    W.ctx.check()


def test_cache_is_transparent_to_sampling_and_gather(W):
    from gpu_common import assert_batch_equal
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    seeds, seeds_dev = W.batch(2)
    ref = W.orc.sample_khop(seeds, spec.fanouts, 31337)
    ref_rows = W.orc.gather(ref.gather_ids)
    total_t = 4 * W.E + 8 * W.V
    for topo_frac, feat_frac in [(0.0, 0.0), (0.2, 0.2), (1.0, 1.0), (0.0, 1.0), (1.0, 0.0), (0.5, 0.01)]:
        plan, qf = _check_cache(W, int(topo_frac * total_t), int(feat_frac * W.V) * 512)
        buf = W.ctx.sample_khop(seeds_dev, spec.fanouts, 31337)
        assert_batch_equal(ref, buf.to_host(seeds_dev), f"cache {topo_frac}/{feat_frac}")
        stats = torch.zeros(2, dtype=torch.int32, device="cuda")
        rows = W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, stats=stats)
        n = int(buf.n_gather.item())
        assert n == ref.gather_ids.size
        assert rows[:n].cpu().numpy().tobytes() == ref_rows.tobytes()
        n_hit = W.orc.count_hits(ref.gather_ids, qf, plan.n_feat)
        assert stats.tolist() == [n_hit, n - n_hit]
    W.ctx.check()


def test_gather_any_id_list(W):
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    W.ctx.build_cache(0, 2000 * 512)
    rng = np.random.default_rng(4)
    for n in (0, 1, 63, 64, 65, 1000, 4097, 30000):
        ids = rng.integers(0, W.V, size=n).astype(np.int32)    # duplicates, arbitrary order
        dev = torch.from_numpy(ids).cuda()
        rows = W.ctx.gather_features(dev)
        assert rows.shape == (n, spec.feat_dim)
        assert rows.cpu().numpy().tobytes() == W.orc.gather(ids).tobytes()
    W.ctx.check()


def test_determinism_same_call_twice(W):
    spec = W.spec
    seeds, seeds_dev = W.batch(1)
    a = W.ctx.sample_khop(seeds_dev, spec.fanouts, 5)
    b = W.ctx.sample_khop(seeds_dev, spec.fanouts, 5)
    torch.cuda.synchronize()
    assert torch.equal(a.n_frontier, b.n_frontier) and torch.equal(a.n_gather, b.n_gather)
    n = int(a.n_gather.item())
    assert torch.equal(a.gather_ids[:n], b.gather_ids[:n]) and torch.equal(a.nbr[0], b.nbr[0])
    ra = W.ctx.gather_features(a.gather_ids[:n].contiguous())
    rb = W.ctx.gather_features(a.gather_ids[:n].contiguous())
    assert torch.equal(ra, rb)


def test_workspace_bytes(W):
    """The library's own HBM use for a batch shape, against the sizes of what it actually allocates."""
    import paper_2305_16588_amd as lgp
    fo = (10, 5)
    fixed, scratch = W.ctx.workspace_bytes(1024, fo)
    V = W.V
    need, gather = lgp.worst_case_sizes(V, 1024, fo)
    assert fixed >= 28 * V and fixed < 28 * V + 2 * (V * 32 // 8 + 8192 * 8) + 4096      # tables + two (sparse) bitmaps
    want = 6 * 4 * gather + (len(fo) + 1) * V * 4 + sum((n // 1024 + 1) * 8 for n in need[:-1]) + 4 * sum(need[1:-1])
    assert scratch == want
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.workspace_bytes(1024, (65,))
    assert e.value.status == -4


def test_argument_errors_are_reported_on_the_host(W):
    import paper_2305_16588_amd as lgp
    seeds_dev = W.tablet_dev[:100]
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.sample_khop(seeds_dev, (65,), 1)
    assert e.value.status == -4
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.sample_khop(seeds_dev, (0,), 1)
    assert e.value.status == -1
    small = lgp.SampleBuffers(W.V, 50, (10, 5))
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.sample_khop(seeds_dev, (2,) * 9, 1, out=small)   # more hops than LGP_MAX_HOPS
    assert e.value.status == -4
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.sample_khop(seeds_dev, (10, 5), 1, out=small)
    assert e.value.status == -3
    fresh = lgp.Context(W.indptr, W.indices, W.features)
    with pytest.raises(lgp.LegionPrepError) as e:
        fresh.build_cache(100, 100)
    assert e.value.status == -2
    unpinned = np.array(W.indptr)
    with pytest.raises(lgp.LegionPrepError) as e:
        lgp.Context(unpinned, W.indices, W.features)
    assert e.value.status == -1
    fresh.close()


def test_invalid_vertex_id_sets_the_device_flag(W):
    import paper_2305_16588_amd as lgp
    bad = torch.tensor([1, W.V, 5], dtype=torch.int32, device="cuda")
    W.ctx.sample_khop(bad, (3,), 1)
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.check()
    assert e.value.status == -7
    W.ctx.check()                                              # the flag is cleared once reported
    W.ctx.gather_features(torch.tensor([-1, 2], dtype=torch.int32, device="cuda"))
    with pytest.raises(lgp.LegionPrepError):
        W.ctx.check()
    # the context keeps working afterwards
    seeds, seeds_dev = W.batch(0)
    from gpu_common import assert_batch_equal
    buf = W.ctx.sample_khop(seeds_dev, (10, 5), 9)
    assert_batch_equal(W.orc.sample_khop(seeds, (10, 5), 9), buf.to_host(seeds_dev))


def test_int64_offsets_and_fp16_rows():
    from gpu_common import Workload, assert_batch_equal
    from dataclasses import replace
    spec = replace(datagen.TINY, name="tiny64", feat_dim=7, feat_dtype="float16", index64=True)
    Wl = Workload(spec)
    assert Wl.indptr.dtype == np.int64 and Wl.features.dtype == np.float16
    seeds, seeds_dev = Wl.batch(0)
    buf = Wl.ctx.sample_khop(seeds_dev, (10, 5), 3)
    ref = Wl.orc.sample_khop(seeds, (10, 5), 3)
    assert_batch_equal(ref, buf.to_host(seeds_dev))
    Wl.ctx.build_hotness(Wl.tablet_dev, 1024, (10, 5), 1, max_batches=2)
    Wl.ctx.build_cache(10**6, 14 * 3000)
    n = int(buf.n_gather.item())
    rows = Wl.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather)       # 14-byte rows: 2-byte chunks
    assert rows[:n].cpu().numpy().tobytes() == Wl.orc.gather(ref.gather_ids).tobytes()
    buf2 = Wl.ctx.sample_khop(seeds_dev, (10, 5), 3)
    assert_batch_equal(ref, buf2.to_host(seeds_dev))
    Wl.ctx.check()


def test_row_longer_than_the_packed_degree_field():
    """A vertex with >= 2^24 - 1 out-neighbours does not fit the 24-bit degree of the row table and is
    served from the CPU-resident CSR, cached or not."""
    import oracle
    import paper_2305_16588_amd as lgp
    from gpu_common import assert_batch_equal
    big = (1 << 24) + 5
    V = big + 10
    indptr = lgp.pinned_empty(V + 1, np.int64)
    indptr[0] = 0
    indptr[1] = big                                            # vertex 0 -> 1 .. big
    indptr[2:] = big + np.arange(1, V, dtype=np.int64)         # every other vertex v -> v - 1
    indices = lgp.pinned_empty(big + V - 1, np.int32)
    indices[:big] = np.arange(1, big + 1, dtype=np.int32)
    indices[big:] = np.arange(0, V - 1, dtype=np.int32)
    ctx = lgp.Context(indptr, indices, None)
    orc = oracle.Oracle(indptr, indices)
    seeds = np.array([0, 9, V - 1], dtype=np.int32)
    dev = torch.from_numpy(seeds).cuda()
    ref = orc.sample_khop(seeds, (12, 3), 99)
    assert ref.cnt[0].tolist() == [12, 1, 1]
    assert_batch_equal(ref, ctx.sample_khop(dev, (12, 3), 99).to_host(dev), "no cache")
    ctx.build_hotness(dev, 3, (12, 3), 99)
    plan = ctx.build_cache(10**12, 0)
    assert plan.n_topo == V
    assert_batch_equal(ref, ctx.sample_khop(dev, (12, 3), 99).to_host(dev), "everything cached")
    ctx.check()


@pytest.mark.parametrize("B,n_tsum,cls,n_alpha", [(600_000, 3_000_000, 64, 101), (2_000_000, 50_000, 64, 11),
                                                  (50_000, 10**9, 128, 21), (0, 5, 64, 2), (10**10, 123, 64, 1024),
                                                  (400_000, 100_000, 64, 101)])
def test_cache_plan_search(B, n_tsum, cls, n_alpha):
    """Cost model + alpha search (Sec. 4.3) against the oracle: every candidate and the winner."""
    from gpu_common import Workload
    Wl = Workload(datagen.TINY)
    spec = Wl.spec
    Wl.ctx.build_hotness(Wl.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    topo, feat = Wl.ctx.get_hotness()
    qt, qf = Wl.orc.rank_by_hotness(topo), Wl.orc.rank_by_hotness(feat)
    best, pts = Wl.ctx.search_cache_plan(B, n_tsum, cls, n_alpha)
    rbest, rpts = Wl.orc.search_cache_plan(topo, feat, qt, qf, B, n_tsum, cls, n_alpha)
    assert best == rbest
    for name in rpts.dtype.names:
        assert (pts[name] == rpts[name]).all(), name
    # building the chosen plan caches exactly what the search promised
    plan = Wl.ctx.build_cache(int(pts["m_topo"][best]), int(pts["m_feat"][best]))
    assert (plan.n_topo, plan.n_feat) == (int(pts["n_topo"][best]), int(pts["n_feat"][best]))
    Wl.ctx.check()


@pytest.mark.parametrize("k_g,V,hi,seed", [(1, 5000, 6, 0), (2, 100_000, 4, 1), (4, 333_333, 3, 2), (8, 1_000_000, 40, 3),
                                           (64, 70_001, 2, 4), (3, 1, 9, 5)])
def test_cslp_algorithm_1(k_g, V, hi, seed):
    """Algorithm 1 for a clique of k_g GPUs against the oracle (sums, ranking, owners, per-GPU queues)."""
    import oracle
    import paper_2305_16588_amd as lgp
    hot = np.random.default_rng(seed).integers(0, hi, size=(k_g, V)).astype(np.uint32)
    if V > 10:
        hot[:, 3] = 2**32 - 1                                   # column sum beyond 32 bits
    acc, order, owner, queues, offsets = lgp.cslp(torch.from_numpy(hot.view(np.int32)).cuda())
    racc, rorder, rowner, rqueues, roffsets = oracle.cslp(hot)
    assert (acc.cpu().numpy().view(np.uint64) == racc).all()
    assert (order.cpu().numpy() == rorder).all() and (owner.cpu().numpy() == rowner).all()
    assert offsets == roffsets.tolist() and (queues.cpu().numpy() == rqueues).all()


@pytest.mark.parametrize("fanouts,n_seeds", [((10, 5), 1024), ((15, 10, 5), 700), ((3,), 1), ((64, 2), 100), ((4, 4), 0),
                                             ((5, 5, 5, 5), 2048)])
def test_graph_constructor_blocks(W, fanouts, n_seeds):
    """Sec. 5's graph constructor: per-hop CSR blocks in local numbering + feature-matrix rows, against the oracle."""
    from gpu_common import assert_batch_equal, assert_blocks_equal
    import paper_2305_16588_amd as lgp
    seeds, seeds_dev = W.tablet[:n_seeds], W.tablet_dev[:n_seeds].contiguous()
    buf = lgp.SampleBuffers(W.V, max(n_seeds, 1), fanouts, last_frontier=True)
    W.ctx.sample_khop(seeds_dev, fanouts, 4242, out=buf)
    blk = W.ctx.build_blocks(seeds_dev, fanouts, buf)
    ref = W.orc.sample_khop(seeds, fanouts, 4242, blocks=True)
    assert_batch_equal(ref, buf.to_host(seeds_dev), str(fanouts))
    assert_blocks_equal(ref, blk.to_host(), str(fanouts))
    # a second batch through the same buffers (the lookup table is reused without clearing)
    W.ctx.sample_khop(seeds_dev, fanouts, 4243, out=buf)
    W.ctx.build_blocks(seeds_dev, fanouts, buf, out=blk)
    ref = W.orc.sample_khop(seeds, fanouts, 4243, blocks=True)
    assert_blocks_equal(ref, blk.to_host(), str(fanouts) + " second batch")
    W.ctx.check()


def test_plan_cache_and_set_hotness():
    """lgp_plan_cache reports what lgp_build_cache then builds; hotness loaded with lgp_set_hotness ranks the same."""
    from gpu_common import Workload
    import paper_2305_16588_amd as lgp
    Wl = Workload(datagen.TINY)
    spec = Wl.spec
    rt, rf, _ = Wl.orc.build_hotness(Wl.tablet, spec.batch, spec.fanouts, spec.base_seed)
    with pytest.raises(lgp.LegionPrepError) as e:
        Wl.ctx.plan_cache(1000, 1000)                           # no hotness yet
    assert e.value.status == -2
    Wl.ctx.set_hotness(rt, rf)                                  # a saved ranking, no pre-sampling on the GPU
    topo_b, feat_b = datagen.budgets(spec, Wl.E)
    p = Wl.ctx.plan_cache(topo_b, feat_b)
    qt, qf = Wl.orc.rank_by_hotness(rt), Wl.orc.rank_by_hotness(rf)
    n_t, n_f = Wl.orc.plan_topo(qt, topo_b), Wl.orc.plan_feat(feat_b)
    assert (p.n_topo, p.n_feat, p.feat_bytes) == (n_t, n_f, n_f * 512)
    assert p.topo_bytes == int((np.diff(Wl.indptr)[qt[:n_t]].astype(np.int64) * 4 + 8).sum()) <= topo_b
    b = Wl.ctx.build_cache(topo_b, feat_b)
    built = (b.n_topo, b.topo_edges, b.topo_bytes, b.n_feat, b.feat_bytes)
    assert built == (p.n_topo, p.topo_edges, p.topo_bytes, p.n_feat, p.feat_bytes)
    topo_ids, _, _, feat_ids, _ = Wl.ctx.get_cache()
    assert (topo_ids == qt[:n_t]).all() and (feat_ids == qf[:n_f]).all()
    with pytest.raises(lgp.LegionPrepError) as e:
        Wl.ctx.plan_cache(topo_b, feat_b)                       # planning re-ranks: only before a cache exists
    assert e.value.status == -2


def test_overlap_profiling_and_three_stream_pipelining(W):
    """The optional modes change scheduling only: same results with hit / miss overlap, with event profiling on,
    and with the three operators on three streams -- sampling of the next batch beside the graph constructor and
    the feature extraction of the current one."""
    from gpu_common import assert_batch_equal, assert_blocks_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    W.ctx.build_cache(*datagen.budgets(spec, W.E))
    refs = [W.orc.sample_khop(W.batch(b)[0], spec.fanouts, 600 + b, blocks=True) for b in range(4)]
    rows_ref = [W.orc.gather(r.gather_ids) for r in refs]
    (sA, sB, sC), found = lgp.concurrent_streams(3)           # three streams, on hardware queues of their own if possible
    assert isinstance(found, bool) and len({sA.cuda_stream, sB.cuda_stream, sC.cuda_stream}) == 3
    bufs = [lgp.SampleBuffers(W.V, spec.batch, spec.fanouts, last_frontier=True) for _ in range(2)]
    blks = [lgp.BlockBuffers(bufs[k]) for k in range(2)]
    W.ctx.build_blocks(W.batch(0)[1], spec.fanouts, W.ctx.sample_khop(W.batch(0)[1], spec.fanouts, 1, out=bufs[0]),
                       out=blks[0])                              # first call allocates the constructor's scratch
    W.ctx.set_overlap(True)
    W.ctx.set_profiling(True)
    outs = [torch.empty((bufs[0].gather_cap, spec.feat_dim), dtype=torch.float32, device="cuda") for _ in range(2)]
    sampled = [torch.cuda.Event() for _ in range(2)]
    gathered = [torch.cuda.Event() for _ in range(2)]
    built = [torch.cuda.Event() for _ in range(2)]
    copied, blocks = [], []
    torch.cuda.synchronize()
    for b in range(4):
        k = b % 2
        if b >= 2:
            sA.wait_event(gathered[k])
            sA.wait_event(built[k])
        W.ctx.sample_khop(W.batch(b)[1], spec.fanouts, 600 + b, out=bufs[k], stream=sA)
        sampled[k].record(sA)
        sB.wait_event(sampled[k])
        sC.wait_event(sampled[k])
        W.ctx.gather_features(bufs[k].gather_ids, n_dev=bufs[k].n_gather, out=outs[k], stream=sB)
        W.ctx.build_blocks(W.batch(b)[1], spec.fanouts, bufs[k], out=blks[k], stream=sC)
        with torch.cuda.stream(sB):                             # snapshot before the buffer is reused
            copied.append((outs[k][:refs[b].gather_ids.size].clone(), bufs[k].gather_ids[:refs[b].gather_ids.size].clone(),
                           bufs[k].n_gather.clone()))
        gathered[k].record(sB)
        with torch.cuda.stream(sC):
            blocks.append(blks[k].to_host())
        built[k].record(sC)
    torch.cuda.synchronize()
    for b in range(4):
        rows, gids, n = copied[b]
        assert int(n.item()) == refs[b].gather_ids.size and (gids.cpu().numpy() == refs[b].gather_ids).all()
        assert rows.cpu().numpy().tobytes() == rows_ref[b].tobytes()
        assert_blocks_equal(refs[b], blocks[b], f"batch {b}")
    prof = W.ctx.get_profile()
    assert prof.n_sample == 4 and prof.n_partition == 4 and prof.n_hit == 4 and prof.n_miss == 4
    assert prof.ms_sample > 0 and prof.ms_hit > 0 and prof.ms_miss > 0
    W.ctx.set_overlap(False)
    W.ctx.set_profiling(False)
    assert W.ctx.get_profile().n_sample == 0                     # reading resets the accumulators
    # mode 2 times the two row gathers only; the launches carry their own start / stop events
    W.ctx.set_profiling(2)
    for b in range(3):
        W.ctx.sample_khop(W.batch(b)[1], spec.fanouts, 600 + b, out=bufs[0])
        W.ctx.gather_features(bufs[0].gather_ids, n_dev=bufs[0].n_gather, out=outs[0])
    torch.cuda.synchronize()
    n = refs[2].gather_ids.size
    assert outs[0][:n].cpu().numpy().tobytes() == rows_ref[2].tobytes()
    prof = W.ctx.get_profile()
    assert (prof.n_sample, prof.n_partition, prof.n_hit, prof.n_miss) == (0, 0, 3, 3)
    assert 0 < prof.ms_hit < 50 and 0 < prof.ms_miss < 50 and prof.ms_sample == 0
    W.ctx.set_profiling(0)
    W.ctx.check()


@pytest.mark.parametrize("overlap", [False, True])
def test_hip_graph_capture_and_replay(W, overlap):
    """One batch's whole launch sequence (sampling, dedup, partition, both gathers) captured into a HIP graph and
    replayed with new seeds in the same buffer: every replay matches the oracle and the eager result.  The path
    records no memset node; eager work and synchronisations run between replays.  With overlap on, the library's
    own miss stream forks from and rejoins the captured stream."""
    from gpu_common import assert_batch_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    W.ctx.build_cache(*datagen.budgets(spec, W.E))
    W.ctx.set_overlap(overlap)
    seeds_buf = W.tablet_dev[:spec.batch].clone()
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
    rows = torch.empty((buf.gather_cap, spec.feat_dim), dtype=torch.float32, device="cuda")
    stats = torch.zeros(2, dtype=torch.int32, device="cuda")
    # warm-up outside capture: grows the library's list scratch (allocation is not capturable)
    W.ctx.sample_khop(seeds_buf, spec.fanouts, 31, out=buf)
    W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        W.ctx.sample_khop(seeds_buf, spec.fanouts, 31, out=buf)
        W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats)
    for b in (3, 0, 7, 3):
        seeds, seeds_dev = W.batch(b)
        seeds_buf.copy_(seeds_dev)                                     # eager work between replays
        rows.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref = W.orc.sample_khop(seeds, spec.fanouts, 31)
        assert_batch_equal(ref, buf.to_host(seeds_buf), f"replay of batch {b}")
        n = ref.gather_ids.size
        assert rows[:n].cpu().numpy().tobytes() == W.orc.gather(ref.gather_ids).tobytes()
        assert int(stats.sum().item()) == n
        eager = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
        W.ctx.sample_khop(seeds_dev, spec.fanouts, 31, out=eager)       # eager call between replays
        assert_batch_equal(ref, eager.to_host(seeds_dev), f"eager after replay {b}")
    W.ctx.set_overlap(False)
    W.ctx.check()


@pytest.mark.parametrize("n,seed,epoch", [(0, 1, 0), (1, 2, 0), (10_000, 2**40 + 17, 3), (1_000_003, 5, 2**31)])
def test_batch_generator_shuffle(n, seed, epoch):
    import oracle
    import paper_2305_16588_amd as lgp
    ids = np.random.default_rng(n).integers(0, 2**31 - 1, size=n).astype(np.int32)
    out = lgp.shuffle_tablet(torch.from_numpy(ids).cuda(), seed, epoch)
    assert (out.cpu().numpy() == oracle.shuffle_tablet(ids, seed, epoch)).all()


def test_duplicate_seeds_and_presampling_through_an_existing_cache(W):
    """Seeds given twice are expanded twice (identical rows) and merge at the first dedup; pre-sampling after a
    cache was built reads through that cache and still counts exactly what the oracle counts."""
    from gpu_common import assert_batch_equal
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    W.ctx.build_cache(*datagen.budgets(spec, W.E))
    seeds = np.concatenate([W.tablet[:50], W.tablet[:50], W.tablet[40:90]]).astype(np.int32)
    dev = torch.from_numpy(seeds).cuda()
    buf = W.ctx.sample_khop(dev, (10, 5), 8)
    ref = W.orc.sample_khop(seeds, (10, 5), 8)
    assert_batch_equal(ref, buf.to_host(dev), "duplicate seeds")
    assert (ref.nbr[0][:50] == ref.nbr[0][50:100]).all()
    tab = torch.from_numpy(np.concatenate([seeds, W.tablet[:3000]])).cuda()
    W.ctx.build_hotness(tab, 700, spec.fanouts, 77)              # cache from above is in place
    topo, feat = W.ctx.get_hotness()
    rt, rf, _ = W.orc.build_hotness(tab.cpu().numpy(), 700, spec.fanouts, 77)
    assert (topo == rt).all() and (feat == rf).all()
    W.ctx.check()


@pytest.mark.parametrize("dim,dtype", [(1, "float16"), (2, "float16"), (3, "float32"), (6, "float32"), (4, "float32"),
                                       (20, "float32"), (36, "float32"), (100, "float16"), (256, "float32"),
                                       (1024, "float32"), (8192, "float16"), (16384, "float32")])
def test_gather_row_widths(dim, dtype):
    """Every chunk width (2 / 4 / 8 / 16 bytes) and lane-group size of the two gather kernels, from 2-byte rows to
    the 64-KiB limit, through the partitioned path and both direct paths (nothing cached / everything cached)."""
    import oracle
    import paper_2305_16588_amd as lgp
    V = 3000
    indptr, indices = datagen.tiny_graph(V, 4.0, 3)
    rng = np.random.default_rng(dim)
    npdt = np.float16 if dtype == "float16" else np.float32
    feats = lgp.pinned_empty((V, dim), npdt)
    feats[...] = rng.standard_normal((V, dim)).astype(npdt)
    p_indptr, p_indices = lgp.pinned_copy(indptr), lgp.pinned_copy(indices)
    ctx = lgp.Context(p_indptr, p_indices, feats)
    orc = oracle.Oracle(indptr, indices, feats)
    row_bytes = dim * np.dtype(npdt).itemsize
    ids = rng.integers(0, V, size=2500).astype(np.int32)
    dev = torch.from_numpy(ids).cuda()
    ref = orc.gather(ids).tobytes()
    ctx.set_hotness(rng.integers(0, 9, V).astype(np.uint32), rng.integers(0, 9, V).astype(np.uint32))
    for n_cached in (0, 1200, V):
        plan = ctx.build_cache(0, n_cached * row_bytes)
        assert plan.n_feat == n_cached
        stats = torch.zeros(2, dtype=torch.int32, device="cuda")
        rows = ctx.gather_features(dev, stats=stats)
        assert rows.cpu().numpy().tobytes() == ref, f"{n_cached} rows cached"
        assert int(stats.sum().item()) == ids.size
    ctx.check()
    ctx.close()


def test_row_wider_than_the_limit_is_refused():
    import paper_2305_16588_amd as lgp
    indptr, indices = datagen.tiny_graph(10, 2.0, 1)
    feats = lgp.pinned_empty((10, 16385), np.float32)           # 65 540-byte rows: 4-byte chunks, 16 385 of them
    with pytest.raises(lgp.LegionPrepError) as e:
        lgp.Context(lgp.pinned_copy(indptr), lgp.pinned_copy(indices), feats)
    assert e.value.status == -4


@pytest.mark.parametrize("case", range(int(os.environ.get("LGP_RANDOM_CASES", "24"))))
def test_randomized_small_workloads(case):
    """Random small graphs, feature widths, fan-out lists, seed sets and cache splits: sampling, blocks and
    gathered bytes against the oracle, also through the fixed-scratch extraction, a random slice of the cache
    and the intra-batch pipeline; then the same graph with the cache of a random clique.
    LGP_RANDOM_CASES sets the number of cases (default 24)."""
    import oracle
    import paper_2305_16588_amd as lgp
    from gpu_common import assert_batch_equal, assert_blocks_equal
    rng = np.random.default_rng(1000 + case)
    V = int(rng.integers(1, 4000))
    indptr, indices = datagen.tiny_graph(V, float(rng.uniform(0.0, 12.0)), case)
    if rng.random() < 0.5:
        indptr = indptr.astype(np.int64)
    dim = int(rng.integers(1, 70))
    npdt = np.float16 if rng.random() < 0.5 else np.float32
    feats = lgp.pinned_empty((V, dim), npdt)
    feats[...] = rng.standard_normal((V, dim)).astype(npdt)
    p_indptr, p_indices = lgp.pinned_copy(indptr), lgp.pinned_copy(indices)
    ctx = lgp.Context(p_indptr, p_indices, feats)
    orc = oracle.Oracle(indptr, indices, feats)
    fanouts = tuple(int(x) for x in rng.integers(1, 65, size=int(rng.integers(1, 5))))
    tablet = rng.permutation(V).astype(np.int32)
    batch = int(rng.integers(1, max(2, V // 2 + 1)))
    tab_dev = torch.from_numpy(tablet).cuda()
    ctx.build_hotness(tab_dev, batch, fanouts, case)
    rt, rf, _ = orc.build_hotness(tablet, batch, fanouts, case)
    gt, gf = ctx.get_hotness()
    assert (gt == rt).all() and (gf == rf).all()
    row_bytes = dim * np.dtype(npdt).itemsize
    topo_b = int(rng.uniform(0, 1.2) * (4 * indices.size + 8 * V))
    feat_b = int(rng.uniform(0, 1.2) * V) * row_bytes
    plan = ctx.build_cache(topo_b, feat_b)
    qt, qf = orc.rank_by_hotness(rt), orc.rank_by_hotness(rf)
    assert (plan.n_topo, plan.n_feat) == (orc.plan_topo(qt, topo_b), orc.plan_feat(feat_b))
    seeds = tablet[:batch]
    dev = tab_dev[:batch].contiguous()
    seed = int(rng.integers(0, 2**63))
    buf = lgp.SampleBuffers(V, batch, fanouts, last_frontier=True)
    ctx.sample_khop(dev, fanouts, seed, out=buf)
    blk = ctx.build_blocks(dev, fanouts, buf)
    stats = torch.zeros(2, dtype=torch.int32, device="cuda")
    rows = ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, stats=stats)
    ref = orc.sample_khop(seeds, fanouts, seed, blocks=True)
    assert_batch_equal(ref, buf.to_host(dev), f"case {case}")
    assert_blocks_equal(ref, blk.to_host(), f"case {case}")
    n = ref.gather_ids.size
    assert rows[:n].cpu().numpy().tobytes() == orc.gather(ref.gather_ids).tobytes()
    n_hit = orc.count_hits(ref.gather_ids, qf, plan.n_feat)
    assert stats.tolist() == [n_hit, n - n_hit]
    # the same extraction through the fixed scratch block, a slice of the cache, and the intra-batch pipeline
    rows2 = torch.empty_like(rows)
    stats.fill_(-1)
    ctx.gather_features_static(buf.gather_ids, buf.n_gather, rows2, stats)
    assert rows2[:n].cpu().numpy().tobytes() == orc.gather(ref.gather_ids).tobytes() and stats.tolist() == [n_hit, n - n_hit]
    if plan.n_feat:
        lo = int(rng.integers(0, plan.n_feat))
        cnt = int(rng.integers(0, plan.n_feat - lo + 1))
        assert ctx.get_cache_part(1, lo, cnt).tobytes() == orc.fill_feat(qf[lo:lo + cnt], cnt).tobytes()
    if plan.topo_edges:
        full = orc.fill_topo(qt, plan.n_topo)[1]
        lo = int(rng.integers(0, plan.topo_edges))
        cnt = int(rng.integers(0, plan.topo_edges - lo + 1))
        assert (ctx.get_cache_part(0, lo, cnt) == full[lo:lo + cnt]).all()
    pbuf = lgp.SampleBuffers(V, batch, fanouts)
    prow = torch.empty((max(pbuf.gather_cap, 1), dim), dtype=ctx.feat_torch_dtype, device="cuda")
    groups = torch.zeros(len(fanouts) + 2, dtype=torch.int32, device="cuda")
    stats.fill_(-1)
    ctx.sample_extract(dev, fanouts, seed, pbuf, prow, groups, stats)
    fr, nbr, cnt_, listing = pbuf.to_host(dev)
    for h in range(len(fanouts)):
        assert (fr[h] == ref.frontier[h]).all() and (nbr[h] == ref.nbr[h]).all() and (cnt_[h] == ref.cnt[h]).all()
    assert listing.tolist() == ref.hop_order.tolist() and groups.tolist() == ref.hop_seg.tolist()
    assert prow[:n].cpu().numpy().tobytes() == orc.gather(ref.hop_order).tobytes() and stats.tolist() == [n_hit, n - n_hit]
    # the cache of a clique of k_g members with random hotness rows (many ties and zeros), three-way extraction
    k_g = int(rng.integers(1, 9))
    HT = rng.integers(0, 4, size=(k_g, V)).astype(np.uint32)
    HF = rng.integers(0, 4, size=(k_g, V)).astype(np.uint32)
    tb, fb = topo_b // k_g, (feat_b // row_bytes // k_g) * row_bytes + int(rng.integers(0, row_bytes))
    plans = ctx.build_clique_cache(torch.from_numpy(HT.view(np.int32)).cuda(), torch.from_numpy(HF.view(np.int32)).cuda(),
                                   tb, fb)
    topo_ids, feat_ids = orc.clique_plan(HT, HF, tb, fb)
    assert [p.n_topo for p in plans] == [t.size for t in topo_ids]
    assert [p.n_feat for p in plans] == [f.size for f in feat_ids]
    g_topo, g_indptr, g_indices, g_feat, g_rows = ctx.get_cache()
    all_t, all_f = np.concatenate(topo_ids), np.concatenate(feat_ids)
    assert (g_topo == all_t).all() and (g_feat == all_f).all()
    r_indptr, r_indices = orc.fill_topo(all_t, all_t.size)
    assert (g_indptr == r_indptr).all() and (g_indices == r_indices).all()
    assert g_rows.tobytes() == orc.fill_feat(all_f, all_f.size).tobytes()
    ctx.sample_khop(dev, fanouts, seed + 1, out=buf)
    ref = orc.sample_khop(seeds, fanouts, seed + 1)
    assert_batch_equal(ref, buf.to_host(dev), f"case {case} with the clique cache")
    n = ref.gather_ids.size
    stats3 = torch.zeros(3, dtype=torch.int32, device="cuda")
    member = int(rng.integers(0, k_g))
    rows = ctx.gather_features_clique(member, buf.gather_ids, n_dev=buf.n_gather, stats=stats3)
    assert rows[:n].cpu().numpy().tobytes() == orc.gather(ref.gather_ids).tobytes()
    assert tuple(stats3.tolist()) == orc.count_three_way(ref.gather_ids, feat_ids, member)
    ctx.check()
    ctx.close()
