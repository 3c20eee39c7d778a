"""GPU parity for the cache of a simulated clique (Algorithm 1's queues, each cut at its member's budget)
and the three-way feature extraction (own cache / peer's cache / CPU memory), against the CPU oracle."""
import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def W():
    from gpu_common import Workload
    return Workload(datagen.TINY)


def member_hotness(W, k_g, max_batches=-1):
    """Hash-split the training tablet into k_g member tablets (Sec. 4.1, S3) and pre-sample each."""
    spec = W.spec
    HT = np.empty((k_g, W.V), dtype=np.uint32)
    HF = np.empty((k_g, W.V), dtype=np.uint32)
    tablets = []
    for g in range(k_g):
        tab = np.ascontiguousarray(W.tablet[g::k_g])
        tablets.append(tab)
        W.ctx.build_hotness(torch.from_numpy(tab).cuda(), spec.batch, spec.fanouts, spec.base_seed + 1000 * g,
                            max_batches=max_batches)
        HT[g], HF[g] = W.ctx.get_hotness()
    return HT, HF, tablets


def as_dev(h):
    return torch.from_numpy(h.view(np.int32)).cuda()


def check_clique(W, k_g, HT, HF, tablets, tb, fb, n_batches=2, contents=True):
    from gpu_common import assert_batch_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    plans = W.ctx.build_clique_cache(as_dev(HT), as_dev(HF), tb, fb)
    topo_ids, feat_ids = W.orc.clique_plan(HT, HF, tb, fb)
    assert [p.n_topo for p in plans] == [t.size for t in topo_ids]
    assert [p.n_feat for p in plans] == [f.size for f in feat_ids]
    all_t, all_f = np.concatenate(topo_ids), np.concatenate(feat_ids)
    total = W.ctx.get_cache_plan()
    assert (total.n_topo, total.n_feat) == (all_t.size, all_f.size)
    g_topo, g_indptr, g_indices, g_feat, g_rows = W.ctx.get_cache(contents=contents)
    assert (g_topo == all_t).all() and (g_feat == all_f).all()
    r_indptr, r_indices = W.orc.fill_topo(all_t, all_t.size)
    assert (g_indptr == r_indptr).all()
    edges = np.diff(r_indptr)
    at = 0
    for g, p in enumerate(plans):                                   # every member's own share
        assert p.topo_edges == int(edges[at:at + p.n_topo].sum()) and p.topo_bytes == p.topo_edges * 4 + p.n_topo * 8
        assert p.topo_bytes <= tb and p.feat_bytes <= fb and p.feat_bytes == p.n_feat * W.orc.row_bytes
        at += p.n_topo
    if contents:
        assert (g_indices == r_indices).all()
        assert (g_rows == W.orc.fill_feat(all_f, all_f.size).view(np.uint8).reshape(all_f.size, W.orc.row_bytes)).all()
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
    stats = torch.zeros(3, dtype=torch.int32, device="cuda")
    stats2 = torch.zeros(2, dtype=torch.int32, device="cuda")
    for g in range(k_g):
        for b in range(n_batches):
            seeds = tablets[g][b * spec.batch:(b + 1) * spec.batch]
            seeds_dev = torch.from_numpy(seeds).cuda()
            W.ctx.sample_khop(seeds_dev, spec.fanouts, 31 * g + b, out=buf)
            ref = W.orc.sample_khop(seeds, spec.fanouts, 31 * g + b)
            assert_batch_equal(ref, buf.to_host(seeds_dev), f"member {g} batch {b}")
            n = ref.gather_ids.size
            rows = W.ctx.gather_features_clique(g, buf.gather_ids, n_dev=buf.n_gather, stats=stats)
            want = W.orc.gather(ref.gather_ids)
            assert torch.equal(rows[:n].cpu(), torch.from_numpy(want)), f"member {g} batch {b} rows"
            assert tuple(stats.tolist()) == W.orc.count_three_way(ref.gather_ids, feat_ids, g), f"member {g} batch {b}"
            rows2 = W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, stats=stats2)
            assert torch.equal(rows2[:n].cpu(), torch.from_numpy(want))
            assert stats2.tolist() == [stats[0].item() + stats[2].item(), stats[1].item()]
    W.ctx.check()


@pytest.mark.parametrize("k_g", [1, 2, 4, 8])
def test_clique_cache_tiny(W, k_g):
    HT, HF, tablets = member_hotness(W, k_g)
    rb = W.orc.row_bytes
    for tb, fb in ((20_000, 300 * rb), (0, 0), (10**9, 10**9), (3_000, 7 * rb + 1), (0, 50 * rb), (5_000, 0)):
        check_clique(W, k_g, HT, HF, tablets, tb, fb, n_batches=1)


def test_one_member_equals_the_single_gpu_cache(W):
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    ht, hf = W.ctx.get_hotness()
    tb, fb = datagen.budgets(spec, int(W.indices.size))
    plan = W.ctx.build_cache(tb, fb)
    single = W.ctx.get_cache()
    plans = W.ctx.build_clique_cache(as_dev(ht[None, :]), as_dev(hf[None, :]), tb, fb)
    assert (plans[0].n_topo, plans[0].topo_edges, plans[0].n_feat) == (plan.n_topo, plan.topo_edges, plan.n_feat)
    for a, b in zip(single, W.ctx.get_cache()):
        assert (a == b).all()


def test_clique_ids_edge_cases(W):
    """Empty id list, duplicates in any order, and hand-picked hotness rows with ties and empty queues."""
    V = W.V
    HT = np.zeros((3, V), dtype=np.uint32)
    HF = np.zeros((3, V), dtype=np.uint32)
    HF[0, :50] = 5                      # member 0 owns 0..49
    HF[2, 25:75] = 5                    # ties on 25..49 stay with member 0; member 2 owns 50..74; member 1 owns nothing hot
    HT[1, ::7] = 3
    rb = W.orc.row_bytes
    plans = W.ctx.build_clique_cache(as_dev(HT), as_dev(HF), 4_000, 60 * rb)
    topo_ids, feat_ids = W.orc.clique_plan(HT, HF, 4_000, 60 * rb)
    assert [p.n_feat for p in plans] == [f.size for f in feat_ids] and [p.n_topo for p in plans] == [t.size for t in topo_ids]
    stats = torch.full((3,), -1, dtype=torch.int32, device="cuda")
    out = W.ctx.gather_features_clique(1, torch.empty(0, dtype=torch.int32, device="cuda"), stats=stats)
    assert out.shape[0] == 0 and stats.tolist() == [0, 0, 0]
    ids = np.random.default_rng(4).integers(0, V, size=5000).astype(np.int32)
    ids[:200] = np.random.default_rng(5).integers(0, 80, size=200)        # many cached ones, with duplicates
    for g in range(3):
        rows = W.ctx.gather_features_clique(g, torch.from_numpy(ids).cuda(), stats=stats)
        assert torch.equal(rows.cpu(), torch.from_numpy(W.orc.gather(ids)))
        assert tuple(stats.tolist()) == W.orc.count_three_way(ids, feat_ids, g)
    W.ctx.check()


def test_clique_errors(W):
    import paper_2305_16588_amd as lgp
    spec = W.spec
    tb, fb = datagen.budgets(spec, int(W.indices.size))
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed, max_batches=1)
    W.ctx.build_cache(tb, fb)                                   # a single-GPU cache drops the clique
    ids = W.tablet_dev[:10].contiguous()
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.gather_features_clique(0, ids)
    assert e.value.status == -2
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.get_clique_plan(0)
    assert e.value.status == -2
    h = torch.zeros((9, W.V), dtype=torch.int32, device="cuda")
    with pytest.raises(lgp.LegionPrepError) as e:
        W.ctx.build_clique_cache(h, h, 0, 0)
    assert e.value.status == -4
    W.ctx.build_clique_cache(h[:2], h[:2], 1000, 1000)
    for member in (-1, 2):
        with pytest.raises(lgp.LegionPrepError) as e:
            W.ctx.gather_features_clique(member, ids)
        assert e.value.status == -1
    W.ctx.check()


def test_clique_cache_mid_full_size():
    """The mid workload (2.4 M vertices, ~62 M edges) at full size as a clique of four members: pre-sampling of each member's tablet, the clique plan,
    cached ids and contents, and three-way extraction of whole batches."""
    from gpu_common import Workload
    Wm = Workload(datagen.MID, device_gen="cuda")
    HT, HF, tablets = member_hotness(Wm, 4)
    spec = Wm.spec
    for g in range(4):                                              # the members' hotness rows themselves
        rt, rf, _ = Wm.orc.build_hotness(tablets[g], spec.batch, spec.fanouts, spec.base_seed + 1000 * g)
        assert (HT[g] == rt).all() and (HF[g] == rf).all()
    tb, fb = datagen.budgets(spec, int(Wm.indices.size))
    check_clique(Wm, 4, HT, HF, tablets, tb // 4, fb // 4, n_batches=1)


def test_clique_cache_large_full_size():
    """The large workload (111 M vertices, int64 offsets, 512-byte rows) as a clique of two members with caches far
    smaller than the graph: plans, cached ids, cached offsets, sampling, extracted bytes and the three counts
    (contents beyond that are covered by what sampling and extraction return).  LGP_SMALL=1 runs it at 1/8 size."""
    import os
    from gpu_common import Workload
    spec = datagen.LARGE
    scale = 1.0 if os.environ.get("LGP_SMALL", "0") != "1" else 0.125
    if scale != 1.0:
        spec = datagen.scaled(spec, scale)
    Wl = Workload(spec, device_gen="cuda")
    HT, HF, tablets = member_hotness(Wl, 2, max_batches=4)
    check_clique(Wl, 2, HT, HF, tablets, int(4e9 * scale), int(20e9 * scale), n_batches=1, contents=False)
