"""GPU parity at full size on the mid workload (config 2: 2.4 M vertices, ~62 M edges,
400-byte rows, fan-outs 15/10/5, batches of 8192), in the launch configuration bench.py
times: worst-case SampleBuffers, device-side counts, caches built from one pre-sampling
epoch with 50 % topology / 30 % features.  Everything is compared bit for bit."""
import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def W():
    from gpu_common import Workload
    w = Workload(datagen.MID, device_gen="cuda")
    assert abs(w.E - 62_000_000) / 62_000_000 < 0.05
    return w


def test_presampling_epoch_hotness(W):
    spec = W.spec
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    topo, feat = W.ctx.get_hotness()
    rt, rf, nb = W.orc.build_hotness(W.tablet, spec.batch, spec.fanouts, spec.base_seed)
    assert nb == 30                                            # 29 full batches + one of 2432 seeds
    assert (topo == rt).all() and (feat == rf).all()
    W.ctx.check()
    W.hot = (rt, rf)


def test_cache_plan_search_on_the_epoch_hotness(W):
    rt, rf = W.hot
    qt, qf = W.orc.rank_by_hotness(rt), W.orc.rank_by_hotness(rf)
    n_tsum = int(rt.sum())                                     # one transaction per traversed edge
    for B in (400_000_000, 1_200_000_000):
        best, pts = W.ctx.search_cache_plan(B, n_tsum)
        rbest, rpts = W.orc.search_cache_plan(rt, rf, qt, qf, B, n_tsum)
        assert best == rbest and 0 <= best <= 100
        for name in rpts.dtype.names:
            assert (pts[name] == rpts[name]).all(), name
    W.ctx.check()


def test_cache_plan_ids_and_contents(W):
    spec = W.spec
    rt, rf = W.hot
    topo_b, feat_b = datagen.budgets(spec, W.E)
    plan = W.ctx.build_cache(topo_b, feat_b)
    qt, qf = W.orc.rank_by_hotness(rt), W.orc.rank_by_hotness(rf)
    n_t, n_f = W.orc.plan_topo(qt, topo_b), W.orc.plan_feat(feat_b)
    assert n_f == 720_000 and (plan.n_topo, plan.n_feat) == (n_t, n_f)
    topo_ids, t_indptr, t_indices, feat_ids, feat_rows = W.ctx.get_cache()
    r_indptr, r_indices = W.orc.fill_topo(qt, n_t)
    assert (topo_ids == qt[:n_t]).all() and (feat_ids == qf[:n_f]).all()
    assert (t_indptr == r_indptr).all() and (t_indices == r_indices).all()
    assert feat_rows.tobytes() == W.orc.fill_feat(qf, n_f).tobytes()
    W.ctx.check()
    W.qf, W.n_f = qf, n_f


@pytest.mark.parametrize("b", [0, 13, 29])
def test_batch_sampling_and_gather(W, b):
    from gpu_common import assert_batch_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
    rows = torch.empty((buf.gather_cap, spec.feat_dim), dtype=torch.float32, device="cuda")
    stats = torch.zeros(2, dtype=torch.int32, device="cuda")
    seeds, seeds_dev = W.batch(b)
    assert seeds.size == (2432 if b == 29 else 8192)
    W.ctx.sample_khop(seeds_dev, spec.fanouts, spec.base_seed + 100 + b, out=buf)
    W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats)
    got = buf.to_host(seeds_dev)
    ref = W.orc.sample_khop(seeds, spec.fanouts, spec.base_seed + 100 + b)
    assert_batch_equal(ref, got, f"batch {b}")
    n = ref.gather_ids.size
    assert rows[:n].cpu().numpy().tobytes() == W.orc.gather(ref.gather_ids).tobytes()
    n_hit = W.orc.count_hits(ref.gather_ids, W.qf, W.n_f)
    assert stats.tolist() == [n_hit, n - n_hit] and 0 < n_hit < n
    W.ctx.check()


def test_graph_constructor_at_full_size(W):
    from gpu_common import assert_batch_equal, assert_blocks_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts, last_frontier=True)
    blk = lgp.BlockBuffers(buf)
    for b in (5, 29):
        seeds, seeds_dev = W.batch(b)
        W.ctx.sample_khop(seeds_dev, spec.fanouts, 99 + b, out=buf)
        W.ctx.build_blocks(seeds_dev, spec.fanouts, buf, out=blk)
        ref = W.orc.sample_khop(seeds, spec.fanouts, 99 + b, blocks=True)
        assert_batch_equal(ref, buf.to_host(seeds_dev), f"batch {b}")
        assert_blocks_equal(ref, blk.to_host(), f"batch {b}")
    W.ctx.check()
