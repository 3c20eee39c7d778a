"""lgp_reserve: after it the per-batch calls allocate nothing and never synchronise, so the whole sampling
server of one batch -- sample_khop + build_blocks + gather_features -- can be captured into a HIP graph on a fresh
context with no warm-up call at that shape (stream capture fails on any allocation or synchronisation), and a
shape beyond the reservation is refused instead of growing the scratch."""
import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


def test_capture_without_warm_up_after_reserve():
    from gpu_common import Workload, assert_batch_equal, assert_blocks_equal
    import paper_2305_16588_amd as lgp
    spec = datagen.scaled(datagen.MID, 0.05, name="mid-twentieth")      # 120 k vertices, 3 hops, 400-byte rows
    W = Workload(spec, device_gen="cuda")
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    plan = W.ctx.build_cache(*datagen.budgets(spec, W.E))
    assert 0 < plan.n_feat < W.V                                        # both gathers and the partition lists are used
    fixed, scratch = W.ctx.workspace_bytes(spec.batch, spec.fanouts)
    W.ctx.reserve(spec.batch, spec.fanouts)
    seeds_buf = W.tablet_dev[:spec.batch].clone()
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts, last_frontier=True)
    blk = lgp.BlockBuffers(buf)
    rows = torch.empty((buf.gather_cap, spec.feat_dim), dtype=torch.float32, device="cuda")
    stats = torch.zeros(2, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):                                           # the first calls of these operators ever
        W.ctx.sample_khop(seeds_buf, spec.fanouts, 77, out=buf)
        W.ctx.build_blocks(seeds_buf, spec.fanouts, buf, out=blk)
        W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, out=rows, stats=stats)
    for b in (1, 0, 2, 1):
        seeds, seeds_dev = W.batch(b)
        seeds_buf[:seeds_dev.numel()].copy_(seeds_dev)                   # eager work between replays
        rows.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref = W.orc.sample_khop(seeds_buf.cpu().numpy(), spec.fanouts, 77, blocks=True)
        assert_batch_equal(ref, buf.to_host(seeds_buf), f"replay of batch {b}")
        assert_blocks_equal(ref, blk.to_host(), f"replay of batch {b}")
        n = ref.gather_ids.size
        assert rows[:n].cpu().numpy().tobytes() == W.orc.gather(ref.gather_ids).tobytes()
        assert int(stats.sum().item()) == n
        eager = W.ctx.gather_features(buf.gather_ids[:n].contiguous())   # eager call between replays
        assert eager.cpu().numpy().tobytes() == W.orc.gather(ref.gather_ids).tobytes()
    # a larger shape than reserved is refused, not grown
    big = torch.zeros(buf.gather_cap + 1, dtype=torch.int32, device="cuda")
    with pytest.raises(lgp.LegionPrepError) as err:
        W.ctx.gather_features(big)
    assert err.value.status == -3                                       # LGP_ECAPACITY
    W.ctx.check()


def test_shapes_beyond_the_reservation_are_refused():
    from gpu_common import Workload
    import paper_2305_16588_amd as lgp
    W = Workload(datagen.TINY)
    spec = W.spec
    W.ctx.reserve(16, spec.fanouts)                                     # room for batches of 16 seeds only
    for call in (lambda: W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed),
                 lambda: W.ctx.build_blocks(W.tablet_dev[:16].contiguous(), (10, 5, 5),
                                            lgp.SampleBuffers(W.V, 16, (10, 5, 5), last_frontier=True))):
        with pytest.raises(lgp.LegionPrepError) as err:
            call()
        assert err.value.status == -3                                   # LGP_ECAPACITY, nothing was launched
    W.ctx.build_hotness(W.tablet_dev, 16, spec.fanouts, spec.base_seed)  # within the reservation
    W.ctx.reserve(spec.batch, spec.fanouts)                             # reserving again for more lifts the limit
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    rt, rf, _ = W.orc.build_hotness(W.tablet, spec.batch, spec.fanouts, spec.base_seed)
    gt, gf = W.ctx.get_hotness()
    assert (gt == rt).all() and (gf == rf).all()
    W.ctx.check()
