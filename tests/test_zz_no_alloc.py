"""lgp_gather_features_static (the entry point for callers that cannot allocate) against lgp_gather_features:
same bytes and the same {n_hit, n_miss}, on two calls in a row -- the second with a smaller input, so the fixed
scratch block still holds the first call's longer lists -- and on the paths that skip the lists."""
import ctypes as C

import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


def _both(W, ids, n_dev=None):
    """(rows, stats) through the allocating entry point and through the static one."""
    D = W.spec.feat_dim
    outs = []
    for static in (False, True):
        out = torch.full((ids.numel(), D), -7.0, dtype=W.ctx.feat_torch_dtype, device="cuda")
        stats = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        if static:
            W.ctx.gather_features_static(ids, n_dev, out, stats)
        else:
            W.ctx.gather_features(ids, n_dev=n_dev, out=out, stats=stats)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy(), stats.tolist()))
    return outs


def _check_pair(W, ids, n_dev=None, tag=""):
    (ref_rows, ref_stats), (rows, stats) = _both(W, ids, n_dev)
    assert stats == ref_stats, f"{tag}: stats {stats} != {ref_stats}"
    assert rows.tobytes() == ref_rows.tobytes(), f"{tag}: gathered bytes differ"
    n = int(n_dev.item()) if n_dev is not None else ids.numel()
    want = W.orc.gather(ids[:n].cpu().numpy())
    assert rows[:n].tobytes() == want.tobytes(), f"{tag}: bytes differ from the oracle's"
    return stats


def test_static_gather_matches_on_two_calls_in_a_row():
    from gpu_common import Workload
    spec = datagen.scaled(datagen.MID, 0.1, name="mid-tenth")           # 240 k vertices, 400-byte rows
    W = Workload(spec, device_gen="cuda")
    W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed)
    topo_b, feat_b = datagen.budgets(spec, W.E)
    plan = W.ctx.build_cache(topo_b, feat_b)
    assert 0 < plan.n_feat < W.V
    g = torch.Generator().manual_seed(77)
    # first call: 200 000 ids (several hundred partition tiles, ragged tail), duplicates and any order allowed
    ids1 = torch.randint(0, W.V, (200_003,), generator=g, dtype=torch.int32).cuda()
    s1 = _check_pair(W, ids1, tag="first call")
    assert s1[0] > 0 and s1[1] > 0
    # second call, smaller, right behind it: the block still holds the first call's lists and counters
    ids2 = torch.randint(0, W.V, (1_237,), generator=g, dtype=torch.int32).cuda()
    s2 = _check_pair(W, ids2, tag="second, smaller call")
    assert s2[0] + s2[1] == 1_237
    # device-side count below n_max, then an empty call
    n_dev = torch.tensor([4_099], dtype=torch.int32, device="cuda")
    s3 = _check_pair(W, ids1[:50_000].contiguous(), n_dev, tag="device-side count")
    assert s3[0] + s3[1] == 4_099
    (ref_rows, ref_stats), (rows, stats) = _both(W, ids1[:0].contiguous())
    assert stats == ref_stats == [0, 0]
    # hit / miss overlap mode uses the same block
    W.ctx.set_overlap(True)
    _check_pair(W, ids1, tag="overlap mode")
    W.ctx.set_overlap(False)
    # the paths that need no lists: everything cached, nothing cached
    W.ctx.build_cache(topo_b, W.V * W.orc.row_bytes)
    assert _check_pair(W, ids2, tag="everything cached") == [1_237, 0]
    W.ctx.build_cache(topo_b, 0)
    assert _check_pair(W, ids2, tag="nothing cached") == [0, 1_237]
    W.ctx.check()


def test_static_gather_refuses_what_does_not_fit():
    from gpu_common import Workload
    import paper_2305_16588_amd as lgp
    from paper_2305_16588_amd.binding import STATIC_GATHER_MAX_IDS
    W = Workload(datagen.TINY)
    W.ctx.build_hotness(W.tablet_dev, W.spec.batch, W.spec.fanouts, W.spec.base_seed)
    W.ctx.build_cache(*datagen.budgets(W.spec, W.E))
    ids = torch.zeros(16, dtype=torch.int32, device="cuda")
    out = torch.zeros((16, W.spec.feat_dim), dtype=torch.float32, device="cuda")
    # refused on the host before any launch, so the short buffers are never touched
    st = W.ctx._L.lgp_gather_features_static(W.ctx._h, ids.data_ptr(), STATIC_GATHER_MAX_IDS + 1, None,
                                              out.data_ptr(), None, C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == -3                                                      # LGP_ECAPACITY
    assert b"LGP_STATIC_GATHER_MAX_IDS" in W.ctx._L.lgp_last_error(W.ctx._h)
    with pytest.raises(lgp.LegionPrepError):
        W.ctx.gather_features_static(torch.full((4,), W.V, dtype=torch.int32, device="cuda"), None, out)
        W.ctx.check()
    torch.cuda.synchronize()
    assert (out == 0).all()
