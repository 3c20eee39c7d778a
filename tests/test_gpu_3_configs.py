"""GPU parity on the three large workloads (configs 3-5).

wide   (config 5): 10 M vertices, ~400 M edges, 2-KiB fp16 rows (20 GB table), feature-cache sweep.
large  (config 3): 111 M vertices, ~1.6 B edges, int64 offsets, 512-byte fp32 rows (57 GB table), all cached.
share  (config 4): 250 M vertices, ~8 B edges, int64 offsets, 256-byte fp16 rows (64 GB table), all cached.
All three run at full size (about 15 s, 25 s and 45 s on the MI355X machine); LGP_SMALL=1 runs large and share at
1/8 of the vertex and edge counts.  The GPU machines pin at most 64 GiB of host memory, so the share workload
(98 GB) keeps its topology in pinned CPU memory and its source feature table in HBM (the library accepts a
device pointer there); the oracle reads a host copy of the same bytes.
Pre-sampling is compared on a bounded number of batches (the same `max_batches` on both sides).  Cache contents
are compared in full whatever their size: the cached column ids and the cached feature rows are read back in
slices of about 1 GB and each slice is compared byte for byte with the oracle's fill of the same rank range.
A share-shaped graph at half size, whose feature table does fit in pinned CPU memory, covers the PCIe miss path
on 256-byte rows.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu
FULL = os.environ.get("LGP_SMALL", "0") != "1"
HOT_BATCHES = 32


def _spec(name):
    spec = datagen.WORKLOADS[name]
    if name in ("large", "share") and not FULL:
        spec = datagen.scaled(spec, 0.125)
    return spec


def _compare_contents(W, qt, n_t, t_indptr, qf, n_f, slice_bytes=1 << 30):
    """Every cached column id and every cached feature row against the oracle, slice by slice.  The oracle fills
    the next slice on a worker thread while this one is read back and compared."""
    row_bytes = W.orc.row_bytes
    jobs = []                                          # (which, first, count, oracle call)
    r = 0
    while r < n_t:                                     # rank ranges holding about slice_bytes of column ids
        r2 = int(np.searchsorted(t_indptr, t_indptr[r] + slice_bytes // 4, side="right")) - 1
        r2 = min(n_t, max(r2, r + 1))
        jobs.append((0, int(t_indptr[r]), int(t_indptr[r2] - t_indptr[r]),
                     lambda a=r, b=r2: W.orc.fill_topo(qt[a:b], b - a)[1]))
        r = r2
    step = max(1, slice_bytes // row_bytes) if row_bytes else 0
    for lo in range(0, n_f, step or 1):
        hi = min(n_f, lo + step)
        jobs.append((1, lo, hi - lo, lambda a=lo, b=hi: W.orc.fill_feat(qf[a:b], b - a)))
    with ThreadPoolExecutor(max_workers=1) as ex:
        pending = ex.submit(jobs[0][3]) if jobs else None
        for k, (which, first, count, _) in enumerate(jobs):
            want = pending.result()
            pending = ex.submit(jobs[k + 1][3]) if k + 1 < len(jobs) else None
            got = W.ctx.get_cache_part(which, first, count)
            assert got.tobytes() == want.tobytes() if count < 1024 else np.array_equal(
                got.reshape(-1).view(np.uint8), want.reshape(-1).view(np.uint8)), \
                f"{W.spec.name}: cache contents differ ({'column ids' if which == 0 else 'feature rows'} from {first})"
            del got, want


def _presample_and_cache(W, topo_b, feat_b, hotness=True):
    spec = W.spec
    if hotness:
        W.ctx.build_hotness(W.tablet_dev, spec.batch, spec.fanouts, spec.base_seed, max_batches=HOT_BATCHES)
        topo, feat = W.ctx.get_hotness()
        rt, rf, nb = W.orc.build_hotness(W.tablet, spec.batch, spec.fanouts, spec.base_seed, max_batches=HOT_BATCHES)
        assert nb == HOT_BATCHES and (topo == rt).all() and (feat == rf).all()
        W.ranking = (W.orc.rank_by_hotness(rt), W.orc.rank_by_hotness(rf))
    qt, qf = W.ranking
    plan = W.ctx.build_cache(topo_b, feat_b)
    n_t, n_f = W.orc.plan_topo(qt, topo_b), W.orc.plan_feat(feat_b)
    assert (plan.n_topo, plan.n_feat) == (n_t, n_f)
    topo_ids, t_indptr, _, feat_ids, _ = W.ctx.get_cache(contents=False)
    assert (topo_ids == qt[:n_t]).all() and (feat_ids == qf[:n_f]).all()
    deg = np.diff(W.indptr)
    assert t_indptr[0] == 0 and (np.diff(t_indptr) == deg[qt[:n_t]]).all()
    assert t_indptr[-1] == plan.topo_edges
    _compare_contents(W, qt, n_t, t_indptr, qf, n_f)
    W.ctx.check()
    return plan, qf


def _check_batch(W, b, rng_seed, qf, n_f):
    from gpu_common import assert_batch_equal
    import paper_2305_16588_amd as lgp
    spec = W.spec
    buf = lgp.SampleBuffers(W.V, spec.batch, spec.fanouts)
    seeds, seeds_dev = W.batch(b)
    W.ctx.sample_khop(seeds_dev, spec.fanouts, rng_seed, out=buf)
    stats = torch.zeros(2, dtype=torch.int32, device="cuda")
    rows = W.ctx.gather_features(buf.gather_ids, n_dev=buf.n_gather, stats=stats)
    ref = W.orc.sample_khop(seeds, spec.fanouts, rng_seed)
    assert_batch_equal(ref, buf.to_host(seeds_dev), f"{spec.name} batch {b}")
    n = ref.gather_ids.size
    assert rows[:n].cpu().numpy().tobytes() == W.orc.gather(ref.gather_ids).tobytes()
    n_hit = W.orc.count_hits(ref.gather_ids, qf, n_f)
    assert stats.tolist() == [n_hit, n - n_hit]
    del rows, buf
    W.ctx.check()
    return n_hit, n


def test_wide_feature_cache_sweep():
    from gpu_common import Workload
    spec = _spec("wide")
    W = Workload(spec, device_gen="cuda")
    print(f"{spec.name}: V={W.V} E={W.E} feature table {W.features.nbytes / 1e9:.1f} GB", flush=True)
    assert W.features.dtype == np.float16 and W.features.shape == (spec.num_vertices, 1024)
    topo_b, _ = datagen.budgets(spec, W.E)
    row = 2048
    last = (W.tablet.size - 1) // spec.batch
    rates = []
    for frac in (0.0, 0.10, 0.25, 0.50, 1.0):
        plan, qf = _presample_and_cache(W, topo_b, int(frac * W.V) * row, hotness=(frac == 0.0))
        assert plan.n_topo == W.V and plan.n_feat == int(frac * W.V)
        n_hit, n = _check_batch(W, 3, spec.base_seed + 500, qf, plan.n_feat)
        rates.append(n_hit / n)
    _check_batch(W, last, spec.base_seed + 501, qf, plan.n_feat)       # short last batch, everything cached
    assert rates[0] == 0.0 and rates[-1] == 1.0 and all(a < b for a, b in zip(rates, rates[1:]))
    # skewed access: the first 10 % of the cache buys more hits than the step from 25 % to 50 %
    assert rates[1] - rates[0] > rates[3] - rates[2]


@pytest.mark.parametrize("name", ["large", "share"])
def test_everything_cached_int64_offsets(name):
    from gpu_common import Workload
    spec = _spec(name)
    W = Workload(spec, device_gen="cuda", features_on_device=(FULL and name == "share"))
    print(f"{spec.name}: V={W.V} E={W.E} feature table {W.features.nbytes / 1e9:.1f} GB", flush=True)
    assert W.indptr.dtype == np.int64
    topo_b, feat_b = datagen.budgets(spec, W.E)
    plan, qf = _presample_and_cache(W, topo_b, feat_b)
    assert plan.n_topo == W.V and plan.n_feat == W.V                    # the HBM budget holds the whole graph
    last = (W.tablet.size - 1) // spec.batch
    for b, s in ((0, 11), (last, 12)):
        n_hit, n = _check_batch(W, b, spec.base_seed + s, qf, plan.n_feat)
        assert n_hit == n
    # a constrained plan at the same shape: misses over PCIe, topology partly in CPU memory
    plan, qf = _presample_and_cache(W, topo_b // 4, (W.V // 8) * W.orc.row_bytes, hotness=False)
    n_hit, n = _check_batch(W, 1, spec.base_seed + 13, qf, plan.n_feat)
    assert 0 < n_hit < n


def test_share_shaped_misses_over_pcie():
    """The share workload's shape (int64 offsets, 256-byte fp16 rows, fan-outs 25 / 10) at half its size, so that
    graph and feature table both fit in pinned CPU memory: misses are read in place over PCIe."""
    from gpu_common import Workload
    spec = datagen.scaled(datagen.WORKLOADS["share"], 0.5 if FULL else 0.0625, name="share-half")
    W = Workload(spec, device_gen="cuda")
    print(f"{spec.name}: V={W.V} E={W.E} feature table {W.features.nbytes / 1e9:.1f} GB in pinned memory", flush=True)
    assert W.features_dev is None and W.orc.row_bytes == 256
    topo_b, feat_b = datagen.budgets(spec, W.E)
    plan, qf = _presample_and_cache(W, topo_b // 4, (W.V // 8) * 256)
    assert 0 < plan.n_topo < W.V and plan.n_feat == W.V // 8
    last = (W.tablet.size - 1) // spec.batch
    for b, s in ((0, 21), (last, 22)):
        n_hit, n = _check_batch(W, b, spec.base_seed + s, qf, plan.n_feat)
        assert 0 < n_hit < n
    plan, qf = _presample_and_cache(W, 0, 0, hotness=False)             # nothing cached: every row over PCIe
    n_hit, n = _check_batch(W, 2, spec.base_seed + 23, qf, 0)
    assert n_hit == 0
