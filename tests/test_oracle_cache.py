"""Pins for the oracle's hotness counting (Sec. 4.2.2 S1), ranking (Algorithm 1 with
one GPU), budget-to-prefix rules (Eq. 3, Eq. 6), cache fill and feature gather."""
from collections import Counter

import numpy as np
import pytest

import datagen


@pytest.fixture(scope="module")
def tiny(oracle_mod):
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    feats = datagen.make_features(spec)
    return spec, indptr, indices, feats, oracle_mod.Oracle(indptr, indices, feats)


def test_hotness_equals_bruteforce_recount(tiny):
    spec, indptr, indices, feats, orc = tiny
    tablet = datagen.make_tablet(spec)[:2500]                  # 2 full batches + a short one
    topo, feat, nb = orc.build_hotness(tablet, 1024, spec.fanouts, 4001)
    assert nb == 3
    ct, cf = Counter(), Counter()
    edges = rows = 0
    for b in range(3):
        res = orc.sample_khop(tablet[b * 1024:(b + 1) * 1024], spec.fanouts, 4001 + b)
        for h in range(len(spec.fanouts)):
            for v, row in zip(res.frontier[h], res.nbr[h]):
                ct[int(v)] += int((row >= 0).sum())            # one per traversed edge, at its source
        for u in res.gather_ids:
            cf[int(u)] += 1                                    # one per vertex per mini-batch
        edges += sum(int(c.sum()) for c in res.cnt)
        rows += res.gather_ids.size
    assert {v: int(c) for v, c in enumerate(topo) if c} == {v: c for v, c in ct.items() if c}
    assert {v: int(c) for v, c in enumerate(feat) if c} == dict(cf)
    assert int(topo.sum()) == edges and int(feat.sum()) == rows


def test_hotness_closed_form_when_nothing_is_random(oracle_mod):
    """fanout >= max degree: sampling is plain BFS, so hotness has a closed form."""
    indptr, indices = datagen.tiny_graph(200, 2.5, 9, max_degree=6)
    orc = oracle_mod.Oracle(indptr, indices)
    tablet = np.random.default_rng(1).permutation(200).astype(np.int32)[:90]
    topo, feat, nb = orc.build_hotness(tablet, 40, [6, 6], 0)
    assert nb == 3
    et, ef = np.zeros(200, np.int64), np.zeros(200, np.int64)
    deg = np.diff(indptr)
    for lo in (0, 40, 80):
        level = [int(x) for x in tablet[lo:lo + 40]]
        seen = set(level)
        for _ in range(2):
            nxt = set()
            for v in level:
                et[v] += deg[v]
                nxt |= set(int(x) for x in indices[indptr[v]:indptr[v + 1]])
            seen |= nxt
            level = sorted(nxt)
        for u in seen:
            ef[u] += 1
    assert (topo == et).all() and (feat == ef).all()


def test_max_batches_limits_presampling(tiny):
    spec, *_ , orc = tiny
    tablet = datagen.make_tablet(spec)
    t1, f1, nb = orc.build_hotness(tablet, 1024, spec.fanouts, 7, max_batches=2)
    t2, f2, _ = orc.build_hotness(tablet[:2048], 1024, spec.fanouts, 7)
    assert nb == 2 and (t1 == t2).all() and (f1 == f2).all()
    assert orc.build_hotness(tablet, 1024, spec.fanouts, 7)[2] == 10


def test_rank_is_descending_hotness_then_ascending_id(tiny):
    spec, *_ , orc = tiny
    rng = np.random.default_rng(3)
    hot = rng.integers(0, 6, size=orc.V).astype(np.uint32)     # many ties
    order = orc.rank_by_hotness(hot)
    assert order.tolist() == sorted(range(orc.V), key=lambda v: (-int(hot[v]), v))


def test_topk_selection_property_quadratic(oracle_mod):
    indptr, indices = datagen.tiny_graph(80, 4.0, 2)
    feats = np.arange(80 * 3, dtype=np.float32).reshape(80, 3)
    orc = oracle_mod.Oracle(indptr, indices, feats)
    hot = np.random.default_rng(5).integers(0, 4, size=80).astype(np.uint32)
    order = orc.rank_by_hotness(hot)
    for n in (0, 1, 17, 80):
        cached = set(int(x) for x in order[:n])
        for c in cached:
            for o in range(80):
                if o not in cached:                            # nothing outside is hotter; ties go to the smaller id
                    assert hot[o] < hot[c] or (hot[o] == hot[c] and o > c)


def test_topology_budget_prefix_rule(tiny):
    spec, indptr, indices, feats, orc = tiny
    topo, _, _ = orc.build_hotness(datagen.make_tablet(spec), 1024, spec.fanouts, 1)
    order = orc.rank_by_hotness(topo)
    cost = (np.diff(indptr)[order].astype(np.int64) * 4 + 8)   # Eq. 3 per-vertex cost
    csum = np.cumsum(cost)
    total = int(csum[-1])
    assert total == 4 * indices.size + 8 * orc.V
    for budget in (0, 7, 8, int(cost[0]), int(cost[0]) - 1, total // 5, total // 2, total - 1, total, total + 100):
        n = orc.plan_topo(order, budget)
        used = int(csum[n - 1]) if n else 0
        assert used <= budget
        assert n == orc.V or used + int(cost[n]) > budget
    assert orc.plan_topo(order, 0) == 0 and orc.plan_topo(order, total) == orc.V


def test_feature_budget_rule(tiny):
    spec, indptr, indices, feats, orc = tiny
    rb = orc.row_bytes
    assert rb == 512
    for budget in (0, 511, 512, 513, 2000 * 512, orc.V * 512 - 1, orc.V * 512, 10**12):
        assert orc.plan_feat(budget) == min(orc.V, budget // rb)


def test_cache_fill_copies_ranked_rows(tiny):
    spec, indptr, indices, feats, orc = tiny
    topo, feat, _ = orc.build_hotness(datagen.make_tablet(spec), 1024, spec.fanouts, 1)
    qt, qf = orc.rank_by_hotness(topo), orc.rank_by_hotness(feat)
    n = 1234
    t_indptr, t_indices = orc.fill_topo(qt, n)
    assert t_indptr[0] == 0 and (np.diff(t_indptr) == np.diff(indptr)[qt[:n]]).all()
    for r in (0, 1, 500, n - 1):
        v = qt[r]
        assert (t_indices[t_indptr[r]:t_indptr[r + 1]] == indices[indptr[v]:indptr[v + 1]]).all()
    assert t_indices.size == t_indptr[-1]
    fc = orc.fill_feat(qf, n)
    assert fc.tobytes() == feats[qf[:n]].tobytes()
    assert orc.fill_feat(qf, 0).shape == (0, spec.feat_dim)


def test_gather_is_fancy_indexing(tiny):
    spec, indptr, indices, feats, orc = tiny
    ids = np.random.default_rng(8).integers(0, orc.V, size=5000).astype(np.int32)   # duplicates, any order
    assert orc.gather(ids).tobytes() == feats[ids].tobytes()
    assert orc.gather(ids[:0]).shape == (0, spec.feat_dim)
    order = orc.rank_by_hotness(np.random.default_rng(9).integers(0, 50, size=orc.V).astype(np.uint32))
    for n in (0, 2000, orc.V):
        assert orc.count_hits(ids, order, n) == int(np.isin(ids, order[:n]).sum())


def test_gather_fp16_rows(oracle_mod):
    feats = np.random.default_rng(0).standard_normal((50, 7)).astype(np.float16)
    indptr = np.zeros(51, np.int32)
    orc = oracle_mod.Oracle(indptr, np.empty(0, np.int32), feats)
    ids = np.array([3, 3, 49, 0], np.int32)
    assert orc.row_bytes == 14 and orc.gather(ids).tobytes() == feats[ids].tobytes()
