"""Pins for the oracle's clique cache plan (Sec. 4.2.2: Algorithm 1's queues drive each GPU's fill-up)
and its three-way count (own cache / peer's cache / CPU memory): brute force with Python sets on small
graphs, the K_g = 1 case that reduces to the single-GPU plan, and hand-made examples."""
import numpy as np
import pytest

import datagen


def small(oracle_mod, V=600, seed=3, dim=6):
    indptr, indices = datagen.tiny_graph(V, 4.0, seed)
    feats = np.random.default_rng(seed).standard_normal((V, dim)).astype(np.float32)
    return oracle_mod.Oracle(indptr, indices, feats), indptr


def hot_matrix(k_g, V, seed, hi=6):
    return np.random.default_rng(seed).integers(0, hi, size=(k_g, V)).astype(np.uint32)


@pytest.mark.parametrize("k_g,tb,fb", [(2, 900, 24 * 40), (4, 300, 24 * 11 + 5), (8, 64, 23), (3, 10**9, 10**9), (2, 0, 0)])
def test_brute_force(oracle_mod, k_g, tb, fb):
    orc, indptr = small(oracle_mod)
    V = indptr.size - 1
    HT, HF = hot_matrix(k_g, V, 10 + k_g), hot_matrix(k_g, V, 20 + k_g)
    topo_ids, feat_ids = orc.clique_plan(HT, HF, tb, fb)
    assert len(topo_ids) == k_g and len(feat_ids) == k_g
    for H, ids, is_topo in ((HT, topo_ids, True), (HF, feat_ids, False)):
        acc = H.astype(np.int64).sum(axis=0)
        owner = np.argmax(H, axis=0)                                   # first maximum = lowest GPU index
        seen = set()
        for g in range(k_g):
            mine = [v for v in sorted(range(V), key=lambda v: (-acc[v], v)) if owner[v] == g]
            got = ids[g].tolist()
            assert got == mine[:len(got)]                              # a prefix of the GPU's own queue
            cost = (lambda v: int(indptr[v + 1] - indptr[v]) * 4 + 8) if is_topo else (lambda v: 24)
            used = sum(cost(v) for v in got)
            budget = tb if is_topo else fb
            assert used <= budget
            if len(got) < len(mine):
                assert used + cost(mine[len(got)]) > budget            # and the longest one that fits
            assert not (seen & set(got))                               # no vertex cached twice in the clique
            seen |= set(got)


def test_single_gpu_reduces_to_the_plain_plan(oracle_mod):
    orc, indptr = small(oracle_mod)
    V = indptr.size - 1
    ht, hf = hot_matrix(1, V, 1), hot_matrix(1, V, 2)
    for tb, fb in ((0, 0), (777, 24 * 100 + 3), (10**9, 10**9)):
        topo_ids, feat_ids = orc.clique_plan(ht, hf, tb, fb)
        ot, of = orc.rank_by_hotness(ht[0]), orc.rank_by_hotness(hf[0])
        assert topo_ids[0].tolist() == ot[:orc.plan_topo(ot, tb)].tolist()
        assert feat_ids[0].tolist() == of[:orc.plan_feat(fb)].tolist()


def test_hand_made_example(oracle_mod):
    # path graph 0 -> 1 -> 2 -> 3 -> 4 plus hub 5 -> {0..4}; degrees 1,1,1,1,0,5; 4-byte feature rows
    indptr = np.array([0, 1, 2, 3, 4, 4, 9], dtype=np.int32)
    indices = np.array([1, 2, 3, 4, 0, 1, 2, 3, 4], dtype=np.int32)
    feats = np.arange(6, dtype=np.float32)[:, None]
    orc = oracle_mod.Oracle(indptr, indices, feats)
    H = np.array([[9, 0, 3, 1, 0, 4],
                  [1, 8, 3, 0, 0, 5]], dtype=np.uint32)
    # column sums 10 8 6 1 0 9 -> order 0 5 1 2 3 4; owners 0 1 0 0 0 1 -> queues [0 2 3 4], [5 1]
    topo_ids, feat_ids = orc.clique_plan(H, H, 24, 9)
    # topology cost per row: 12 12 12 12 8 28; budget 24: GPU 0 takes 0, 2 (24 bytes); GPU 1's first row (28) does not fit
    assert [t.tolist() for t in topo_ids] == [[0, 2], []]
    # feature rows are 4 bytes, budget 9 -> two rows per GPU
    assert [f.tolist() for f in feat_ids] == [[0, 2], [5, 1]]
    ids = np.array([0, 1, 2, 3, 4, 5, 5, 0], dtype=np.int32)
    assert orc.count_three_way(ids, feat_ids, 0) == (3, 2, 3)           # own: 0 2 0; peer: 1 5 5; CPU: 3 4
    assert orc.count_three_way(ids, feat_ids, 1) == (3, 2, 3)           # own: 1 5 5; peer: 0 2 0
    assert orc.count_three_way(ids[:0], feat_ids, 1) == (0, 0, 0)


@pytest.mark.parametrize("k_g", [2, 4, 8])
def test_three_way_counts_brute_force(oracle_mod, k_g):
    orc, indptr = small(oracle_mod)
    V = indptr.size - 1
    _, feat_ids = orc.clique_plan(hot_matrix(k_g, V, 5), hot_matrix(k_g, V, 6), 100, 24 * 30)
    ids = np.random.default_rng(k_g).integers(0, V, size=2000).astype(np.int32)      # duplicates on purpose
    sets = [set(f.tolist()) for f in feat_ids]
    for g in range(k_g):
        local = sum(1 for i in ids.tolist() if i in sets[g])
        anywhere = sum(1 for i in ids.tolist() if any(i in s for s in sets))
        assert orc.count_three_way(ids, feat_ids, g) == (local, ids.size - anywhere, anywhere - local)
