"""Pins for the oracle's cost model and alpha search (Sec. 4.3, Eq. 2-8): an independent
evaluation of the paper's formulas with Python fractions, plus closed-form corner cases."""
from fractions import Fraction

import numpy as np
import pytest

import datagen


@pytest.fixture(scope="module")
def setup(oracle_mod):
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    feats = datagen.make_features(spec)
    orc = oracle_mod.Oracle(indptr, indices, feats)
    topo, feat, _ = orc.build_hotness(datagen.make_tablet(spec), 1024, spec.fanouts, 1)
    return orc, indptr, topo, feat, orc.rank_by_hotness(topo), orc.rank_by_hotness(feat)


def paper_formulas(indptr, topo, feat, qt, qf, row_bytes, B, n_tsum, cls, n_alpha):
    """Eq. 2-8 evaluated literally, one alpha at a time, in exact rational arithmetic."""
    deg = np.diff(indptr)
    out = []
    all_t, all_f = int(topo.sum()), int(feat.sum())
    for i in range(n_alpha):
        alpha = Fraction(i, n_alpha - 1)
        m_t = int(B * alpha)                                   # floor
        m_f = B - m_t
        used, n_t = 0, 0
        for v in qt:                                           # Eq. 3
            c = int(deg[v]) * 4 + 8
            if used + c > m_t:
                break
            used += c
            n_t += 1
        n_f = min(len(qf), m_f // row_bytes)                   # Eq. 6
        r_t = Fraction(int(topo[qt[:n_t]].sum()), all_t) if all_t else Fraction(1)   # Eq. 4
        n_T = n_tsum * (1 - r_t)                               # Eq. 5
        u_f = all_f - int(feat[qf[:n_f]].sum())                # Eq. 7
        n_F = -(-row_bytes // cls) * u_f                       # Eq. 8
        out.append((m_t, n_t, n_f, n_T + n_F))                 # Eq. 2
    return out


@pytest.mark.parametrize("B,n_tsum,n_alpha", [(600_000, 3_000_000, 101), (2_000_000, 50_000, 11), (50_000, 10**9, 21),
                                              (0, 5, 5), (10**9, 123, 101)])
def test_alpha_search_matches_the_formulas(setup, B, n_tsum, n_alpha):
    orc, indptr, topo, feat, qt, qf = setup
    best, pts = orc.search_cache_plan(topo, feat, qt, qf, B, n_tsum, 64, n_alpha)
    ref = paper_formulas(indptr, topo, feat, qt, qf, orc.row_bytes, B, n_tsum, 64, n_alpha)
    all_t, all_f = int(topo.sum()), int(feat.sum())
    totals = []
    for i, (m_t, n_t, n_f, n_total) in enumerate(ref):
        assert (int(pts["m_topo"][i]), int(pts["m_feat"][i])) == (m_t, B - m_t)
        assert (int(pts["n_topo"][i]), int(pts["n_feat"][i])) == (n_t, n_f)
        mine = Fraction(n_tsum * int(pts["uncached_topo_hot"][i]), all_t) + 8 * int(pts["uncached_feat_hot"][i])
        assert mine == n_total                                  # 512-byte rows, CLS 64 -> 8 transactions per row (Eq. 8)
        totals.append(n_total)
    assert best == totals.index(min(totals))                    # smallest N_total, first one on ties
    assert all(a >= b for a, b in zip(pts["uncached_topo_hot"], pts["uncached_topo_hot"][1:]))   # N_T falls with alpha
    assert all(a <= b for a, b in zip(pts["uncached_feat_hot"], pts["uncached_feat_hot"][1:]))   # N_F rises with alpha


def test_corner_cases(setup):
    orc, indptr, topo, feat, qt, qf = setup
    # no topology traffic measured: every byte should go to features
    best, pts = orc.search_cache_plan(topo, feat, qt, qf, 1_000_000, 0, 64, 101)
    assert best == 0 and pts["n_topo"][0] == 0
    # features never touched: every byte should go to topology (first alpha that caches all the hot rows wins)
    zero = np.zeros_like(feat)
    best, pts = orc.search_cache_plan(topo, zero, qt, qf, 300_000, 10**6, 64, 101)
    assert pts["uncached_topo_hot"][best] == pts["uncached_topo_hot"].min() and (pts["uncached_feat_hot"] == 0).all()
    assert best == int(np.argmin(pts["uncached_topo_hot"]))
    # a budget that holds everything twice over: some alpha reaches zero traffic
    best, pts = orc.search_cache_plan(topo, feat, qt, qf, 10**10, 10**6, 64, 101)
    assert pts["uncached_topo_hot"][best] == 0 and pts["uncached_feat_hot"][best] == 0
    # granularity of Eq. 8: 512-byte rows cost 8 transactions at CLS 64 and 4 at CLS 128; the split can move
    b64, _ = orc.search_cache_plan(topo, feat, qt, qf, 600_000, 3_000_000, 64, 101)
    b128, _ = orc.search_cache_plan(topo, feat, qt, qf, 600_000, 3_000_000, 128, 101)
    assert b128 >= b64                                          # cheaper feature rows -> never less topology


def test_row_width_that_is_not_a_multiple_of_the_transfer_size(oracle_mod, setup):
    """400-byte rows at CLS 64 cost ceil(400 / 64) = 7 transactions each (Eq. 8), not 6.25 or 6."""
    _, indptr, topo, feat, qt, qf = setup
    spec = datagen.TINY
    _, indices = datagen.make_graph(spec)
    feats = np.zeros((spec.num_vertices, 100), dtype=np.float32)
    orc = oracle_mod.Oracle(indptr, indices, feats)
    for B, n_tsum in ((600_000, 3_000_000), (400_000, 100_000), (1_000_000, 100_000)):   # last two: 6 vs 7 moves alpha
        best, pts = orc.search_cache_plan(topo, feat, qt, qf, B, n_tsum, 64, 101)
        ref = paper_formulas(indptr, topo, feat, qt, qf, 400, B, n_tsum, 64, 101)
        totals = [r[3] for r in ref]
        all_t = int(topo.sum())
        for i, r in enumerate(ref):
            assert (int(pts["n_topo"][i]), int(pts["n_feat"][i])) == (r[1], r[2])
            assert Fraction(n_tsum * int(pts["uncached_topo_hot"][i]), all_t) + 7 * int(pts["uncached_feat_hot"][i]) == r[3]
        assert best == totals.index(min(totals))
