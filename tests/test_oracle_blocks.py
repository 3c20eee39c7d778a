"""Pins for the oracle's graph constructor (Sec. 5): the blocks must reproduce the sampled edges
exactly when mapped back through the frontiers, and feat_row must index gather_ids."""
import numpy as np

import datagen


def test_blocks_reconstruct_the_sampled_edges(oracle_mod):
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    orc = oracle_mod.Oracle(indptr, indices)
    seeds = datagen.make_tablet(spec)[:300]
    fanouts = (10, 5, 3)
    b = orc.sample_khop(seeds, fanouts, 77, blocks=True)
    assert len(b.frontier) == 4 and len(b.blk_indptr) == 3 and len(b.feat_row) == 4
    for h, f in enumerate(fanouts):
        n = b.frontier[h].size
        assert b.blk_indptr[h][0] == 0 and (np.diff(b.blk_indptr[h]) == b.cnt[h]).all()      # CSR over destinations
        assert b.blk_src[h].size == b.blk_indptr[h][-1]
        src_set = b.frontier[h + 1]
        assert (np.diff(src_set) > 0).all()
        valid = b.nbr[h][b.nbr[h] >= 0]                                                     # row-major = edge order
        assert (src_set[b.blk_src[h]] == valid).all()                                       # maps back to global ids
        assert sorted(set(valid.tolist())) == src_set.tolist()                              # sources = exactly the samples
        for i in (0, n // 2, n - 1):
            lo, hi = b.blk_indptr[h][i], b.blk_indptr[h][i + 1]
            assert (src_set[b.blk_src[h][lo:hi]] == b.nbr[h][i, :b.cnt[h][i]]).all()
    for h in range(4):
        assert (b.gather_ids[b.feat_row[h]] == b.frontier[h]).all()                         # rows of the feature matrix


def test_blocks_with_empty_rows_and_empty_frontier(oracle_mod):
    indptr = np.array([0, 0, 2, 2, 3], dtype=np.int32)
    indices = np.array([0, 2, 1], dtype=np.int32)
    orc = oracle_mod.Oracle(indptr, indices)
    b = orc.sample_khop(np.array([0, 1, 3], np.int32), (2, 2), 5, blocks=True)
    assert b.blk_indptr[0].tolist() == [0, 0, 2, 3] and b.frontier[1].tolist() == [0, 1, 2]
    assert b.blk_src[0].tolist() == [0, 2, 1]
    assert b.blk_indptr[1].tolist() == [0, 0, 2, 2] and b.frontier[2].tolist() == [0, 2]
    assert b.feat_row[0].tolist() == [0, 1, 3] and b.gather_ids.tolist() == [0, 1, 2, 3]
    e = orc.sample_khop(np.array([0], np.int32), (2, 2), 5, blocks=True)
    assert e.frontier[1].size == 0 and e.blk_indptr[1].tolist() == [0] and e.blk_src[1].size == 0
