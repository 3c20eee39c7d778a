"""Pins for the oracle's neighbour sampler: brute force on tiny graphs, uniformity
(chi-square against the closed-form inclusion / subset probabilities), the
degenerate case fanout >= max degree (equals plain BFS expansion) and an
independent Python model of the subset algorithm."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

import datagen
from test_oracle_philox import py_philox4x32_10, M32


def adjacency(indptr, indices, v):
    return indices[indptr[v]:indptr[v + 1]]


def py_sample_row(indptr, indices, v, hop, f, seed):
    """Floyd's subset algorithm with the big-integer Philox model."""
    s, d = int(indptr[v]), int(indptr[v + 1] - indptr[v])
    if d <= f:
        return [int(x) for x in indices[s:s + d]] + [-1] * (f - d), d
    pos = []
    for i in range(f):
        j = d - f + i
        o = py_philox4x32_10([v & M32, v >> 32, hop, i], [seed & M32, seed >> 32])
        t = ((o[0] | (o[1] << 32)) * (j + 1)) >> 64
        pos.append(j if t in pos else t)
    return [int(indices[s + p]) for p in pos], f


@pytest.mark.parametrize("gseed", [1, 2, 3])
def test_bruteforce_invariants_tiny(oracle_mod, gseed):
    indptr, indices = datagen.tiny_graph(60, 6.0, gseed)
    orc = oracle_mod.Oracle(indptr, indices)
    for v in range(60):
        adj = set(int(x) for x in adjacency(indptr, indices, v))
        d = len(adj)
        for f in (1, 3, 5, 8, 64):
            for seed in (0, 1, 2**40 + 5):
                out, cnt = orc.sample_row(v, 1, f, seed)
                valid = [int(x) for x in out if x >= 0]
                assert cnt == min(d, f) == len(valid)
                assert all(x >= 0 for x in out[:cnt]) and all(x == -1 for x in out[cnt:])
                assert set(valid) <= adj                      # every sample is a real out-edge
                assert len(set(valid)) == len(valid)          # without replacement
                if d <= f:                                    # small rows come back whole, in CSR order
                    assert valid == [int(x) for x in adjacency(indptr, indices, v)]
                assert (out.tolist(), cnt) == py_sample_row(indptr, indices, v, 1, f, seed)


def test_isolated_vertex(oracle_mod):
    indptr = np.array([0, 0, 2, 2], dtype=np.int32)
    indices = np.array([0, 2], dtype=np.int32)
    orc = oracle_mod.Oracle(indptr, indices)
    out, cnt = orc.sample_row(0, 0, 4, 9)
    assert cnt == 0 and out.tolist() == [-1] * 4
    b = orc.sample_khop(np.array([0], np.int32), [3, 3], 1)
    assert b.cnt[0].tolist() == [0] and b.frontier[1].size == 0 and b.gather_ids.tolist() == [0]


def _fan_graph(n_src, d):
    """n_src source vertices, each with the same d out-neighbours n_src .. n_src+d-1."""
    indptr = np.concatenate([np.arange(n_src + 1) * d, np.full(d, n_src * d)]).astype(np.int64)
    indices = np.tile(np.arange(n_src, n_src + d, dtype=np.int32), n_src)
    return indptr, indices


@pytest.mark.parametrize("d,f", [(5, 2), (7, 3), (6, 5)])
def test_uniform_over_subsets(oracle_mod, d, f):
    n = 120_000
    indptr, indices = _fan_graph(n, d)
    orc = oracle_mod.Oracle(indptr, indices)
    b = orc.sample_khop(np.arange(n, dtype=np.int32), [f], 12345)
    rows = np.sort(b.nbr[0] - n, axis=1)
    assert (b.cnt[0] == f).all()
    subsets = {s: k for k, s in enumerate(itertools.combinations(range(d), f))}
    counts = np.zeros(len(subsets))
    for key, c in zip(*np.unique(rows, axis=0, return_counts=True)):
        counts[subsets[tuple(int(x) for x in key)]] = c
    assert counts.sum() == n and (counts > 0).all()
    assert len(subsets) == math.comb(d, f)
    assert stats.chisquare(counts).pvalue > 1e-3              # each f-subset has probability 1 / C(d, f)


@pytest.mark.parametrize("d,f", [(30, 10), (100, 15), (1000, 25)])
def test_inclusion_probability(oracle_mod, d, f):
    n = 60_000
    indptr, indices = _fan_graph(n, d)
    orc = oracle_mod.Oracle(indptr, indices)
    b = orc.sample_khop(np.arange(n, dtype=np.int32), [f], 99)
    counts = np.bincount((b.nbr[0] - n).ravel(), minlength=d).astype(float)
    p = f / d
    z = (counts - n * p) / math.sqrt(n * p * (1 - p))
    assert np.abs(z).max() < 4.5                              # every neighbour is included with probability f / d
    assert abs(z.mean()) < 1e-9 or counts.sum() == n * f


def test_hop_index_changes_the_draw(oracle_mod):
    indptr, indices = _fan_graph(50, 40)
    orc = oracle_mod.Oracle(indptr, indices)
    a = [orc.sample_row(v, 0, 5, 3)[0].tolist() for v in range(50)]
    b = [orc.sample_row(v, 1, 5, 3)[0].tolist() for v in range(50)]
    assert a != b


def test_full_fanout_equals_bfs(oracle_mod):
    indptr, indices = datagen.tiny_graph(300, 3.0, 5, max_degree=8)
    orc = oracle_mod.Oracle(indptr, indices)
    seeds = np.array([4, 250, 17, 99], dtype=np.int32)
    b = orc.sample_khop(seeds, [8, 8, 8], 77)
    level = [int(s) for s in seeds]
    seen = set(level)
    for h in range(3):
        assert b.frontier[h].tolist() == level
        nxt = set()
        for i, v in enumerate(level):
            adj = [int(x) for x in adjacency(indptr, indices, v)]
            assert b.nbr[h][i, :len(adj)].tolist() == adj and b.cnt[h][i] == len(adj)
            nxt |= set(adj)
        seen |= nxt
        level = sorted(nxt)
    assert b.gather_ids.tolist() == sorted(seen)


def test_frontier_and_gather_set_semantics(oracle_mod):
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    orc = oracle_mod.Oracle(indptr, indices)
    seeds = datagen.make_tablet(spec)[:256]
    b = orc.sample_khop(seeds, [10, 5, 3], 2024)
    allv = set(int(s) for s in seeds)
    for h in range(3):
        valid = b.nbr[h][b.nbr[h] >= 0]
        assert (np.count_nonzero(b.nbr[h] >= 0, axis=1) == b.cnt[h]).all()
        allv |= set(int(x) for x in valid)
        if h + 1 < 3:
            nxt = b.frontier[h + 1]
            assert (np.diff(nxt) > 0).all()                   # strictly ascending = sorted and unique
            assert nxt.tolist() == sorted(set(int(x) for x in valid))
        for i in (0, 7, len(b.frontier[h]) - 1):              # rows are the per-vertex definition
            v = int(b.frontier[h][i])
            assert b.nbr[h][i].tolist() == py_sample_row(indptr, indices, v, h, [10, 5, 3][h], 2024)[0]
    assert b.gather_ids.tolist() == sorted(allv)


def test_seed_order_only_permutes_first_hop(oracle_mod):
    indptr, indices = datagen.make_graph(datagen.TINY)
    orc = oracle_mod.Oracle(indptr, indices)
    seeds = datagen.make_tablet(datagen.TINY)[:200]
    perm = np.random.default_rng(0).permutation(200)
    a = orc.sample_khop(seeds, [10, 5], 5)
    b = orc.sample_khop(seeds[perm], [10, 5], 5)
    assert (b.nbr[0] == a.nbr[0][perm]).all() and (b.cnt[0] == a.cnt[0][perm]).all()
    assert (a.frontier[1] == b.frontier[1]).all() and (a.nbr[1] == b.nbr[1]).all()
    assert (a.gather_ids == b.gather_ids).all()


def test_int64_offsets_give_same_result(oracle_mod):
    indptr, indices = datagen.make_graph(datagen.TINY)
    a = oracle_mod.Oracle(indptr, indices).sample_khop(np.arange(100, dtype=np.int32), [10, 5], 8)
    b = oracle_mod.Oracle(indptr.astype(np.int64), indices).sample_khop(np.arange(100, dtype=np.int32), [10, 5], 8)
    assert all((x == y).all() for x, y in zip(a.nbr + [a.gather_ids], b.nbr + [b.gather_ids]))


def test_hop_order_is_first_reach_order():
    """Extraction order of the intra-batch pipeline: seeds as given, then per hop the vertices that hop reaches for
    the first time, ascending -- rebuilt here from the oracle's own frontiers with Python sets, plus what must hold
    whatever the order: it is a permutation of the ascending extraction set, every vertex sits in the group of the
    first hop whose samples contain it, and a hop that reaches nothing new has an empty group."""
    import oracle
    spec = datagen.TINY
    indptr, indices = datagen.make_graph(spec)
    orc = oracle.Oracle(indptr, indices)
    seeds = datagen.make_tablet(spec)[:300]
    for fanouts in ((10, 5), (3, 3, 3), (25,)):
        b = orc.sample_khop(seeds, fanouts, 99)
        seen, want, seg = set(seeds.tolist()), list(seeds.tolist()), [0, len(seeds)]
        for h in range(1, len(fanouts) + 1):
            new = sorted(set(b.frontier[h].tolist()) - seen)
            want += new
            seen |= set(new)
            seg.append(len(want))
        assert b.hop_order.tolist() == want and b.hop_seg.tolist() == seg
        assert sorted(b.hop_order.tolist()) == b.gather_ids.tolist()          # same set as the ascending list
        first_hop = {}
        for h in range(len(fanouts)):
            for u in b.nbr[h][b.nbr[h] >= 0].tolist():
                first_hop.setdefault(u, h + 1)
        for g in range(1, len(seg) - 1):
            for u in b.hop_order[seg[g]:seg[g + 1]].tolist():
                assert first_hop[u] == g and u not in set(seeds.tolist())
    # hand-worked: path 0 -> 1 -> 2 -> 0 with a chord 0 -> 2; seeds [2, 0]
    ip = np.array([0, 2, 3, 4], dtype=np.int32)
    ix = np.array([1, 2, 2, 0], dtype=np.int32)
    b = oracle.Oracle(ip, ix).sample_khop(np.array([2, 0], dtype=np.int32), (2, 2), 1)
    assert b.frontier[1].tolist() == [0, 1, 2] and b.hop_order.tolist() == [2, 0, 1] and b.hop_seg.tolist() == [0, 2, 3, 3]
    # duplicate seeds stay as given
    b = oracle.Oracle(ip, ix).sample_khop(np.array([1, 1], dtype=np.int32), (1,), 1)
    assert b.hop_order.tolist() == [1, 1, 2] and b.hop_seg.tolist() == [0, 2, 3]
