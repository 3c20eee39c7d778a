"""Pins for the oracle's Algorithm 1 (CSLP): a direct Python transcription of its three steps
on small matrices, the K_g = 1 special case, and structural invariants."""
import numpy as np
import pytest


def py_cslp(hot):
    k_g, V = hot.shape
    acc = [int(hot[:, v].sum()) for v in range(V)]                         # step 1: column-wise sum
    order = sorted(range(V), key=lambda v: (-acc[v], v))                   # step 2: descending, ties by id
    queues = [[] for _ in range(k_g)]
    owner = [int(np.argmax(hot[:, v])) for v in range(V)]                  # np.argmax: first maximum
    for v in order:                                                        # step 3
        queues[owner[v]].append(v)
    return acc, order, owner, queues


@pytest.mark.parametrize("k_g,V,hi,seed", [(1, 200, 5, 0), (2, 300, 4, 1), (4, 500, 3, 2), (8, 1000, 50, 3), (3, 7, 2, 4)])
def test_matches_direct_transcription(oracle_mod, k_g, V, hi, seed):
    hot = np.random.default_rng(seed).integers(0, hi, size=(k_g, V)).astype(np.uint32)   # many ties
    acc, order, owner, queues, offsets = oracle_mod.cslp(hot)
    racc, rorder, rowner, rqueues = py_cslp(hot)
    assert acc.tolist() == racc and order.tolist() == rorder and owner.tolist() == rowner
    assert offsets[0] == 0 and offsets[-1] == V
    for g in range(k_g):
        assert queues[offsets[g]:offsets[g + 1]].tolist() == rqueues[g]
    assert sorted(queues.tolist()) == list(range(V))                       # every vertex in exactly one queue


def test_single_gpu_reduces_to_plain_ranking(oracle_mod):
    import datagen
    indptr, indices = datagen.tiny_graph(400, 3.0, 1)
    orc = oracle_mod.Oracle(indptr, indices)
    hot = np.random.default_rng(5).integers(0, 9, size=400).astype(np.uint32)
    acc, order, owner, queues, offsets = oracle_mod.cslp(hot[None, :])
    assert (order == orc.rank_by_hotness(hot)).all() and (queues == order).all() and (owner == 0).all()
    assert (acc == hot).all() and offsets.tolist() == [0, 400]


def test_local_preference_and_sums_beyond_32_bits(oracle_mod):
    hot = np.zeros((3, 6), dtype=np.uint32)
    hot[:, 0] = [2**32 - 1, 2**32 - 1, 2**32 - 1]      # column sum needs 34 bits; tie -> GPU 0
    hot[:, 1] = [1, 5, 5]                               # tie between GPUs 1 and 2 -> GPU 1
    hot[:, 2] = [0, 0, 7]
    hot[:, 3] = [9, 0, 0]
    acc, order, owner, queues, offsets = oracle_mod.cslp(hot)
    assert int(acc[0]) == 3 * (2**32 - 1) and order.tolist() == [0, 1, 3, 2, 4, 5]
    assert owner.tolist() == [0, 1, 2, 0, 0, 0]
    assert [queues[offsets[g]:offsets[g + 1]].tolist() for g in range(3)] == [[0, 3, 4, 5], [1], [2]]
