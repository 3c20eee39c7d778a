"""Pins for the oracle's batch generator: the epoch order is a permutation defined by Philox keys."""
import numpy as np

from test_oracle_philox import py_philox4x32_10, M32


def test_shuffle_is_the_key_sorted_permutation(oracle_mod):
    ids = (np.arange(500, dtype=np.int32) * 7 + 3)
    seed = 2**40 + 17
    for epoch in (0, 1, 5):
        out = oracle_mod.shuffle_tablet(ids, seed, epoch)
        keys = []
        for i in range(ids.size):
            o = py_philox4x32_10([i, 0, epoch, 0], [seed & M32, seed >> 32])
            keys.append((o[0] | (o[1] << 32), i))
        assert out.tolist() == [int(ids[i]) for _, i in sorted(keys)]
        assert sorted(out.tolist()) == ids.tolist()                     # a permutation of the tablet
    a, b = oracle_mod.shuffle_tablet(ids, seed, 0), oracle_mod.shuffle_tablet(ids, seed, 1)
    assert (a != b).any() and (oracle_mod.shuffle_tablet(ids, seed, 0) == a).all()
    assert oracle_mod.shuffle_tablet(ids[:0], seed, 0).size == 0


def test_shuffle_is_close_to_uniform(oracle_mod):
    """Each element lands in each quarter of the output about a quarter of the time."""
    n, reps = 64, 4000
    ids = np.arange(n, dtype=np.int32)
    counts = np.zeros((n, 4))
    for e in range(reps):
        out = oracle_mod.shuffle_tablet(ids, 99, e)
        pos = np.empty(n, dtype=np.int64)
        pos[out] = np.arange(n)
        counts[np.arange(n), pos // 16] += 1
    z = (counts - reps / 4) / np.sqrt(reps * 0.25 * 0.75)
    assert np.abs(z).max() < 4.5
