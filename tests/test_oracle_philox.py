"""Pins for the oracle's Philox4x32-10 and its (seed, vertex, hop, slot) keying."""
import os
import random

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
M32 = 0xFFFFFFFF


def py_philox4x32_10(ctr, key):
    """Independent big-integer evaluation of the round function (Salmon et al., SC'11)."""
    c = [int(x) for x in ctr]
    k = [int(x) for x in key]
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M32, (p0 >> 32) ^ c[3] ^ k[1], p0 & M32]
    return c


def test_known_answer_vectors(oracle_mod):
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for w in rows:
        words = [int(x, 16) for x in w]
        out = oracle_mod.philox4x32_10(words[0:4], words[4:6])
        assert [int(x) for x in out] == words[6:10]
        assert py_philox4x32_10(words[0:4], words[4:6]) == words[6:10]


def test_against_bigint_model_random_inputs(oracle_mod):
    rnd = random.Random(7)
    for _ in range(300):
        ctr = [rnd.getrandbits(32) for _ in range(4)]
        key = [rnd.getrandbits(32) for _ in range(2)]
        assert [int(x) for x in oracle_mod.philox4x32_10(ctr, key)] == py_philox4x32_10(ctr, key)


def test_draw_keying(oracle_mod):
    """counter = (v low, v high, hop, slot); key = (seed low, seed high); draw = word0 | word1 << 32."""
    rnd = random.Random(11)
    for _ in range(200):
        seed = rnd.getrandbits(64)
        v = rnd.getrandbits(rnd.choice([8, 20, 31, 40]))
        hop, slot = rnd.randrange(8), rnd.randrange(64)
        out = py_philox4x32_10([v & M32, v >> 32, hop, slot], [seed & M32, seed >> 32])
        assert oracle_mod.draw64(seed, v, hop, slot) == out[0] | (out[1] << 32)


def test_each_key_component_matters(oracle_mod):
    base = oracle_mod.draw64(5, 6, 1, 2)
    assert len({base, oracle_mod.draw64(6, 6, 1, 2), oracle_mod.draw64(5, 7, 1, 2), oracle_mod.draw64(5, 6, 2, 2),
                oracle_mod.draw64(5, 6, 1, 3), oracle_mod.draw64(5 + (1 << 32), 6, 1, 2)}) == 6
