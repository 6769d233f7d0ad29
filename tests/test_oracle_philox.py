"""Pins for oracle.philox: published known-answer vectors (Salmon et al., SC'11)."""
import os
import numpy as np
from oracle import philox


def _vectors(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answers_scalar(golden_dir):
    vecs = _vectors(golden_dir)
    assert len(vecs) == 3
    for ctr, key, out in vecs:
        assert list(philox.philox4x32_10(ctr, key)) == out


def test_known_answers_vectorised(golden_dir):
    for ctr, key, out in _vectors(golden_dir):
        got = philox.philox4x32_10_array(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1])
        assert [int(x) for x in got] == out


def test_vectorised_matches_scalar_on_random_counters():
    rng = np.random.default_rng(5)
    c = rng.integers(0, 2 ** 32, size=(4, 257), dtype=np.uint64)
    k0, k1 = 0x9abcdef0, 0x12345678
    got = philox.philox4x32_10_array(c[0], c[1], c[2], c[3], k0, k1)
    for j in range(c.shape[1]):
        ref = philox.philox4x32_10([int(c[i, j]) for i in range(4)], (k0, k1))
        assert tuple(int(g[j]) for g in got) == ref


def test_bijection_on_counter_low_bits():
    # a counter-based generator is a bijection of the counter for a fixed key:
    # distinct counters give distinct 128-bit blocks
    outs = {philox.philox4x32_10((c, 0, 0, 0), (1, 2)) for c in range(4096)}
    assert len(outs) == 4096
