"""Pins for the oracle's Philox4x32-10 and its uniform slot map."""
import os

import numpy as np

from oracle import philox


def _rows(path):
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        yield [int(x, 16) for x in line.split()]


def test_known_answers(golden_dir):
    n = 0
    for w in _rows(os.path.join(golden_dir, "philox_kat.txt")):
        out = philox.philox4x32_10(w[0:4], w[4:6])
        assert [int(o) for o in out] == w[6:10]
        n += 1
    assert n == 3


def test_uniform_mapping_is_exact_fp32_in_unit_interval():
    u = philox.uniforms(5, 3, 11, seed=0x1234567890ABCDEF, offset=7)
    assert u.shape == (5, 3, 11)
    assert np.all(u >= 0.0) and np.all(u < 1.0)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert np.array_equal(u * 2.0 ** 24, np.round(u * 2.0 ** 24))


def test_slot_map_matches_scalar_calls():
    seed, off = (0xDEADBEEF << 32) | 0x01020304, 9
    u = philox.uniforms(3, 2, 9, seed=seed, offset=off)
    for b in range(3):
        for s in range(2):
            for t in range(9):
                w = philox.philox4x32_10((t // 4, b, s, off), (seed & 0xFFFFFFFF, seed >> 32))
                assert u[b, s, t] == (int(w[t % 4]) >> 8) * 2.0 ** -24


def test_zero_seed_first_words(golden_dir):
    # slot 0..3 of (b=0, s=0, offset=0, seed=0) are the four words of the all-zero KAT
    w = next(_rows(os.path.join(golden_dir, "philox_kat.txt")))[6:10]
    u = philox.uniforms(1, 1, 4, seed=0, offset=0)[0, 0]
    assert [int(x * 2 ** 24) for x in u] == [x >> 8 for x in w]


def test_streams_differ_across_b_s_offset_seed():
    a = philox.uniforms(4, 4, 8, seed=1, offset=0)
    flat = a.reshape(-1)
    assert len(np.unique(flat)) > 0.99 * flat.size
    assert not np.array_equal(a, philox.uniforms(4, 4, 8, seed=2, offset=0))
    assert not np.array_equal(a, philox.uniforms(4, 4, 8, seed=1, offset=1))
    # mean / variance of U(0,1)
    big = philox.uniforms(64, 16, 32, seed=3).reshape(-1)
    assert abs(big.mean() - 0.5) < 0.01 and abs(big.var() - 1 / 12) < 0.01
