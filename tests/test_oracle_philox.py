"""Pins for the oracle's Philox generator (CPU only)."""
import os

import numpy as np

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], tuple(w[6:10])))
    return rows


def test_generic_matches_published_known_answers():
    rows = _kat()
    assert len(rows) >= 3
    for ctr, key, out in rows:
        assert philox.philox4_generic(ctr, key, 32, 10) == out


def test_vectorised_matches_published_known_answers():
    for ctr, key, out in _kat():
        got = philox.philox4x32_10(*ctr, *key)
        assert tuple(int(g) for g in got) == out


def test_generic_at_64_bits_matches_numpy_philox():
    # NumPy's Philox is an independent Philox-4x64-10; it bumps the counter
    # before producing its first block.
    rng = np.random.default_rng(7)
    for _ in range(20):
        ctr = [int(v) for v in rng.integers(0, 2 ** 62, size=4)]
        key = [int(v) for v in rng.integers(0, 2 ** 62, size=2)]
        bg = np.random.Philox(counter=np.array(ctr, dtype=np.uint64),
                              key=np.array(key, dtype=np.uint64))
        raw = [int(r) for r in bg.random_raw(4)]
        bumped = [ctr[0] + 1] + ctr[1:]
        assert list(philox.philox4_generic(bumped, key, 64, 10)) == raw


def test_vectorised_matches_generic_on_random_counters():
    rng = np.random.default_rng(3)
    n = 2000
    c = rng.integers(0, 2 ** 32, size=(4, n), dtype=np.uint64)
    k = rng.integers(0, 2 ** 32, size=(2, n), dtype=np.uint64)
    got = philox.philox4x32_10(c[0], c[1], c[2], c[3], k[0], k[1])
    for j in range(n):
        ref = philox.philox4_generic([int(c[i, j]) for i in range(4)],
                                     [int(k[i, j]) for i in range(2)], 32, 10)
        assert tuple(int(got[i][j]) for i in range(4)) == ref


def test_unit_interval_mapping():
    u = philox.u32_to_unit(np.array([0, 0xFF, 0x100, 0xFFFFFFFF], dtype=np.uint32))
    assert u[0] == 0.5 * 2.0 ** -24 and u[1] == u[0]
    assert u[2] == 1.5 * 2.0 ** -24
    assert u[3] == 1.0 - 0.5 * 2.0 ** -24
    assert np.all((u > 0) & (u < 1))


def test_sv_uniform_layout_and_statistics():
    # counter = (i, b, stream, step), key = (seed lo, seed hi); word 0 / word 1
    seed = (0x12345678 << 32) | 0x9ABCDEF0
    u, up = philox.sv_uniforms(seed, 5, 3, 2)
    w = philox.philox4_generic([2, 3, 0, 5], [0x9ABCDEF0, 0x12345678], 32, 10)
    assert float(u) == ((w[0] >> 8) + 0.5) * 2.0 ** -24
    assert float(up) == ((w[1] >> 8) + 0.5) * 2.0 ** -24
    b, i = np.meshgrid(np.arange(512), np.arange(64), indexing="ij")
    u, up = philox.sv_uniforms(0, 0, b, i)
    for a in (u, up):
        assert abs(a.mean() - 0.5) < 0.01
        assert abs(a.var() - 1.0 / 12.0) < 0.005
    assert abs(np.corrcoef(u.ravel(), up.ravel())[0, 1]) < 0.02
