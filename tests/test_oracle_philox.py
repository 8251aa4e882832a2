"""Pins for oracle/philox.py: published known answers, an independent big-integer
implementation, bijectivity, and the distribution of the derived normals."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import philox


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                rows.append([int(w, 16) for w in line.split()])
    return rows


def philox_bigint(ctr, key):
    """Independent statement of the same public algorithm with Python integers."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) % 2 ** 32, (k[1] + 0xBB67AE85) % 2 ** 32]
        prod0 = 0xD2511F53 * c[0]
        prod1 = 0xCD9E8D57 * c[2]
        c = [(prod1 // 2 ** 32) ^ c[1] ^ k[0], prod1 % 2 ** 32, (prod0 // 2 ** 32) ^ c[3] ^ k[1], prod0 % 2 ** 32]
    return c


def test_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for row in rows:
        got = philox.philox4x32_10(*row[:6])
        assert [int(g) for g in got] == row[6:]
        assert philox_bigint(row[:4], row[4:6]) == row[6:]


def test_matches_bigint_on_random_counters():
    r = np.random.default_rng(0)
    ctr = r.integers(0, 2 ** 32, size=(200, 4), dtype=np.uint64)
    for key in [(0, 0), (123456789, 987654321), (0xFFFFFFFF, 1)]:
        got = np.stack(philox.philox4x32_10(ctr[:, 0], ctr[:, 1], ctr[:, 2], ctr[:, 3], *key), axis=1)
        for i in range(ctr.shape[0]):
            assert philox_bigint([int(x) for x in ctr[i]], key) == [int(x) for x in got[i]]


def test_counter_layout_and_seed_split():
    seed = 0x0123456789ABCDEF
    got = [int(w) for w in philox.philox_block(seed, 7, 11, 13, 1)]
    assert got == philox_bigint([7, 11, 13, 1], [0x89ABCDEF, 0x01234567])
    stream = philox.philox_u32_stream(seed, 13, 11, 5, 4, 1)
    assert [int(w) for w in stream[8:12]] == got


def test_bijective_on_counter_sample():
    j = np.arange(1 << 16)
    words = np.stack(philox.philox_block(42, j, 3, 1, 0), axis=1)
    packed = words.astype(np.uint64)
    a = (packed[:, 0] << np.uint64(32)) | packed[:, 1]
    b = (packed[:, 2] << np.uint64(32)) | packed[:, 3]
    assert len(set(zip(a.tolist(), b.tolist()))) == 1 << 16


def test_unit_interval_map():
    u = philox.u32_to_unit(np.array([0, 511, 512, 0xFFFFFFFF], dtype=np.uint32))
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24 and u[2] == 3 * 2.0 ** -24
    assert u[3] == 1.0 - 2.0 ** -24
    x = np.random.default_rng(1).integers(0, 2 ** 32, size=100000, dtype=np.uint64).astype(np.uint32)
    u = philox.u32_to_unit(x)
    assert (u > 0).all() and (u < 1).all()
    assert (u.astype(np.float32).astype(np.float64) == u).all()     # exactly representable in fp32


def test_box_muller_geometry():
    """Radius comes from the first word, angle from the second; cosine first, sine second."""
    r = np.random.default_rng(2)
    xa = r.integers(0, 2 ** 32, size=5000, dtype=np.uint64).astype(np.uint32)
    xb = r.integers(0, 2 ** 32, size=5000, dtype=np.uint64).astype(np.uint32)
    z0, z1 = philox.box_muller(xa, xb)
    np.testing.assert_allclose(z0 ** 2 + z1 ** 2, -2.0 * np.log(philox.u32_to_unit(xa)), rtol=1e-12)
    ang = np.mod(np.arctan2(z1, z0), 2 * np.pi)
    np.testing.assert_allclose(ang, 2 * np.pi * philox.u32_to_unit(xb), rtol=0, atol=1e-9)


def test_word_to_parameter_mapping():
    """(x0,x1) feed parameters 4j, 4j+1 and (x2,x3) feed 4j+2, 4j+3."""
    seed, t, k = 99, 4, 6
    z = philox.pair_noise(seed, t, [k], 16)[0]
    for j in range(4):
        x = philox.philox_block(seed, j, k, t, philox.TAG_NOISE)
        for half in range(2):
            rad2 = -2.0 * np.log(philox.u32_to_unit(x[2 * half]))
            assert abs(z[4 * j + 2 * half] ** 2 + z[4 * j + 2 * half + 1] ** 2 - rad2) < 1e-12
            ang = np.mod(np.arctan2(z[4 * j + 2 * half + 1], z[4 * j + 2 * half]), 2 * np.pi)
            assert abs(ang - 2 * np.pi * philox.u32_to_unit(x[2 * half + 1])) < 1e-9


def test_normal_distribution_moments_and_ks():
    z = philox.pair_noise(20220509, 1, np.arange(250), 4000).reshape(-1)      # 10^6 draws
    n = z.size
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs(stats.kurtosis(z, fisher=False) - 3.0) < 4.0 * np.sqrt(24.0 / n)
    assert abs(stats.skew(z)) < 4.0 * np.sqrt(6.0 / n)
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert np.abs(z).max() <= np.sqrt(-2.0 * np.log(2.0 ** -24)) + 1e-12     # 5.768...


def test_streams_differ_by_every_counter_word():
    base = philox.pair_noise(5, 1, [0], 64)[0]
    assert not np.allclose(base, philox.pair_noise(5, 2, [0], 64)[0])
    assert not np.allclose(base, philox.pair_noise(5, 1, [1], 64)[0])
    assert not np.allclose(base, philox.pair_noise(6, 1, [0], 64)[0])
    assert not np.allclose(base, philox.pair_noise(5 + (1 << 32), 1, [0], 64)[0])
    # independent pairs are uncorrelated
    z = philox.pair_noise(5, 1, [0, 1], 40000)
    assert abs(np.corrcoef(z[0], z[1])[0, 1]) < 0.03


def test_random_access_equals_bulk():
    full = philox.pair_noise(77, 3, np.arange(10), 103)
    cols = np.array([0, 1, 2, 3, 50, 101, 102])
    part = philox.pair_noise(77, 3, [2, 9], 103, cols)
    assert (part == full[[2, 9]][:, cols]).all()
