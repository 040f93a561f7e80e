"""Pins for the oracle's counter-based random streams (no GPU)."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = philox.philox4x32_10(v[0], v[1], v[2], v[3], v[4], v[5])
        assert [int(o) for o in out] == v[6:10]


def test_philox_is_a_bijection_on_small_cube():
    # distinct counters -> distinct outputs (spot check of the permutation property)
    c = np.arange(4096, dtype=np.uint64)
    o = np.stack(philox.philox4x32_10(c, 0, 7, 1, 123, 456), axis=1)
    assert np.unique(o, axis=0).shape[0] == 4096


def test_uniform_is_open_interval_and_fp32_exact():
    w = np.array([0, 1, 511, 512, 2 ** 31, 2 ** 32 - 1], dtype=np.uint32)
    u = philox.word_to_uniform(w)
    assert u.min() == 2.0 ** -24 and u.max() == 1.0 - 2.0 ** -24
    assert np.all(u.astype(np.float32).astype(np.float64) == u)


def test_normals_layout_keyed_by_chain_step_and_block():
    z = philox.normals(5, np.array([3, 4]), np.array([9, 9]), 10)
    assert z.shape == (2, 10)
    # element i depends only on block i//4: a longer vector has the same prefix
    z2 = philox.normals(5, np.array([3, 4]), np.array([9, 9]), 16)
    assert np.array_equal(z, z2[:, :10])
    # rebuild element 5 of chain 4 by hand from words 0 and 1 of block 1
    w = philox.philox4x32_10(4, 0, 9, (philox.STREAM_NOISE << 28) | 1, 5, 0)
    u0, u1 = philox.word_to_uniform(w[0]), philox.word_to_uniform(w[1])
    assert z[1, 5] == np.sqrt(-2 * np.log(u0)) * np.sin(2 * np.pi * u1)
    # streams, steps, seeds and chains are all distinct
    base = philox.normals(5, np.array([3]), np.array([9]), 8)
    for other in (philox.normals(6, np.array([3]), np.array([9]), 8),
                  philox.normals(5, np.array([2]), np.array([9]), 8),
                  philox.normals(5, np.array([3]), np.array([8]), 8),
                  philox.normals(5, np.array([3]), np.array([9]), 8, stream=philox.STREAM_INIT)):
        assert not np.any(base == other)
    # 64-bit chain ids and seeds use their high words
    assert not np.array_equal(philox.normals(1, np.array([1]), np.array([0]), 4),
                              philox.normals(1, np.array([1 + 2 ** 32]), np.array([0]), 4))
    assert not np.array_equal(philox.normals(1, np.array([1]), np.array([0]), 4),
                              philox.normals(1 + 2 ** 32, np.array([1]), np.array([0]), 4))


def test_normals_and_uniforms_distribution():
    ids = np.arange(2000)
    z = philox.normals(11, ids, np.full(2000, 3), 64).ravel()
    assert abs(z.mean()) < 4 / np.sqrt(z.size)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / z.size)
    assert abs(stats.kurtosis(z)) < 0.1
    assert stats.kstest(z, "norm").pvalue > 1e-3
    u = philox.uniforms(11, ids[:, None], np.arange(1, 101)[None, :]).ravel()
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    # neighbouring elements / steps are uncorrelated
    zz = philox.normals(11, ids, np.full(2000, 3), 64)
    assert abs(np.corrcoef(zz[:, 0], zz[:, 1])[0, 1]) < 0.1
    z4 = philox.normals(11, ids, np.full(2000, 4), 64)
    assert abs(np.corrcoef(zz.ravel(), z4.ravel())[0, 1]) < 0.02
