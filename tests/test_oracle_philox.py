"""Pins for the oracle's Philox4x32-10 and uniform conventions."""
import numpy as np
from conftest import golden_rows
from oracle import philox


def test_known_answer_vectors():
    rows = golden_rows("philox4x32_10_kat.txt")
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert philox.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_uniform_ranges_and_endpoints():
    assert philox.u_open_closed(0) == 2.0 ** -24
    assert philox.u_open_closed(0xFFFFFFFF) == 1.0
    assert philox.u_closed_open(0) == 0.0
    assert philox.u_closed_open(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert philox.u_closed_open(0x000000FF) == 0.0          # low 8 bits are dropped


def test_streams_are_distinct_and_roughly_uniform():
    us = np.array([philox.accept_uniform(7, b, t, i) for b in range(8) for t in range(16) for i in range(8)])
    vs = np.array([philox.draft_uniform(7, b, t, i) for b in range(8) for t in range(16) for i in range(8)])
    assert len(set(us)) > 1000 and len(set(vs)) > 1000
    assert not np.any(us == vs + 2.0 ** -24)                # different purposes give different words
    assert abs(us.mean() - 0.5) < 0.04 and abs(vs.mean() - 0.5) < 0.04
    assert us.min() > 0.0 and us.max() <= 1.0 and vs.min() >= 0.0 and vs.max() < 1.0
    # the seed's upper 32 bits matter
    assert philox.word(1, 0, 0, 0, 0) != philox.word(1 + (1 << 32), 0, 0, 0, 0)


def test_vectorised_philox_equals_the_scalar_one():
    seed = 0x1234_5678_9ABC_DEF0
    g = np.arange(50)
    w = philox.philox4x32_10_vec(3, 7, 2, 4 + 8 * g, (seed & 0xFFFFFFFF, seed >> 32))
    for j in (0, 1, 17, 49):
        ref = philox.philox4x32_10((3, 7, 2, 4 + 8 * j), (seed & 0xFFFFFFFF, seed >> 32))
        assert [int(w[k][j]) for k in range(4)] == ref


def test_noise_normals_are_standard_normal_and_addressed_by_counter():
    from scipy import stats
    z = np.concatenate([philox.noise_normals(11, b, 5, i, 4096) for b in range(4) for i in range(6)])
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(z.mean()) < 0.02 and abs(z.var() - 1.0) < 0.03
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 0.02            # the two members of a Box-Muller pair
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.02
    a = philox.noise_normals(11, 0, 5, 0, 1000)
    assert np.array_equal(a, philox.noise_normals(11, 0, 5, 0, 1000))
    assert np.array_equal(a[:997], philox.noise_normals(11, 0, 5, 0, 997))      # a prefix of the same stream
    for other in ((12, 0, 5, 0), (11, 1, 5, 0), (11, 0, 6, 0), (11, 0, 5, 1)):
        assert not np.allclose(a, philox.noise_normals(*other, 1000))
    # the pair (z0, z1) lies on the circle of radius sqrt(-2 ln u1): its squared radius is chi-square with 2 dof
    r2 = z[0::2] ** 2 + z[1::2] ** 2
    assert stats.kstest(r2, "chi2", args=(2,)).pvalue > 1e-3
