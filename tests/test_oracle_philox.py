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
