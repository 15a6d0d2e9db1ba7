"""Pins for the oracle's Philox4x32-10 and the dropout keep mask built on it."""
import os

import numpy as np

from oracle.layer_oracle import philox4x32_10, dropout_keep_mask, dropout_threshold

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = philox4x32_10([v[0]], [v[1]], [v[2]], [v[3]], v[4], v[5])
        assert [int(o[0]) for o in out] == v[6:10]


def test_mask_word_order_and_counter_layout():
    # element e uses word (e mod 4) of counter q = e div 4; site and layer sit in counter words 2, 3
    seed, layer, site, h, p = 0x1234_5678_9ABC_DEF0, 3, 1, 8, 0.25
    m = dropout_keep_mask(seed, layer, site, 4, h, p)
    T = dropout_threshold(p)
    for e in range(4 * h):
        w = philox4x32_10([e // 4], [0], [site], [layer], seed & 0xFFFFFFFF, seed >> 32)
        assert bool(m[e // h, e % h]) == ((int(w[e % 4][0]) >> 8) >= T)


def test_mask_is_a_function_of_the_global_element():
    full = dropout_keep_mask(7, 1, 0, 64, 32, 0.1)
    for row0, n in ((0, 16), (16, 16), (40, 24)):
        assert np.array_equal(dropout_keep_mask(7, 1, 0, n, 32, 0.1, row0=row0), full[row0:row0 + n])
    assert not np.array_equal(full, dropout_keep_mask(7, 1, 1, 64, 32, 0.1))   # other site
    assert not np.array_equal(full, dropout_keep_mask(7, 2, 0, 64, 32, 0.1))   # other layer
    assert not np.array_equal(full, dropout_keep_mask(8, 1, 0, 64, 32, 0.1))   # other seed


def test_keep_fraction():
    for p in (0.1, 0.5):
        m = dropout_keep_mask(0, 0, 0, 512, 1024, p)
        n = m.size
        assert abs(m.mean() - (1 - p)) < 4 * np.sqrt(p * (1 - p) / n)
    assert dropout_keep_mask(0, 0, 0, 8, 16, 0.0).all()
