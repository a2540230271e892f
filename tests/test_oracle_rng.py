"""Pins for the oracle's random numbers: the published Philox4x32-10 known-answer vectors, the
counter/key layout, and the exactly representable uniform mappings."""
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            assert len(w) == 10
            rows.append((w[0:4], w[4:6], w[6:10]))
    assert len(rows) == 3
    return rows


def test_philox_known_answers(oracle):
    for ctr, key, want in _kat_rows():
        assert list(oracle.philox4x32_10(ctr, key)) == want


def test_philox_is_a_bijection_of_the_counter(oracle):
    # distinct counters under one key never collide (Philox is a keyed permutation)
    outs = {oracle.philox4x32_10([i, 0, 0, 0], [7, 9]) for i in range(2000)}
    assert len(outs) == 2000


def test_word_layout(oracle):
    from oracle.ears_oracle import philox_word
    seed = 0x0123456789ABCDEF
    seq = (0xABCDEF << 32) | 0x13572468   # 56-bit sequence id
    pos = 5
    key = [seed & 0xFFFFFFFF, seed >> 32]
    # acceptance uniform: domain 0, block 0, word 0
    blk = oracle.philox4x32_10([0, pos, seq & 0xFFFFFFFF, (0 << 24) | (seq >> 32)], key)
    assert philox_word(seed, seq, pos, 0, 0, 0) == blk[0]
    assert oracle.accept_uniform(seed, seq, pos) == (blk[0] >> 8) * 2.0 ** -24
    # Gumbel noise: 8 coarse bits (domain 1, one block per sixteen vocabulary indices, one byte
    # each) and 32 fine bits (domain 2, one block per four indices, one word each)
    for v in (0, 1, 2, 3, 4, 5, 15, 16, 17, 1023, 128255):
        coarse = oracle.philox4x32_10([v >> 4, pos, seq & 0xFFFFFFFF, (1 << 24) | (seq >> 32)], key)
        fine = oracle.philox4x32_10([v >> 2, pos, seq & 0xFFFFFFFF, (2 << 24) | (seq >> 32)], key)
        h = (coarse[(v >> 2) & 3] >> (8 * (v & 3))) & 0xFF
        f = fine[v & 3]
        u = (h + (f + 0.5) / 2.0 ** 32) / 256.0
        assert oracle.gumbel_uniform(seed, seq, pos, v) == u
        assert oracle.gumbel(seed, seq, pos, v) == pytest.approx(-math.log(-math.log(u)), rel=1e-15)


def test_uniform_ranges_and_exactness(oracle):
    us = np.array([oracle.accept_uniform(11, s, p) for s in range(300) for p in range(8)])
    gs = np.array([oracle.gumbel_uniform(11, s, 0, v) for s in range(30) for v in range(80)])
    assert us.min() >= 0.0 and us.max() < 1.0
    assert gs.min() > 0.0 and gs.max() < 1.0
    # the acceptance uniform lands on values an fp32 holds exactly; the Gumbel uniform on odd
    # multiples of 2^-41 (exact in fp64)
    assert np.all(us.astype(np.float32).astype(np.float64) == us)
    k = gs * 2.0 ** 41
    assert np.all(k == np.floor(k)) and np.all(k % 2 == 1)
    # and both look uniform (Kolmogorov-Smirnov)
    from scipy import stats
    assert stats.kstest(us, "uniform").pvalue > 1e-3
    assert stats.kstest(gs, "uniform").pvalue > 1e-3
    # the coarse byte alone is uniform over its 256 values
    hs = np.floor(np.array([oracle.gumbel_uniform(3, 1, 2, v) for v in range(20000)]) * 256).astype(int)
    assert stats.chisquare(np.bincount(hs, minlength=256)).pvalue > 1e-3


def test_gumbel_extremes():
    # the smallest and largest u the mapping can produce bound the noise
    u_min = (0 + (0 + 0.5) / 2.0 ** 32) / 256.0
    u_max = (255 + (2 ** 32 - 1 + 0.5) / 2.0 ** 32) / 256.0
    assert u_min == 2.0 ** -41 and u_max == 1.0 - 2.0 ** -41
    assert -math.log(-math.log(u_min)) == pytest.approx(-math.log(41 * math.log(2.0)), abs=1e-12)
    assert -math.log(-math.log(u_max)) == pytest.approx(41 * math.log(2.0), abs=1e-9)


def test_gumbel_law(oracle):
    # g = -log(-log u) must follow the standard Gumbel law: CDF exp(-exp(-g))
    from scipy import stats
    g = np.array([oracle.gumbel(5, s, 1, v) for s in range(20) for v in range(200)])
    assert stats.kstest(g, "gumbel_r").pvalue > 1e-3
