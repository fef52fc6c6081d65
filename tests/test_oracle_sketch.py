"""Pins for oracle.sketch: the element map re-derived token by token with the
plain-int generator, sample moments and normality of the Gaussian entries,
exactness of the Rademacher entries, E[S S^T] = I (Section 2.1)."""
import math

import numpy as np
from scipy import stats

from oracle import sketch
from oracle.philox import philox4x32_10_scalar

SEED = 0x0123456789ABCDEF
OFFSET = (7 << 32) | 5


def _one_entry(i, j, kind, seed, offset):
    key = (seed & 0xFFFFFFFF, seed >> 32)
    tail = (offset & 0xFFFFFFFF, offset >> 32)
    if kind == sketch.GAUSSIAN:
        r = philox4x32_10_scalar((i // 8, j) + tail, key)
        w = r[(i % 8) // 2]
        u1 = ((w >> 16) + 0.5) / 65536.0
        u2 = (w & 0xFFFF) / 65536.0
        rad = math.sqrt(-2.0 * math.log(u1))
        return rad * (math.cos(2 * math.pi * u2) if i % 2 == 0 else math.sin(2 * math.pi * u2))
    r = philox4x32_10_scalar((i // 128, j) + tail, key)
    t = i % 128
    return 1.0 - 2.0 * ((r[t // 32] >> (t % 32)) & 1)


def test_element_map_token_by_token():
    for kind, n in ((sketch.GAUSSIAN, 21), (sketch.RADEMACHER, 261)):
        k = 5
        P = sketch.sketch_P(n, k, kind, SEED, OFFSET)
        assert P.shape == (n, k)
        for i in list(range(0, n, 7)) + [n - 1]:
            for j in range(k):
                assert P[i, j] == _one_entry(i, j, kind, SEED, OFFSET) or \
                    abs(P[i, j] - _one_entry(i, j, kind, SEED, OFFSET)) < 1e-14


def test_prefix_property():
    """Entry (i, j) does not depend on n or k: a larger sketch extends a smaller one."""
    for kind in (sketch.GAUSSIAN, sketch.RADEMACHER):
        big = sketch.sketch_P(300, 9, kind, SEED, OFFSET)
        small = sketch.sketch_P(133, 4, kind, SEED, OFFSET)
        assert np.array_equal(big[:133, :4], small)


def test_state_sensitivity():
    a = sketch.sketch_P(64, 8, sketch.GAUSSIAN, 1, 0)
    assert not np.allclose(a, sketch.sketch_P(64, 8, sketch.GAUSSIAN, 2, 0))
    assert not np.allclose(a, sketch.sketch_P(64, 8, sketch.GAUSSIAN, 1, 1))
    assert not np.allclose(a, sketch.sketch_P(64, 8, sketch.GAUSSIAN, 1, 1 << 32))
    assert not np.allclose(a, sketch.sketch_P(64, 8, sketch.GAUSSIAN, 1 | (1 << 32), 0))
    assert np.array_equal(a, sketch.sketch_P(64, 8, sketch.GAUSSIAN, 1, 0))


def test_gaussian_moments_and_normality():
    P = sketch.sketch_P(4096, 256, sketch.GAUSSIAN, 11, 3)          # ~1.05e6 entries
    z = P.ravel()
    m = z.size
    assert abs(z.mean()) < 5 / math.sqrt(m)
    assert abs(z.var() - 1.0) < 5 * math.sqrt(2.0 / m)
    assert abs(np.mean(z ** 4) - 3.0) < 5 * math.sqrt(96.0 / m)
    assert abs(np.mean(z ** 3)) < 5 * math.sqrt(15.0 / m)
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert np.abs(z).max() < math.sqrt(2 * 17 * math.log(2)) + 1e-12   # radius cap of a 16-bit u1
    # cos / sin halves of a pair, neighbours in a column, neighbours in a row: uncorrelated
    for a, b in ((P[0::2], P[1::2]), (P[:-2:2], P[2::2]), (P[:, :-1], P[:, 1:])):
        r = np.mean(a * b)
        assert abs(r) < 5 / math.sqrt(a.size)


def test_rademacher_entries():
    n, k = 4096, 256
    bits = sketch.rademacher_bits(n, k, 11, 3)
    P = sketch.sketch_P(n, k, sketch.RADEMACHER, 11, 3)
    assert set(np.unique(P)) == {-1.0, 1.0}
    assert np.array_equal(P, 1.0 - 2.0 * bits)
    m = P.size
    assert abs(P.mean()) < 5 / math.sqrt(m)
    for a, b in ((P[:-1], P[1:]), (P[:, :-1], P[:, 1:]), (P[:-32], P[32:])):
        assert abs(np.mean(a * b)) < 5 / math.sqrt(a.size)


def test_scaling_is_one_over_sqrt_k():
    for kind in (sketch.GAUSSIAN, sketch.RADEMACHER):
        P = sketch.sketch_P(40, 16, kind, 5, 6)
        S = sketch.sketch_S(40, 16, kind, 5, 6)
        assert np.allclose(S * 4.0, P, rtol=0, atol=1e-15)


def test_expected_gram_is_identity():
    """E[S S^T] = I_N: average S S^T over independent states (N = 8, k = 4)."""
    n, k, draws = 8, 4, 6000
    for kind in (sketch.GAUSSIAN, sketch.RADEMACHER):
        acc = np.zeros((n, n))
        for t in range(draws):
            S = sketch.sketch_S(n, k, kind, 99, t)
            acc += S @ S.T
        acc /= draws
        # each entry of S S^T has variance <= 2/k (diagonal, Gaussian)
        assert np.abs(acc - np.eye(n)).max() < 5 * math.sqrt(2.0 / k / draws)
