"""Pins for the oracle's distance functions (Sec. 2; negative inner product per Appendix A)."""
import numpy as np
import pytest

from helpers import np_dist


def test_closed_forms(oracle):
    O = oracle
    a = np.zeros(128, np.uint8)
    b = np.full(128, 255, np.uint8)
    assert O.distance(a, b) == 128 * 255 * 255 == 8323200
    assert O.distance(b, a) == 8323200
    assert O.distance(a, a) == 0
    a = np.full(100, -127, np.int8)
    b = np.full(100, 127, np.int8)
    assert O.distance(a, b) == 100 * 254 * 254 == 6451600
    assert O.distance(a, b, O.MIPS) == 100 * 127 * 127
    assert O.distance(a, a, O.MIPS) == -100 * 127 * 127
    # a single coordinate: (3 - 250)^2
    a = np.zeros(8, np.uint8); b = np.zeros(8, np.uint8)
    a[5] = 3; b[5] = 250
    assert O.distance(a, b) == 247 * 247


@pytest.mark.parametrize("dtype,lo,hi", [(np.uint8, 0, 256), (np.int8, -127, 128)])
@pytest.mark.parametrize("d", [1, 3, 4, 100, 128, 131])
def test_integer_exact(oracle, dtype, lo, hi, d):
    rng = np.random.default_rng(d * 7 + (dtype == np.int8))
    for _ in range(20):
        a = rng.integers(lo, hi, d).astype(dtype)
        b = rng.integers(lo, hi, d).astype(dtype)
        for metric in (0, 1):
            assert oracle.distance(a, b, metric) == np_dist(a, b, metric)
        # expansion identity ||a-b||^2 = ||a||^2 + ||b||^2 - 2<a,b>
        A = a.astype(np.int64); B = b.astype(np.int64)
        assert oracle.distance(a, b, 0) == int((A * A).sum() + (B * B).sum() - 2 * (A * B).sum())


@pytest.mark.parametrize("d", [1, 7, 200])
def test_float_rounding(oracle, d):
    rng = np.random.default_rng(d)
    for _ in range(20):
        a = rng.standard_normal(d).astype(np.float32)
        b = rng.standard_normal(d).astype(np.float32)
        l2 = oracle.distance(a, b, 0)
        ip = oracle.distance(a, b, 1)
        # exact rational value via python fractions on the float inputs
        from fractions import Fraction
        fa = [Fraction(float(x)) for x in a]; fb = [Fraction(float(x)) for x in b]
        l2x = sum((x - y) ** 2 for x, y in zip(fa, fb))
        ipx = -sum(x * y for x, y in zip(fa, fb))
        assert abs(Fraction(l2) - l2x) <= abs(l2x) * Fraction(1, 2 ** 23)
        assert abs(Fraction(ip) - ipx) <= sum(abs(x * y) for x, y in zip(fa, fb)) * Fraction(1, 2 ** 23)
        assert l2 == float(np.float32(l2)) and ip == float(np.float32(ip))
        assert l2 == oracle.distance(b, a, 0)


def test_negative_zero_becomes_positive(oracle):
    a = np.zeros(4, np.float32)
    b = np.ones(4, np.float32)
    v = oracle.distance(a, b, 1)
    assert v == 0.0 and not np.signbit(v)
