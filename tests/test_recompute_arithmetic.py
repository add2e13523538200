"""The division-free stage time of the recomputing kernels, checked in exact rational arithmetic.

The kernels form ceil(x / r) for odd r as the integer left in the low bits of
    fma(t, 1/r, 1.5 * 2^52),   t = x + (r/2 - 1 + r * offset),
with offset = 2^-18 for 32-bit values (x < 2^32) and 2^-8 for 64-bit values (x <= 2^40), and the
even counts as ceil(ceil(x / r) / 2^k) (h of Sec. III-C without the communication term is
ceil(T / r)).  Here the fused multiply-add is evaluated exactly (fractions, one rounding to
nearest-even at the end, which at that magnitude is a rounding to an integer), the reciprocal
is the correctly rounded double, and the result is compared with integer division at the values
where a rounding error would show first: multiples of r and their neighbours, the top of the
range, and random values."""
from fractions import Fraction

import numpy as np
import pytest

MAGIC = Fraction(3 * 2 ** 51)   # 1.5 * 2^52


def _round_half_even(q: Fraction) -> int:
    f = q.numerator // q.denominator
    rem = q - f
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f


def quotient_odd(x: int, r: int, offset: Fraction, low_bits: int) -> int:
    t = Fraction(x) + Fraction(r, 2) - 1 + r * offset
    assert Fraction(float(t)) == t, "t must be exact in double precision"
    inv = Fraction(1.0 / r)                       # the rounded reciprocal the kernel holds
    y = _round_half_even(t * inv + MAGIC)         # one rounding: the sum lies in [2^52, 2^53)
    assert 2 ** 52 <= y < 2 ** 53
    return (y - 2 ** 52) & ((1 << low_bits) - 1)  # the mantissa bits the kernel keeps


def edge_values(top: int, g) -> list:
    xs = {0, 1, 2, top, top - 1, top - 2}
    for r in range(1, 65):
        for m in (1, 2, 3, 1000, top // r, top // r - 1, top // (2 * r)):
            for d in (-1, 0, 1):
                v = m * r + d
                if 0 <= v <= top:
                    xs.add(v)
    xs.update(int(v) for v in g.integers(0, top, 2000, endpoint=True))
    xs.update(int(top - v) for v in g.integers(0, 1 << 12, 200))
    return sorted(xs)


@pytest.mark.parametrize("top,offset,low_bits", [((1 << 32) - 1, Fraction(1, 1 << 18), 32),
                                                 (1 << 40, Fraction(1, 1 << 8), 51)])
def test_quotient_matches_integer_division(top, offset, low_bits):
    g = np.random.default_rng(5)
    xs = edge_values(top, g)
    for r in range(1, 64, 2):
        for x in xs:
            assert quotient_odd(x, r, offset, low_bits) == -(-x // r), (x, r)


def test_even_counts_follow_from_the_odd_ones():
    g = np.random.default_rng(6)
    for x in edge_values(1 << 40, g)[::7]:
        for odd in range(1, 33, 2):
            k = -(-x // odd)
            sh = 1
            while (odd << sh) <= 64:
                assert (k + (1 << sh) - 1) >> sh == -(-x // (odd << sh)), (x, odd, sh)
                sh += 1


def test_running_numerator_is_exact():
    """t for the next odd r is the previous t plus 1 + 2 * offset; every partial sum must be a
    double, or the kernel's running addition would drift from the closed form."""
    for top, offset in (((1 << 32) - 1, Fraction(1, 1 << 18)), (1 << 40, Fraction(1, 1 << 8))):
        for x in (0, 1, top - 1, top):
            t = float(Fraction(x) + offset - Fraction(1, 2))
            for r in range(1, 64, 2):
                want = Fraction(x) + Fraction(r, 2) - 1 + r * offset
                assert Fraction(t) == want, (x, r)
                t = t + float(1 + 2 * offset)
