"""The arithmetic behind the k <= 32 pass, checked on the CPU with exact rationals.

The pass forms every product w * a from three bf16 pieces of each operand.  What
has to hold for its sums to be the fp32 sums of the exact products:
  * the pieces of a float add up to it exactly,
  * each piece has at most 8 significant bits (it is a bf16),
  * each of the nine piece products has at most 16 significant bits, so a
    float32 (24 bits) holds it exactly, and the nine add up to w * a.
No GPU code is involved: the pieces are produced here with integer masks.
"""
from fractions import Fraction

import numpy as np


def pieces(x):
    x = np.asarray(x, dtype=np.float32)
    h = (x.view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)
    r = x - h
    m = (r.view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)
    l = r - m
    return h, m, l


def significant_bits(v):
    f = Fraction(float(v))
    if f == 0:
        return 0
    num = abs(f.numerator)
    while num % 2 == 0:
        num //= 2
    return num.bit_length()


def sample(n, seed):
    r = np.random.default_rng(seed)
    x = r.random(n, dtype=np.float32) * np.float32(2.0) ** r.integers(-60, 60, n).astype(np.float32)
    x[:4] = [0.0, 1.0, np.float32(1.0) - np.float32(2.0) ** -24, np.float32(3.0e38)]
    return x.astype(np.float32)


def test_pieces_are_bf16_and_sum_exactly():
    x = sample(2000, 1)
    h, m, l = pieces(x)
    for p in (h, m, l):
        assert ((p.view(np.uint32) & np.uint32(0xffff)) == 0).all()       # representable as bf16
        assert max(significant_bits(v) for v in p) <= 8
    for xi, hi, mi, li in zip(x, h, m, l):
        assert Fraction(float(hi)) + Fraction(float(mi)) + Fraction(float(li)) == Fraction(float(xi))
    # pieces of a non-negative number are non-negative and ordered
    assert (h >= 0).all() and (m >= 0).all() and (l >= 0).all()
    assert (m <= h).all() and (l <= np.maximum(m, h)).all()


def test_nine_piece_products_are_exact_in_float32_and_sum_to_the_product():
    x, y = sample(300, 2), sample(300, 3)
    px, py = pieces(x), pieces(y)
    for i in range(x.size):
        total = Fraction(0)
        for a in px:
            for b in py:
                prod = Fraction(float(a[i])) * Fraction(float(b[i]))
                if prod != 0 and Fraction(1, 2 ** 120) <= abs(prod) < Fraction(2 ** 127):
                    # fits a float32 significand, hence no rounding when it enters the fp32 sum
                    num = abs(prod.numerator)
                    while num % 2 == 0:
                        num //= 2
                    assert num.bit_length() <= 16
                    assert Fraction(float(np.float32(float(prod)))) == prod
                total += prod
        assert total == Fraction(float(x[i])) * Fraction(float(y[i]))


def test_the_product_of_the_two_lowest_pieces_is_below_2_to_minus_30_of_the_term():
    """The kernels leave l_x l_y out: each lowest piece is below 2^-15 of its float (h keeps 8
    significant bits, m the next 8 from the remainder's leading bit on), so the eight products
    they keep give x y to 2^-30, a 64th of one float32 rounding."""
    x, y = sample(2000, 5), sample(2000, 6)
    px, py = pieces(x), pieces(y)
    for i in range(x.size):
        exact = Fraction(float(x[i])) * Fraction(float(y[i]))
        assert abs(Fraction(float(px[2][i]))) * 2 ** 15 <= abs(Fraction(float(x[i])))
        dropped = Fraction(float(px[2][i])) * Fraction(float(py[2][i]))
        assert abs(dropped) * 2 ** 30 <= abs(exact)
        kept = sum(Fraction(float(a[i])) * Fraction(float(b[i]))
                   for ia, a in enumerate(px) for ib, b in enumerate(py) if (ia, ib) != (2, 2))
        assert kept + dropped == exact
