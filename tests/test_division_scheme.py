"""The selection kernel divides softmax numerators E (integers below 2^32) by the integer sums Z (below
2^48) in fp64 and must get the correctly rounded quotient, because the oracle uses IEEE division.  To
avoid one full division per (candidate, head) it computes y = RN(1/Z) once per head with a true division
and then refines q = E*y with fused multiply-adds: r = E - Z*q, q += r*y, twice.  The second correction is
Markstein's final step, which returns RN(E/Z) whenever q is within one ulp and y is the correctly
rounded reciprocal.  This test replays the scheme with exact rational arithmetic (every fused
multiply-add rounded once) and compares with the correctly rounded quotient."""
from fractions import Fraction
import random


def rn(x: Fraction) -> float:
    return x.numerator / x.denominator          # int / int is correctly rounded in Python


def fma(a: float, b: float, c: float) -> float:
    return rn(Fraction(a) * Fraction(b) + Fraction(c))


def div_scheme(a: float, b: float) -> float:
    y = 1.0 / b
    q = a * y
    r = fma(-b, q, a)
    q = fma(r, y, q)
    r = fma(-b, q, a)
    return fma(r, y, q)


def test_refined_reciprocal_division_is_correctly_rounded():
    rng = random.Random(5)
    cases = []
    for _ in range(60000):
        z = rng.randrange(1, 1 << rng.randrange(1, 49))
        e = rng.randrange(0, min(z, (1 << 32) - 1) + 1)       # a numerator never exceeds its sum
        cases.append((e, z))
    for _ in range(20000):                                     # sums with all-ones and sparse significands
        k = rng.randrange(2, 49)
        z = (1 << k) - rng.randrange(1, 4)
        cases.append((rng.randrange(0, min(z, (1 << 32) - 1) + 1), z))
        z = (1 << k) + rng.randrange(0, 4)
        cases.append((rng.randrange(0, min(z, (1 << 32) - 1) + 1), z))
    cases += [(0, 1), (1, 1), ((1 << 31), (1 << 31)), ((1 << 31), (1 << 47) + 1), (1, (1 << 48) - 1), ((1 << 32) - 1, (1 << 48) - 1)]
    for e, z in cases:
        assert div_scheme(float(e), float(z)) == e / z, (e, z)
