"""The selection kernel divides softmax numerators E (integers below 2^32) by the integer sums Z (below
2^48) in fp64 and must get the correctly rounded quotient, because the oracle uses IEEE division.  To
avoid one full division per (candidate, head) it computes a reciprocal y of Z once per head -- the
hardware's approximate reciprocal, sharpened by three Newton steps y += y*(1 - Z*y) to within an ulp or
two -- and then refines q = E*y with fused multiply-adds: r = E - Z*q (exact), q += r*y, twice.  After
the first correction q is within an ulp; the second leaves an error of at most |r|*|y - 1/Z| <= 2^-52 ulp,
while E/Z, a quotient of integers with Z < 2^48, is either a floating-point number or at least 2^-49 ulp
away from the nearest rounding boundary: the rounding cannot go wrong.  This test replays the scheme with
exact rational arithmetic (every fused multiply-add rounded once), starting from seeds with relative
errors up to 2^-12 of either sign, and compares with the correctly rounded quotient."""
from fractions import Fraction
import random


def rn(x: Fraction) -> float:
    return x.numerator / x.denominator          # int / int is correctly rounded in Python


def fma(a: float, b: float, c: float) -> float:
    return rn(Fraction(a) * Fraction(b) + Fraction(c))


def reciprocal(b: float, seed_error: float) -> float:
    y = (1.0 / b) * (1.0 + seed_error)          # stands in for the hardware's approximate reciprocal
    for _ in range(3):
        e = fma(-b, y, 1.0)
        y = fma(y, e, y)
    return y


def div_scheme(a: float, b: float, seed_error: float = 0.0) -> float:
    y = reciprocal(b, seed_error)
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
    for i, (e, z) in enumerate(cases):
        seed_error = (2.0 ** -rng.randrange(12, 40)) * (1 if i % 2 else -1)
        assert div_scheme(float(e), float(z), seed_error) == e / z, (e, z, seed_error)
        assert abs(reciprocal(float(z), seed_error) * z - 1.0) <= 2.0 ** -51
