"""Plain reference of the latency table for models whose latency depends on the input (arXiv 1812.01776,
Section 8, second limitation): per table entry, the tail of the latencies measured over the sample queries.

TEST INFRASTRUCTURE ONLY: imported by tests/ and nothing else.

Two tails, both named in that passage: a percentile of the samples, and the mean plus k standard deviations.
Readings where the passage is silent: the percentile is the nearest-rank one (as for the SLO's P99: the smallest
sample with at least that share of the samples at or below it); the standard deviation is the population one;
a latency is a whole number of microseconds, so the second tail is rounded up (the plan stays feasible).
"""
import math
from decimal import ROUND_CEILING, Decimal, getcontext
from fractions import Fraction


def percentile_tail(samples, pct_hundredths):
    """Smallest sample v such that at least pct_hundredths/100 percent of the samples are <= v."""
    xs = sorted(int(x) for x in samples)
    n = len(xs)
    for v in xs:
        at_or_below = sum(1 for x in xs if x <= v)
        if Fraction(at_or_below, n) >= Fraction(pct_hundredths, 10000):
            return v
    raise ValueError("empty sample set")


def sigma_tail(samples, k_thousandths):
    """ceil(mean + k sigma), k = k_thousandths / 1000.  When the variance is the square of a fraction the sum is a
    fraction and is rounded up exactly; otherwise sigma is irrational, the sum is no integer, and 120-digit decimal
    arithmetic decides which integers it lies between."""
    xs = [int(x) for x in samples]
    n = len(xs)
    mean = Fraction(sum(xs), n)
    var = sum((Fraction(x) - mean) ** 2 for x in xs) / n
    k = Fraction(k_thousandths, 1000)
    rn, rd = math.isqrt(var.numerator), math.isqrt(var.denominator)
    if rn * rn == var.numerator and rd * rd == var.denominator:
        return math.ceil(mean + k * Fraction(rn, rd))
    getcontext().prec = 120
    sigma = (Decimal(var.numerator) / Decimal(var.denominator)).sqrt()
    value = Decimal(mean.numerator) / Decimal(mean.denominator) + Decimal(k.numerator) / Decimal(k.denominator) * sigma
    return int(value.to_integral_value(rounding=ROUND_CEILING))
