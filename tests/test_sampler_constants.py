"""The constants of the truncated sampler's fixed-point exponential (csrc/kernels_sample.hip, mass45): read from the
source and checked against exact arithmetic, and the scheme itself (argument reduction by ln 2 / 32, a table of
2^(j/32), six Taylor terms) evaluated here in float64 against math.exp over the range it is used on."""
import math
import os
import re
from decimal import Decimal, getcontext

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2506_24119_amd", "csrc",
                   "kernels_sample.hip")


def _constants():
    text = open(SRC).read()
    tab = re.search(r"kExp2Tab\[32\] = \{(.*?)\};", text, re.S).group(1)
    table = [float(x) for x in tab.replace("\n", " ").split(",")]
    body = text[text.index("uint64_t mass45("):]
    body = body[:body.index("\n}\n")]
    scale = float(re.search(r"rint\(x \* ([0-9.eE+-]+)\)", body).group(1))
    hi, lo = (float(v) for v in re.findall(r"fma\(-k, ([0-9.eE+-]+), ", body)[:2])
    return table, scale, hi, lo


def test_table_and_reduction_constants_are_the_exact_values_rounded():
    table, scale, hi, lo = _constants()
    getcontext().prec = 60
    ln2 = Decimal(2).ln()
    assert len(table) == 32
    for j, t in enumerate(table):
        exact = (ln2 * j / 32).exp()
        assert abs(Decimal(t) - exact) <= exact * Decimal(2) ** -52, j                 # within one unit in the last place
    assert abs(Decimal(scale) - 32 / ln2) <= Decimal(2) ** -47
    assert abs(Decimal(hi) + Decimal(lo) - ln2 / 32) <= Decimal(10) ** -30             # the two parts add up to ln 2 / 32
    m, _ = math.frexp(hi)
    assert (int(m * 2 ** 53) & 0xFFF) == 0                                             # 12 trailing zero bits: k * hi is exact for |k| < 2^11


def test_scheme_matches_exp_to_a_few_units_in_the_last_place():
    table, scale, hi, lo = _constants()
    worst = 0.0
    n = 200_001
    for i in range(n):
        x = -32.0 * i / (n - 1)
        if not x > -32.0:
            continue
        k = float(round(x * scale))
        r = (x - k * hi) - k * lo
        p = 1.0 / 720.0
        for c in (1.0 / 120.0, 1.0 / 24.0, 1.0 / 6.0, 0.5, 1.0, 1.0):
            p = p * r + c
        ki = int(k)
        v = math.ldexp(table[ki & 31] * p, ki >> 5)
        e = math.exp(x)
        worst = max(worst, abs(v - e) / e)
    assert worst < 1e-15, worst
