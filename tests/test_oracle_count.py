"""Pins for the oracle's nugget count (Sec. 2.3: k = ceil(n / r); Eq. 7: 1 <= k <= t)."""
import math
import os
from fractions import Fraction

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "nugget_counts.txt")


def test_paper_worked_sizes():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for n, r, k in rows:
        assert oracle.nugget_count(int(n), 1, int(r)) == int(k), (n, r, k)


def test_benchmark_config_counts():
    assert oracle.nugget_count(512, 1, 10) == 52
    assert oracle.nugget_count(4096, 1, 10) == 410
    assert oracle.nugget_count(8192, 1, 20) == 410
    assert oracle.nugget_count(2048, 1, 20) == 103
    assert oracle.nugget_count(32768, 1, 10) == 3277


def test_exact_rational_ceiling_and_clamps():
    for n in list(range(0, 200)) + [4095, 4096, 4097, 32768, 10**6]:
        for num, den in [(1, 10), (1, 20), (1, 5), (1, 1), (3, 7), (1, 1000), (2, 1)]:
            k = oracle.nugget_count(n, num, den)
            if n == 0:
                assert k == 0
                continue
            want = min(n, max(1, math.ceil(Fraction(n * num, den))))
            assert k == want
            assert 1 <= k <= n


def test_integer_arithmetic_avoids_binary_fraction_trap():
    # ceil(0.07 * 100) evaluates to 8 in binary floating point; the count is 7.
    assert math.ceil((7 / 100) * 100) == 8
    assert oracle.nugget_count(100, 7, 100) == 7


def test_ratio_one_keeps_everything():
    for n in (1, 2, 17, 4096):
        assert oracle.nugget_count(n, 1, 1) == n
