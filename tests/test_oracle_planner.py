"""Pins of the planner oracle (Optimal GPU partitioning; Attention Co-processing Eq. 1-3)."""
import os
from fractions import Fraction

import pytest

from oracle import planner as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "head_padding_example.txt")


def test_paper_head_padding_example():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert rows
    for H, n, padded, per, needed in (map(int, r) for r in rows):
        assert P.head_padding(H, n) == (padded, per, needed)


@pytest.mark.parametrize("tden,tdec,N", [(90.0, 10.0, 8), (300.0, 45.0, 8), (12.5, 12.5, 7), (1.0, 3.0, 4), (1000.0, 1.0, 8)])
def test_n_decode_against_exact_rationals(tden, tdec, N):
    x = Fraction(tdec) / (Fraction(tdec) + Fraction(tden)) * N
    exact = -(-x.numerator // x.denominator)
    assert P.n_decode(tden, tdec, N) == min(max(exact, 1), N - 1)


def test_n_decode_closed_forms():
    for N in range(2, 17):
        assert P.n_decode(5.0, 5.0, N) == min(-(-N // 2), N - 1)   # equal stage times: half, rounded up
    assert P.n_decode(1e9, 1.0, 8) == 1                             # decode negligible: still one GPU
    assert P.n_decode(1.0, 1e9, 8) == 7                             # denoise negligible: leave one GPU
    # balance: with the chosen split the decode group is not slower than the denoise group by more than one GPU's worth
    tden, tdec, N = 300.0, 45.0, 8
    nd = P.n_decode(tden, tdec, N)
    assert tdec / nd <= tden / (N - nd) + 1e-12 or nd == N - 1
    assert nd == 1 or tdec / (nd - 1) > tden / (N - nd + 1)


def test_n_decode_monotone_in_decode_time():
    last = 0
    for tdec in [0.5, 1, 2, 4, 8, 16, 32, 64]:
        cur = P.n_decode(16.0, float(tdec), 8)
        assert cur >= last
        last = cur


def test_aco_speedup_forms():
    tb, tc, s = P.aco_times(2.0, 6.0, 6, 2)
    assert tb == 8.0 and tc == pytest.approx(2.0 + 6.0 * 6 / 8) and s == pytest.approx(8.0 / 6.5)
    assert P.aco_times(3.0, 0.0, 6, 2)[2] == 1.0                       # no attention: nothing to share
    assert P.aco_times(0.0, 5.0, 6, 2)[2] == pytest.approx(8 / 6)      # attention only: S = N / N_denoise
    assert P.aco_times(1.0, 5.0, 6, 0)[2] == 1.0                       # no helpers
    # S grows with the helper count and is bounded by N / N_denoise
    prev = 1.0
    for nd in range(1, 6):
        s = P.aco_times(1.0, 9.0, 4, nd)[2]
        assert prev < s < (4 + nd) / 4
        prev = s
    # exact rational check
    tL, tA, a, b = Fraction(7, 3), Fraction(11, 2), 5, 3
    want = (tL + tA) / (tL + tA * Fraction(a, a + b))
    assert P.aco_times(float(tL), float(tA), a, b)[2] == pytest.approx(float(want), rel=1e-14)


def test_padding_and_ragged_groups():
    for H in range(1, 40):
        for n in range(1, 12):
            padded, per, needed = P.head_padding(H, n)
            assert padded % n == 0 and padded >= H and padded - H < n and per * n == padded
            assert (needed - 1) * per < H <= needed * per and needed <= n
            g = P.ragged_groups(H, n)
            assert sum(g) == H and len(g) == n and max(g) - min(g) <= 1 and g == sorted(g, reverse=True)
            assert max(g) == per                                       # same critical path, no wasted heads
