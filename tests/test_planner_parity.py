"""The library's planner entry points (host code, no device work) against the oracle: exact for the
integer results, 1e-15 relative for the times (same double-precision formulas)."""
import os
import random

import pytest

from oracle import planner as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "head_padding_example.txt")


@pytest.fixture(scope="module")
def pda():
    import paper_2511_12056_amd as pda
    return pda


def test_paper_example_through_the_library(pda):
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            H, n, padded, per, needed = map(int, line.split())
            assert pda.plan_head_padding(H, n) == (padded, per, needed)


def test_n_decode_matches_oracle(pda):
    rng = random.Random(2511)
    for _ in range(5000):
        N = rng.randint(2, 64)
        tden = rng.choice([rng.uniform(0.01, 1000.0), float(rng.randint(1, 64))])
        tdec = rng.choice([rng.uniform(0.01, 1000.0), float(rng.randint(1, 64))])
        assert pda.plan_n_decode(tden, tdec, N) == P.n_decode(tden, tdec, N), (tden, tdec, N)
    # exact ties (ratio * N is an integer): both sides must take the ceiling of the same double
    for N in (2, 4, 8, 16):
        for a in range(1, N):
            assert pda.plan_n_decode(float(N - a), float(a), N) == P.n_decode(float(N - a), float(a), N)


def test_aco_matches_oracle(pda):
    rng = random.Random(12056)
    for _ in range(2000):
        tL, tA = rng.uniform(0, 50), rng.uniform(0.001, 500)
        a, b = rng.randint(1, 16), rng.randint(0, 16)
        got, want = pda.plan_aco(tL, tA, a, b), P.aco_times(tL, tA, a, b)
        for g, w in zip(got, want):
            assert g == pytest.approx(w, rel=1e-15, abs=0)


def test_padding_and_groups_match_oracle(pda):
    for H in range(1, 70):
        for n in range(1, 20):
            assert pda.plan_head_padding(H, n) == P.head_padding(H, n)
            assert pda.plan_ragged_groups(H, n) == P.ragged_groups(H, n)
    assert pda.plan_ragged_groups(0, 3) == [0, 0, 0]
