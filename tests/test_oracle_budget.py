"""Pins for the oracle's budget and partition arithmetic (Sec. 3.1; App. B equation)."""
import math
import os

import numpy as np
import pytest
from scipy.stats import hmean

from oracle import laserkv_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "budget_paper_settings.txt")


def test_budget_paper_settings_golden():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for s, l, rn, rd, b in rows:
        assert O.budget(int(s), int(l), int(rn), int(rd)) == int(b)


@pytest.mark.parametrize("s,l", [(4096, 16384), (2048, 65536), (8192, 131072), (512, 4096), (1000, 7777)])
def test_budget_is_scaled_harmonic_mean(s, l):
    # App. B prose: the harmonic mean of block size and context length times r.
    hm = hmean([float(s), float(l)])
    for rn, rd in [(1, 4), (1, 2), (1, 8), (3, 10)]:
        exact = rn / rd * hm
        b = O.budget(s, l, rn, rd)
        if abs(exact - round(exact)) > 1e-6:          # away from a floor boundary
            assert b == math.floor(exact)
        assert exact - 1 - 1e-6 < b <= exact + 1e-6


def test_budget_limits():
    for s in (512, 1024, 4096):
        assert O.budget(s, s, 1, 4) == s // 4              # L = S  =>  B = floor(r S)
        assert O.budget(s, 10**12, 1, 4) == s // 2 - 1      # L -> inf: B -> 2 r S from below
        prev = 0
        for l in (s, 2 * s, 8 * s, 64 * s):
            b = O.budget(s, l, 1, 4)
            assert prev <= b < 2 * s // 4 + 1
            prev = b


@pytest.mark.parametrize("B,n,alpha,s_t", [(227, 4, 0.75, 512), (910, 4, 0.75, 2048), (992, 8, 0.75, 2048),
                                           (1985, 8, 0.75, 4096), (3855, 16, 0.75, 8192), (1985, 8, 0.0, 4096),
                                           (1985, 8, 1.0, 4096), (300, 3, 0.5, 100), (7, 2, 0.3, 512)])
def test_partition_sums_to_budget(B, n, alpha, s_t):
    a, loc, ke, kl = O.partition(B, n, alpha, s_t)
    bt = min(B, s_t)
    assert a == loc == bt // n                           # "B/n" anchors and "B/n" local window
    assert a + loc + ke + kl == bt                       # kept count == budget
    assert ke + kl == bt - 2 * (bt // n)                 # "B - 2B/n"
    assert ke + kl <= s_t - a - loc                      # fits the candidate set
    assert abs(ke - alpha * (ke + kl)) < 1.0 and ke <= alpha * (ke + kl) + 1e-9
    if alpha == 1.0:
        assert kl == 0
    if alpha == 0.0:
        assert ke == 0


def test_partition_table_values():
    # Values worked by hand for the benchmark's configurations (B from the App. B equation).
    assert O.partition(227, 4, 0.75, 512) == (56, 56, 86, 29)
    assert O.partition(1985, 8, 0.75, 4096) == (248, 248, 1116, 373)
    assert O.partition(3855, 16, 0.75, 8192) == (240, 240, 2531, 844)


def test_partition_rejects_bad_arguments():
    with pytest.raises(ValueError):
        O.partition(100, 1, 0.75, 512)
    with pytest.raises(ValueError):
        O.partition(100, 4, 1.5, 512)
