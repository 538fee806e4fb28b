"""Pins of the table-statistics oracle: closed forms, a library routine, brute force (CPU only)."""
import itertools
import math
from fractions import Fraction

import numpy as np
import scipy.stats

from oracle import table_stats as OS


def test_uniform_and_point_mass():
    for n in (1, 2, 7, 1000):
        for c in (1, 5):
            s = OS.table_stats([c] * n)
            assert s["n_entries"] == n and s["total"] == c * n
            assert abs(s["shannon"] - math.log(n)) < 1e-12 and abs(s["renyi2"] - math.log(n)) < 1e-12
            assert s["n_cover"] == math.ceil(Fraction(4, 5) * n)          # equal counts: 80 % of the entries
    assert OS.table_stats([]) == {"n_entries": 0, "total": 0, "n_cover": 0, "shannon": 0.0, "renyi2": 0.0}
    assert OS.table_stats([0, 0, 9, 0])["n_entries"] == 1                 # empty slots are not entries
    assert OS.table_stats([0, 0, 9, 0])["shannon"] == 0.0


def test_two_point_closed_form():
    # p = (3/4, 1/4): H = ln 4 - (3/4) ln 3 ; H2 = -ln(9/16 + 1/16) = ln(8/5)
    s = OS.table_stats([3, 1])
    assert abs(s["shannon"] - (math.log(4) - 0.75 * math.log(3))) < 1e-14
    assert abs(s["renyi2"] - math.log(8 / 5)) < 1e-14
    assert s["n_cover"] == 2                                               # 3/4 < 0.8
    assert OS.table_stats([4, 1])["n_cover"] == 1                          # 4/5 attains 0.8 exactly
    assert OS.coverage_count([4, 1], Fraction(81, 100)) == 2
    assert OS.coverage_count([4, 1], 0) == 0 and OS.coverage_count([4, 1], 1) == 2


def test_geometric_distribution():
    # counts 2^(m-1), ..., 2, 1, 1 : p_i = 2^-i (i = 1..m-1... ) with the last two equal -> H = (2 - 2^(2-m)) ln 2
    m = 12
    counts = [2 ** (m - 1 - i) for i in range(m)] + [1]
    s = OS.table_stats(counts)
    assert s["total"] == 2 ** m
    h = sum(i * 2.0 ** -i for i in range(1, m + 1)) * math.log(2) + m * 2.0 ** -m * math.log(2)
    assert abs(s["shannon"] - h) < 1e-13
    p2 = sum(4.0 ** -i for i in range(1, m + 1)) + 4.0 ** -m
    assert abs(s["renyi2"] + math.log(p2)) < 1e-13
    assert s["n_cover"] == 3                                               # 1/2 + 1/4 + 1/8 = 0.875 >= 0.8 > 0.75


def test_against_scipy_and_order_relations():
    rng = np.random.default_rng(3)
    for _ in range(20):
        counts = rng.zipf(1.3, size=int(rng.integers(1, 400))).astype(np.int64)
        counts = np.minimum(counts, 10 ** 6)
        s = OS.table_stats(counts.tolist())
        assert abs(s["shannon"] - scipy.stats.entropy(counts)) < 1e-10
        p = counts / counts.sum()
        assert abs(s["renyi2"] + math.log(float((p * p).sum()))) < 1e-10
        assert s["renyi2"] <= s["shannon"] + 1e-12                          # Renyi entropies fall with the order
        assert s["shannon"] <= math.log(len(counts)) + 1e-12
        # permutation invariance
        assert OS.table_stats(rng.permutation(counts).tolist()) == s or \
            abs(OS.table_stats(rng.permutation(counts).tolist())["shannon"] - s["shannon"]) < 1e-12


def test_coverage_brute_force():
    rng = np.random.default_rng(9)
    for _ in range(60):
        n = int(rng.integers(1, 8))
        counts = rng.integers(1, 12, size=n).tolist()
        for cov in (Fraction(1, 2), Fraction(4, 5), Fraction(99, 100), Fraction(1)):
            best = None
            for m in range(0, n + 1):                                      # smallest subset size reaching the share
                if any(sum(sub) >= cov * sum(counts) for sub in itertools.combinations(counts, m)):
                    best = m
                    break
            assert OS.coverage_count(counts, cov) == best
