"""Test oracle (not part of the product path): size and dominance of the typical set of a count table.

Written from the paper's definitions: the Shannon entropy of the n-gram distribution and the number of unique
n-grams that attain a given share (80 % in the paper) of its CDF ("Task-Induced n-Grams Concentration"), and the
Renyi entropy of order 2 (Appendix, "Predicting Model Speedup ... from the Data":
H_alpha(p) = log(sum_x p(x)^alpha) / (1 - alpha)).  The distribution is p(x) = count(x) / sum of counts over the
entries of one table.  Entropies in nats, float64 with compensated sums; the coverage count in exact integers.
"""
import math
from fractions import Fraction


def shannon_entropy(counts):
    c = [int(x) for x in counts if int(x) > 0]
    total = sum(c)
    if total == 0:
        return 0.0
    return -math.fsum((x / total) * math.log(x / total) for x in c)


def renyi_entropy(counts, alpha=2):
    assert alpha != 1
    c = [int(x) for x in counts if int(x) > 0]
    total = sum(c)
    if total == 0:
        return 0.0
    return math.log(math.fsum((x / total) ** alpha for x in c)) / (1 - alpha)


def coverage_count(counts, coverage=Fraction(4, 5)):
    """Fewest entries, most frequent first, whose counts sum to at least `coverage` of the total."""
    c = sorted((int(x) for x in counts if int(x) > 0), reverse=True)
    need = Fraction(coverage) * sum(c)
    run = 0
    for m, x in enumerate(c):
        if run >= need:
            return m
        run += x
    return len(c)


def table_stats(counts, coverage=Fraction(4, 5)):
    c = [int(x) for x in counts if int(x) > 0]
    return {"n_entries": len(c), "total": sum(c), "n_cover": coverage_count(c, coverage),
            "shannon": shannon_entropy(c), "renyi2": renyi_entropy(c, 2)}
