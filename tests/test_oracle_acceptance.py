"""Pins of the acceptance-statistics oracle and of the product's histogram -> rate conversion (CPU only)."""
from fractions import Fraction

import numpy as np

from oracle import acceptance as OA


def test_position_rates_closed_forms():
    k = 4
    # every draft accepted: all ones; none: all zeros
    assert OA.acceptance_by_position([k] * 7, k) == [Fraction(1)] * k
    assert OA.acceptance_by_position([0] * 7, k) == [Fraction(0)] * k
    # one verification per accept length 0..k: position i accepted by the k + 1 - i longest
    assert OA.acceptance_by_position(list(range(k + 1)), k) == [Fraction(k + 1 - i, k + 1) for i in range(1, k + 1)]
    # the mean accept length is the sum of the position rates (each accepted draft counted once at its position)
    lens = [3, 0, 4, 4, 1, 2, 4, 0]
    assert sum(OA.acceptance_by_position(lens, k)) == OA.mean_accept(lens) == Fraction(18, 8)
    # the product of the conditional rates up to i is the rate at i
    cond = OA.conditional_acceptance(lens, k)
    run = Fraction(1)
    for i, r in enumerate(OA.acceptance_by_position(lens, k)):
        run *= cond[i]
        assert run == r
    assert OA.acceptance_by_position([], 3) == [Fraction(0)] * 3


def test_position_rates_against_simulation():
    """Independent draft positions with acceptance p_i: the rate at i is prod_{j<=i} p_j (within sampling error)."""
    rng = np.random.default_rng(5)
    p = np.array([0.9, 0.8, 0.5, 0.9])
    ok = rng.random((200000, 4)) < p
    lens = np.where(ok.all(axis=1), 4, np.argmin(ok, axis=1)).tolist()
    rate = [float(x) for x in OA.acceptance_by_position(lens, 4)]
    assert np.allclose(rate, np.cumprod(p), atol=5e-3)
    cond = [float(x) for x in OA.conditional_acceptance(lens, 4)]
    assert np.allclose(cond, p, atol=5e-3)


def test_product_conversion_matches_oracle():
    """paper_2602_24174_amd.acceptance_sweeps.position_rates (host arithmetic on the GPU's histogram) against the oracle."""
    from paper_2602_24174_amd.acceptance_sweeps import position_rates
    rng = np.random.default_rng(11)
    for k in (1, 3, 8, 15):
        lens = rng.integers(0, k + 1, size=137).tolist()
        hist = OA.histogram(lens, k)
        rate, cond = position_rates(hist, k)
        assert np.allclose(rate, [float(x) for x in OA.acceptance_by_position(lens, k)], atol=1e-12)
        assert np.allclose(cond, [float(x) for x in OA.conditional_acceptance(lens, k)], atol=1e-12)
    assert position_rates([0, 0, 0], 2) == ([0.0, 0.0], [0.0, 0.0])
