"""Test oracle (not part of the product path): acceptance statistics of draft-then-verify decoding.

Written from the definitions in the paper's Results ("TASC-spec": acceptance rate as a function of the draft
position; mean number of accepted tokens per verification): given the accept length m_t of every verification
(0 <= m_t <= k), draft position i (1-based) was accepted in verification t exactly when m_t >= i, because the
accepted drafts are always a prefix.
"""
from fractions import Fraction


def acceptance_by_position(accept_lens, k):
    """rate[i - 1] = share of verifications whose draft at position i was accepted, as exact fractions."""
    n = len(accept_lens)
    return [Fraction(sum(1 for m in accept_lens if m >= i), n) if n else Fraction(0) for i in range(1, k + 1)]


def conditional_acceptance(accept_lens, k):
    """cond[i - 1] = P(position i accepted | position i - 1 accepted) (position 0 = always), 0 where never reached."""
    out = []
    for i in range(1, k + 1):
        reached = sum(1 for m in accept_lens if m >= i - 1)
        out.append(Fraction(sum(1 for m in accept_lens if m >= i), reached) if reached else Fraction(0))
    return out


def mean_accept(accept_lens):
    return Fraction(sum(accept_lens), len(accept_lens)) if accept_lens else Fraction(0)


def histogram(accept_lens, k):
    h = [0] * (k + 1)
    for m in accept_lens:
        h[m] += 1
    return h
