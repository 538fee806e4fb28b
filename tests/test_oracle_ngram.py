"""Pins for oracle/ngram.py: what the paper's definition of the n-gram drafter and elementary
counting fix, independent of the oracle's own code path where possible."""
import itertools
import random
from collections import Counter
from fractions import Fraction

import numpy as np
import pytest

from oracle import ngram as O


# ---------------------------------------------------------------- tables
def test_hand_worked_example():
    # two outputs; every count below was worked out by hand
    docs = [[1, 2, 1, 2, 3], [1, 2, 3]]
    t = O.build_tables(docs, vocab=4, n_max=3, p_min=1)
    assert t.orders[2] == {(1,): {2: 3}, (2,): {1: 1, 3: 2}}
    assert t.orders[3] == {(1, 2): {1: 1, 3: 2}, (2, 1): {2: 1}}
    assert t.unigram.tolist() == [0, 3, 3, 2]
    assert t.fallback == 1                       # tokens 1 and 2 tie at 3: smallest id
    # pruning at 2 keeps only what occurs at least twice; a context left without successors vanishes
    t = O.build_tables(docs, vocab=4, n_max=3, p_min=2)
    assert t.orders[2] == {(1,): {2: 3}, (2,): {3: 2}}
    assert t.orders[3] == {(1, 2): {3: 2}}
    assert t.export(2).tolist() == [[1, 2, 3], [2, 3, 2]]
    assert t.export_contexts(2).tolist() == [[1, 3, 2, 3], [2, 2, 3, 2]]


def test_windows_do_not_span_outputs():
    t = O.build_tables([[5, 6], [7, 8]], vocab=9, n_max=3, p_min=1)
    assert t.orders[2] == {(5,): {6: 1}, (7,): {8: 1}}      # no (6, 7)
    assert t.orders[3] == {}


@pytest.mark.parametrize("D,ell,p_min", [(7, 12, 5), (4, 9, 5), (5, 6, 5), (1, 5, 1)])
def test_closed_form_distinct_sequence(D, ell, p_min):
    # D copies of one all-distinct sequence: every order-n window occurs exactly D times and there
    # are ell - n + 1 of them; all are kept iff D >= p_min.
    seq = list(range(100, 100 + ell))
    n_max = 5
    t = O.build_tables([seq] * D, vocab=200, n_max=n_max, p_min=p_min)
    for n in range(2, n_max + 1):
        ex = t.export(n)
        if D >= p_min:
            assert ex.shape[0] == ell - n + 1
            assert (ex[:, -1] == D).all()
            assert ex[:, :n].tolist() == [seq[i:i + n] for i in range(ell - n + 1)]
        else:
            assert ex.shape[0] == 0
    assert t.fallback == 100


def _random_docs(rng, n_docs, vocab, lo, hi):
    return [[rng.randrange(vocab) for _ in range(rng.randint(lo, hi))] for _ in range(n_docs)]


@pytest.mark.parametrize("seed", range(6))
def test_counting_invariants(seed):
    rng = random.Random(seed)
    vocab = rng.choice([2, 3, 8])
    docs = _random_docs(rng, rng.randint(1, 20), vocab, 0, 14)
    n_max = 4
    raw = O.build_tables(docs, vocab, n_max, p_min=1)
    for n in range(2, n_max + 1):
        total = sum(c for succ in raw.orders[n].values() for c in succ.values())
        assert total == sum(max(0, len(d) - n + 1) for d in docs)
    # every occurrence of u is followed by something unless it ends its output
    last = Counter(d[-1] for d in docs if d)
    for u in range(vocab):
        assert sum(raw.orders[2].get((u,), {}).values()) == raw.unigram[u] - last.get(u, 0)
    # marginalising an order-n table over its first token gives the order-(n-1) counts of windows
    # that are not at the start of an output
    for p_min in (2, 3):
        pruned = O.build_tables(docs, vocab, n_max, p_min)
        for n in range(2, n_max + 1):
            kept = {ctx + (x,): c for ctx, s in pruned.orders[n].items() for x, c in s.items()}
            full = {ctx + (x,): c for ctx, s in raw.orders[n].items() for x, c in s.items()}
            assert all(c >= p_min for c in kept.values())
            assert kept == {g: c for g, c in full.items() if c >= p_min}
    # building twice gives the same export
    again = O.build_tables(docs, vocab, n_max, 1)
    for n in range(2, n_max + 1):
        assert (again.export(n) == raw.export(n)).all()


@pytest.mark.parametrize("seed", range(4))
def test_sorted_counter_equals_definition(seed):
    rng = random.Random(100 + seed)
    vocab = rng.choice([2, 5, 300000])
    docs = _random_docs(rng, rng.randint(1, 30), vocab, 0, 12)
    tokens = np.array([t for d in docs for t in d], dtype=np.int32)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.int64)
    for n in range(2, 6):
        w, c = O.count_windows_sorted(tokens, off, n)
        ref = sorted(O.count_windows(docs, n).items())
        assert [tuple(r) for r in w.tolist()] == [g for g, _ in ref]
        assert c.tolist() == [v for _, v in ref]
    a = O.build_tables(docs, vocab, 4, 2)
    b = O.build_tables_flat(tokens, off, vocab, 4, 2)
    assert a.orders == b.orders and a.fallback == b.fallback and (a.unigram == b.unigram).all()


def test_sorted_counter_on_cfg1_corpus_and_bias_counts():
    import workload as W
    cfg = W.get_config("cfg1")
    tokens, off = W.make_corpus(cfg)
    docs = O.split_docs(tokens, off)
    assert len(docs) == cfg.n_docs and all(cfg.doc_len_lo <= len(d) <= cfg.doc_len_hi for d in docs)
    a = O.build_tables(docs, cfg.vocab, cfg.n_max, cfg.p_min)
    b = O.build_tables_flat(tokens, off, cfg.vocab, cfg.n_max, cfg.p_min)
    assert a.orders == b.orders and a.fallback == b.fallback
    assert sum(len(s) for s in a.orders[2].values()) > 100      # the workload has a typical set
    # the workload's LM-head bias is built from the same raw bigram counts
    raw = O.build_tables_flat(tokens, off, cfg.vocab, 2, 1)
    bias = W.bigram_bias_csr(tokens, off, cfg.vocab, cfg.bias_alpha)
    for u in (0, 7, 100, 511):
        succ = raw.orders[2].get((u,), {})
        lo, hi = bias["rowptr"][u], bias["rowptr"][u + 1]
        assert bias["col"][lo:hi].tolist() == sorted(succ)
        c1 = sum(succ.values())
        want = [8.0 * (np.log(succ[v] + 1.0) - np.log(c1 + 512.0)) for v in sorted(succ)]
        np.testing.assert_allclose(bias["val"][lo:hi], want, rtol=1e-6)
        np.testing.assert_allclose(bias["base"][u], -8.0 * np.log(c1 + 512.0), rtol=1e-6)


# ---------------------------------------------------------------- back-off and mixture
def _tables(n_max, orders, fallback=0):
    return O.NgramTables(n_max, 1, {n: orders.get(n, {}) for n in range(2, n_max + 1)}, None, fallback)


def test_backoff_descending_first_match():
    t = _tables(4, {2: {(3,): {9: 5}}, 3: {(2, 3): {8: 5}}, 4: {(1, 2, 3): {7: 5}}})
    assert O.backoff(t, [1, 2, 3]) == (4, {7: 5})
    assert O.backoff(t, [0, 2, 3]) == (3, {8: 5})         # order 4 misses, order 3 matches
    assert O.backoff(t, [0, 0, 3]) == (2, {9: 5})
    assert O.backoff(t, [0, 0, 0]) is None
    assert O.backoff(t, [3]) == (2, {9: 5})               # short history: only orders that fit
    assert O.backoff(t, []) is None


def test_pruned_context_backs_off():
    # (1,2)->x occurs but never 5 times: at p_min=5 the trigram context is gone, the bigram remains
    docs = [[1, 2, 3], [1, 2, 4], [9, 2, 3], [9, 2, 3], [9, 2, 3], [1, 2, 3]]
    t = O.build_tables(docs, vocab=10, n_max=3, p_min=5)
    assert O.backoff(t, [1, 2]) == (2, {3: 5})


def test_fallback_only_when_nothing_matches():
    corp = _tables(3, {2: {(1,): {2: 5}}}, fallback=42)
    ctx = O.context_tables([7, 8, 7], 3, 1)
    assert O.propose(corp, ctx, [0, 0], 49152) == 42
    assert O.propose(corp, ctx, [0, 1], 49152) == 2        # corpus only
    assert O.propose(corp, ctx, [0, 7], 49152) == 8        # context only
    assert O.propose(corp, None, [0, 7], 49152) == 42


def test_lambda_extremes_and_ties():
    corp = _tables(2, {2: {(1,): {5: 6, 4: 6, 9: 1}}}, fallback=0)
    ctx = O.context_tables([1, 9, 1, 9, 1, 3], 2, 1)          # after 1: 9 twice, 3 once
    assert O.propose(corp, ctx, [1], 65536) == 4             # pure corpus, tie 4/5 -> smallest
    assert O.propose(corp, ctx, [1], 0) == 9                 # pure context
    # lambda = 0.5: p(4)=p(5)=6/26, p(9)=1/26+2/3*... evaluate exactly
    p = O.mixture_probability(corp, ctx, [1], Fraction(1, 2))
    assert p[9] == Fraction(1, 2) * Fraction(1, 13) + Fraction(1, 2) * Fraction(2, 3)
    assert O.propose(corp, ctx, [1], 32768) == 9


@pytest.mark.parametrize("seed", range(20))
def test_propose_equals_exact_rational_argmax(seed):
    rng = random.Random(seed)
    vocab = 4
    docs = _random_docs(rng, 12, vocab, 2, 10)
    corp = O.build_tables(docs, vocab, 3, rng.choice([1, 2]))
    seq = [rng.randrange(vocab) for _ in range(rng.randint(1, 14))]
    ctx = O.context_tables(seq, 3, 1)
    for q16 in (1, 9000, 32768, 49152, 65535):
        lam = Fraction(q16, 65536)
        for hist in itertools.product(range(vocab), repeat=2):
            p = O.mixture_probability(corp, ctx, list(hist), lam)
            got = O.propose(corp, ctx, list(hist), q16)
            if not p:
                assert got == corp.fallback
            else:
                best = max(p.values())
                assert got == min(x for x, v in p.items() if v == best)


def test_context_successor_must_exist():
    # the current suffix has no successor yet, so it adds nothing to its own statistics
    ctx = O.context_tables([4, 5, 6, 4, 5], 3, 1)
    assert O.backoff(ctx, [4, 5]) == (3, {6: 1})
    assert O.backoff(O.context_tables([4, 5], 3, 1), [4, 5]) is None


def test_draft_worked_example():
    # corpus says 1->2->3->1..., context says 3 is followed by 7
    docs = [[1, 2, 3, 1, 2, 3, 1, 2, 3]] * 5
    corp = O.build_tables(docs, vocab=8, n_max=3, p_min=5)
    assert O.draft(corp, [5, 1], 4, 65536) == [2, 3, 1, 2]
    # lambda small: after (2,3) the context (3 -> 7 seen once via order 2) competes with the corpus;
    # context weight 0.9 on one-point distribution beats corpus 0.1
    got = O.draft(corp, [3, 7, 0, 2, 3], 2, 6554)
    assert got[0] == 7
    # drafts extend the running context but not the statistics: after 7 the context knows 7 -> 0
    assert got[1] == 0
    assert len(O.draft(corp, [6, 6, 6], 5, 49152)) == 5


@pytest.mark.parametrize("seed", range(6))
def test_lazy_tables_equal_the_full_tables(seed):
    """LazyTables (single-context counting for corpora too large for full tables) against the definition: every
    context of every order, contexts that do not occur, and whole drafts."""
    rng = random.Random(900 + seed)
    vocab = rng.choice([3, 6, 40])
    docs = [[rng.randrange(vocab) for _ in range(rng.randint(0, 25))] for _ in range(rng.choice([1, 5, 30]))]
    docs.append([1, 1, 1, 1, 2])
    n_max, p_min = rng.choice([2, 4, 5]), rng.choice([1, 2, 3])
    tokens = np.array([t for d in docs for t in d], dtype=np.int32)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.int64)
    full = O.build_tables(docs, vocab, n_max, p_min)
    lazy = O.LazyTables(tokens, off, vocab, n_max, p_min)
    assert lazy.fallback == full.fallback and (lazy.unigram == full.unigram).all()
    for n in range(2, n_max + 1):
        unpruned = O.count_windows(docs, n)
        contexts = {w[:n - 1] for w in unpruned} | {tuple(rng.randrange(vocab) for _ in range(n - 1)) for _ in range(30)}
        for ctx in contexts:
            assert (lazy.orders[n].get(ctx) or None) == (full.orders[n].get(ctx) or None), (n, ctx)
    for _ in range(20):
        seq = [rng.randrange(vocab) for _ in range(rng.randint(1, 30))]
        lam = rng.choice([0, 16384, 49152, 65536])
        assert O.draft(lazy, seq, 5, lam, 1) == O.draft(full, seq, 5, lam, 1)
