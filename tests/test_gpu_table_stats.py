"""tasc_ngram_entropy on the GPU against the oracle: entry count, total and coverage count bit-exact, the two
entropies within 1e-11 relative (fp64 sums in a different order)."""
import random
from fractions import Fraction

import numpy as np
import pytest

import workload as W
from oracle import ngram as ON
from oracle import table_stats as OS

pytestmark = pytest.mark.gpu

COVERAGES = [0, 1, 500000, 800000, 990000, 999999, 1000000]


def _check(T, ng, order, counts, label):
    for ppm in COVERAGES:
        got = T.tasc_ngram_entropy(ng, order, ppm)
        want = OS.table_stats(counts, Fraction(ppm, 1000000))
        assert got.n_entries == want["n_entries"], f"{label} order {order}: entries"
        assert got.total == want["total"], f"{label} order {order}: total"
        assert got.n_cover == want["n_cover"], f"{label} order {order} ppm {ppm}: cover {got.n_cover}, oracle {want['n_cover']}"
        assert abs(got.shannon - want["shannon"]) <= 1e-11 * max(1.0, want["shannon"]), f"{label} order {order}: shannon"
        assert abs(got.renyi2 - want["renyi2"]) <= 1e-11 * max(1.0, want["renyi2"]), f"{label} order {order}: renyi2"


@pytest.mark.parametrize("seed", range(6))
def test_entropy_tiny_random_corpora(seed):
    import paper_2602_24174_amd as T
    rng = random.Random(100 + seed)
    vocab = rng.choice([2, 5, 300, 151936])
    docs = [[rng.randrange(min(vocab, 5)) + (vocab - 5 if vocab > 5 and rng.random() < 0.3 else 0)
             for _ in range(rng.randint(0, 30))] for _ in range(rng.choice([1, 4, 60]))]
    if not any(docs):
        docs[0] = [1, 1, 0]
    tokens = np.array([t for d in docs for t in d], dtype=np.int32)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.int64)
    n_max, p_min = rng.choice([2, 4, 6]), rng.choice([1, 1, 3])
    print(f"seed {seed} vocab {vocab} docs {len(docs)} n_max {n_max} p_min {p_min}", flush=True)
    ng = T.tasc_ngram_build(tokens, off, vocab, n_max, p_min)
    ref = ON.build_tables(docs, vocab, n_max, p_min)
    _check(T, ng, 1, ref.unigram.tolist(), "tiny")
    for n in range(2, n_max + 1):
        _check(T, ng, n, ref.export(n)[:, n].tolist(), "tiny")


def test_entropy_counts_beyond_two_bytes_and_empty():
    """One bigram counted 200,000 times among rare ones: the select has to walk the high bytes; and the empty table."""
    import paper_2602_24174_amd as T
    rng = np.random.default_rng(4)
    heavy = np.zeros(200001, dtype=np.int32) + 7                       # 200,000 windows (7, 7)
    mid = np.tile(np.array([3, 4], dtype=np.int32), 300)               # (3, 4) x 300, (4, 3) x 299
    rare = rng.integers(8, 5000, size=4000).astype(np.int32)
    tokens = np.concatenate([heavy, mid, rare])
    off = np.array([0, heavy.size, heavy.size + mid.size, tokens.size], dtype=np.int64)
    ng = T.tasc_ngram_build(tokens, off, 5000, 2, 1)
    counts = ON.count_windows_sorted(tokens, off, 2)[1].tolist()
    assert max(counts) == 200000
    _check(T, ng, 2, counts, "heavy")
    _check(T, ng, 1, np.bincount(tokens, minlength=5000).tolist(), "heavy")
    empty = T.tasc_ngram_build(np.zeros(0, dtype=np.int32), np.zeros(1, dtype=np.int64), 16, 3, 1)
    for n in (1, 2, 3):
        g = T.tasc_ngram_entropy(empty, n, 800000)
        assert (g.n_entries, g.total, g.n_cover, g.shannon, g.renyi2) == (0, 0, 0, 0.0, 0.0)
    with pytest.raises(T.TascError):
        T.tasc_ngram_entropy(ng, 3, 800000)                            # order above n_max
    with pytest.raises(T.TascError):
        T.tasc_ngram_entropy(ng, 2, 1000001)


def test_entropy_full_config_corpus():
    """The 135M configuration's corpus (about 8 M tokens), unpruned: bigram and 4-gram distributions and the tokens."""
    import paper_2602_24174_amd as T
    cfg = W.get_config("cfg2")
    tok, off = W.make_corpus(cfg)
    ng = T.tasc_ngram_build(tok, off, cfg.vocab, cfg.n_max, 1)
    _check(T, ng, 1, np.bincount(tok, minlength=cfg.vocab).tolist(), "cfg2")
    for n in (2, cfg.n_max):
        _check(T, ng, n, ON.count_windows_sorted(tok, off, n)[1].tolist(), "cfg2")
        g = T.tasc_ngram_entropy(ng, n, 800000)
        print(f"cfg2 order {n}: {g.n_entries} distinct, H {g.shannon:.4f} nats, H2 {g.renyi2:.4f} nats, "
              f"{g.n_cover} n-grams reach 80 % of the mass", flush=True)
