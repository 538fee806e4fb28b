"""Pins of the tokenizer-enrichment oracle (CPU only): a hand-worked example, the BPE special case written a
different way, and invariants checked by brute force."""
import os
import random
import re

from oracle import tok_enrich as OT

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tok_enrich_worked_example.txt")


def load_example(path=GOLDEN):
    docs, merges, out = [], [], []
    for ln in open(path):
        f = ln.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "vocab":
            vocab, n_max, budget = int(f[1]), int(f[3]), int(f[5])
        elif f[0] == "doc":
            docs.append([int(x) for x in f[1:]])
        elif f[0] == "merge":
            merges.append((tuple(int(x) for x in f[5:]), int(f[3]), int(f[1])))
        elif f[0] == "lengths":
            lengths = [int(x) for x in f[1:]]
        elif f[0] == "out":
            out.append([int(x) for x in f[1:]])
    return vocab, n_max, budget, docs, merges, lengths, out


def test_worked_example():
    vocab, n_max, budget, docs, merges, lengths, out = load_example()
    m, d, l = OT.enrich(docs, vocab, n_max, budget)
    assert m == merges and d == out and l == lengths


def test_self_overlapping_ngram_and_exhaustion():
    # (7,7) occurs in 4 windows of [7 7 7 7 7] but only two disjoint copies can be replaced, left to right
    m, d, l = OT.enrich([[7, 7, 7, 7, 7]], 8, 2, 1)
    assert m == [((7, 7), 4, 8)] and d == [[8, 8, 7]] and l == [5, 3]
    # the loop ends when no n-gram is left, whatever the budget
    m, d, l = OT.enrich([[1, 2], [3]], 4, 3, 10)
    assert m == [((1, 2), 1, 4)] and d == [[4], [3]] and l == [3, 2]
    assert OT.enrich([[], [5]], 6, 2, 3) == ([], [[], [5]], [1])


def _bpe_by_strings(words, n_merges, vocab):
    """Byte-pair merges learnt the textbook way on space-separated symbol strings with a regex replace
    (pair counts over adjacent symbols; most frequent pair; ties: smallest pair of ids)."""
    corpus = [" ".join(str(t) for t in w) for w in words]
    merges, next_id = [], vocab
    for _ in range(n_merges):
        pairs = {}
        for s in corpus:
            sym = s.split()
            for a, b in zip(sym, sym[1:]):
                pairs[(int(a), int(b))] = pairs.get((int(a), int(b)), 0) + 1
        if not pairs:
            break
        top = max(pairs.values())
        a, b = min(p for p, c in pairs.items() if c == top)
        pat = re.compile(r"(?<!\S)" + f"{a} {b}" + r"(?!\S)")
        corpus = [pat.sub(str(next_id), s) for s in corpus]
        merges.append(((a, b), top, next_id))
        next_id += 1
    return merges, [[int(t) for t in s.split()] for s in corpus]


def test_n_max_2_is_bpe():
    rng = random.Random(3)
    for _ in range(25):
        words = [[rng.randrange(4) for _ in range(rng.randint(1, 12))] for _ in range(rng.randint(1, 6))]
        m, d, _ = OT.enrich(words, 4, 2, 5)
        bm, bd = _bpe_by_strings(words, 5, 4)
        assert m == bm and d == bd


def test_invariants_random():
    rng = random.Random(8)
    for _ in range(30):
        vocab, n_max = rng.choice([2, 3, 6]), rng.choice([2, 3, 4, 5])
        docs = [[rng.randrange(vocab) for _ in range(rng.randint(0, 20))] for _ in range(rng.randint(1, 5))]
        m, d, l = OT.enrich(docs, vocab, n_max, 6)
        assert OT.expand(d, m, vocab) == docs                         # lossless
        assert all(a > b for a, b in zip(l, l[1:]))                   # every merge shortens the corpus
        cur = [list(x) for x in docs]
        for i, (g, f, new_id) in enumerate(m):
            counts = OT.ngram_counts(cur, n_max)
            assert counts[g] == f and new_id == vocab + i
            assert all(c * (len(h) - 1) <= f * (len(g) - 1) for h, c in counts.items())   # maximal reward
            cur = [OT.replace_ngram(x, g, new_id) for x in cur]
            # the corpus shrinks by (n - 1) per replaced copy, and no copy of g is left
            assert l[i] - l[i + 1] == (len(g) - 1) * sum(x.count(new_id) for x in cur)
            assert OT.ngram_counts(cur, n_max)[g] == 0
        assert cur == d
