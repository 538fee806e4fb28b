"""Test oracle (not part of the product path): the counting core of the tokenizer-enrichment scheme, without
the prefix-collision filter.

Written from the paper's "Enriching the Tokenizer" subsection: the merge reward f_merge(t^n) = freq(t^n) (n - 1)
(its equation) and the loop of its Algorithm "Tokenizer Enrichment" with the PCS test always passing: starting
from the base vocabulary, at every step collect the token n-grams (2 <= n <= n_max) of the corpus as currently
tokenised, take the one with the largest reward, add it to the vocabulary as one new token and re-tokenise the
corpus with it; stop at the token budget M (or when the corpus holds no n-gram any more).

Readings where the paper is silent: freq = the number of windows, inside one output, equal to the n-gram (the same
count the drafter's tables use); reward ties go to the shorter n-gram, then to the lexicographically smallest
token tuple; the new token gets the next free id; re-tokenising replaces occurrences left to right without overlap
inside each output (as a BPE merge does).
"""
from collections import Counter


def ngram_counts(docs, n_max):
    """Counter over all n-grams, 2 <= n <= n_max: windows inside one output."""
    c = Counter()
    for doc in docs:
        for n in range(2, n_max + 1):
            for i in range(len(doc) - n + 1):
                c[tuple(doc[i:i + n])] += 1
    return c


def best_merge(counts):
    """(n-gram, freq) maximising freq (n - 1); ties: shorter first, then the smallest tuple.  None if empty."""
    best = None
    for g, f in counts.items():
        key = (-f * (len(g) - 1), len(g), g)
        if best is None or key < best[0]:
            best = (key, g, f)
    return None if best is None else (best[1], best[2])


def replace_ngram(doc, g, new_id):
    """Left-to-right, non-overlapping replacement of the n-gram g by the single token new_id."""
    out, i, n = [], 0, len(g)
    while i < len(doc):
        if tuple(doc[i:i + n]) == g:
            out.append(new_id)
            i += n
        else:
            out.append(doc[i])
            i += 1
    return out


def enrich(docs, vocab, n_max, budget):
    """Returns (merges, docs_out, lengths): merges[i] = (n-gram over the vocabulary at step i, its freq, new id);
    lengths[i] = corpus length in tokens before merge i (lengths[-1]: after the last)."""
    docs = [[int(t) for t in d] for d in docs]
    merges, lengths = [], [sum(len(d) for d in docs)]
    for i in range(budget):
        pick = best_merge(ngram_counts(docs, n_max))
        if pick is None:
            break
        g, f = pick
        new_id = vocab + i
        docs = [replace_ngram(d, g, new_id) for d in docs]
        merges.append((g, f, new_id))
        lengths.append(sum(len(d) for d in docs))
    return merges, docs, lengths


def expand(docs, merges, vocab):
    """Undo the merges: every added token back to base-vocabulary tokens (the enrichment is lossless)."""
    table = {}
    for g, _, new_id in merges:
        flat = []
        for t in g:
            flat.extend(table.get(t, [t]))
        table[new_id] = flat
    return [[b for t in d for b in table.get(t, [t])] for d in docs]
