"""CPU oracle for the n-gram drafter of TASC-spec.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path never does.  It shares no code with the HIP
library.  Integers only; every function cites the passage of the paper it
follows (section "Proposed Method: TASC-spec" of "n-Gram Speculative Decoding
Method", called [M] below, and the hyper-parameters given in the Results
section, "TASC-spec: Inference-Time Acceleration", called [R]).

Readings taken where the paper is silent (all listed in the design notes):
  * M_n maps an (n-1)-token context to its n-th token, n = 2..n_max; n = 1 is
    the "most frequent token" fallback of [M].
  * the pruning threshold is an absolute count, an element is kept iff
    count >= p_min ([M] "frequency below a prescribed threshold", [R] p_min=5).
  * p(x | c) of a pruned model is normalised over the retained successors.
  * windows never span two outputs of the corpus.
  * the prompt/context drafter is built "similarly" ([M]) from the tokens
    available so far (prompt and committed output) with its own threshold.
  * each source backs off on its own to its first matching order and
    contributes its whole conditional distribution there; the proposal is the
    argmax of the mixture ([R] beam size 1), ties to the smallest token id;
    the fallback fires only if neither source matches.

Pinned by tests/test_oracle_ngram.py (hand-worked example, closed forms,
counting invariants, exact rational evaluation of the mixture formula).
"""
from collections import Counter
from fractions import Fraction

import numpy as np


class NgramTables:
    """orders[n][ctx][x] = retained count of the n-gram ctx + (x,), len(ctx) = n - 1."""

    def __init__(self, n_max, p_min, orders, unigram, fallback):
        self.n_max = n_max
        self.p_min = p_min
        self.orders = orders
        self.unigram = unigram
        self.fallback = fallback

    def export(self, n):
        """Canonical dump of order n: rows (t_1..t_n, count) sorted by the n tokens."""
        rows = [ctx + (x, c) for ctx, succ in self.orders[n].items() for x, c in succ.items()]
        rows.sort()
        return np.array(rows, dtype=np.int64).reshape(len(rows), n + 1)

    def export_contexts(self, n):
        """Rows (c_1..c_{n-1}, T, top, top_count) sorted by context: T = sum of retained successor
        counts, top = most frequent retained successor (smallest id among equals)."""
        rows = []
        for ctx, succ in self.orders[n].items():
            top = min(succ, key=lambda x: (-succ[x], x))
            rows.append(ctx + (sum(succ.values()), top, succ[top]))
        rows.sort()
        return np.array(rows, dtype=np.int64).reshape(len(rows), n + 2)


def count_windows(docs, n):
    """[M]: "n-gram frequencies in C_task" -- the number of times every n-token window occurs inside
    one output.  The definition, written out."""
    c = Counter()
    for doc in docs:
        doc = [int(t) for t in doc]
        for i in range(len(doc) - n + 1):
            c[tuple(doc[i:i + n])] += 1
    return c


def count_windows_sorted(tokens, doc_off, n, starts=None):
    """Same counts as count_windows for a flat corpus, by sorting all windows (for corpora too large
    for a Python Counter).  Returns (windows int64[R, n] sorted, counts int64[R]).
    `starts` restricts the count to the windows beginning at these positions (sampled checks)."""
    tokens = np.asarray(tokens)
    doc_off = np.asarray(doc_off, dtype=np.int64)
    if starts is None:
        starts = window_starts(doc_off, n)
    if starts.size == 0:
        return np.zeros((0, n), dtype=np.int64), np.zeros(0, dtype=np.int64)
    cols = [tokens[starts + j].astype(np.int64) for j in range(n)]
    order = np.lexsort(tuple(reversed(cols)))          # primary key = first token
    w = np.stack([c[order] for c in cols], axis=1)
    new = np.ones(w.shape[0], dtype=bool)
    new[1:] = np.any(w[1:] != w[:-1], axis=1)
    first = np.flatnonzero(new)
    counts = np.diff(np.append(first, w.shape[0]))
    return w[first], counts.astype(np.int64)


def window_starts(doc_off, n):
    """Start positions of all n-token windows that lie inside one document."""
    doc_off = np.asarray(doc_off, dtype=np.int64)
    lens = np.diff(doc_off)
    nwin = np.maximum(lens - n + 1, 0)
    total = int(nwin.sum())
    first = np.cumsum(nwin) - nwin
    return np.repeat(doc_off[:-1], nwin) + (np.arange(total, dtype=np.int64) - np.repeat(first, nwin))


def _tables_from_counts(items, n, p_min):
    """[M]: prune M_n by dropping the elements whose frequency is below p_min."""
    table = {}
    for win, c in items:
        if c >= p_min:
            table.setdefault(tuple(win[:n - 1]), {})[int(win[n - 1])] = int(c)
    return table


def build_tables(docs, vocab, n_max, p_min):
    """[M]: the drafter is the collection M_n, n <= n_max, each from the n-gram frequencies of the
    corpus, pruned at p_min; the unigram model only supplies the most frequent token."""
    orders = {}
    for n in range(2, n_max + 1):
        orders[n] = _tables_from_counts(count_windows(docs, n).items(), n, p_min)
    unigram = np.zeros(vocab, dtype=np.int64)
    for doc in docs:
        for t in doc:
            unigram[int(t)] += 1
    fallback = int(np.argmax(unigram))                 # first maximum = smallest id among equals
    return NgramTables(n_max, p_min, orders, unigram, fallback)


def build_tables_flat(tokens, doc_off, vocab, n_max, p_min):
    """build_tables for a flat (tokens, doc_offsets) corpus of any size, by sorting."""
    orders = {}
    for n in range(2, n_max + 1):
        w, c = count_windows_sorted(tokens, doc_off, n)
        keep = c >= p_min
        orders[n] = _tables_from_counts(zip(w[keep].tolist(), c[keep].tolist()), n, 0)
    unigram = np.bincount(np.asarray(tokens), minlength=vocab).astype(np.int64)
    return NgramTables(n_max, p_min, orders, unigram, int(np.argmax(unigram)))


class _LazyOrder:
    """M_n of a large corpus, one context at a time: get(ctx) counts the successors of ctx when it is first asked
    for, by the definition ([M]: the n-gram frequencies of the corpus, pruned at p_min), over the positions where the
    context's first token occurs."""

    def __init__(self, owner, n):
        self.owner, self.n, self.seen = owner, n, {}

    def get(self, ctx, default=None):
        ctx = tuple(int(t) for t in ctx)
        if ctx not in self.seen:
            self.seen[ctx] = self.owner.successors(ctx)
        return self.seen[ctx] or default


class LazyTables:
    """The same object as build_tables_flat returns, for corpora whose full tables are too large to build in a test:
    the tables of every order answer single-context queries on demand.  Only `orders[n].get(ctx)`, `unigram`,
    `fallback`, `n_max` and `p_min` exist (what backoff / propose / draft use)."""

    def __init__(self, tokens, doc_off, vocab, n_max, p_min):
        self.tokens = np.asarray(tokens)
        self.doc_off = np.asarray(doc_off, dtype=np.int64)
        self.n_max, self.p_min = n_max, p_min
        self.by_token = np.argsort(self.tokens, kind="stable").astype(np.int32)          # positions grouped by token
        self.unigram = np.bincount(self.tokens, minlength=vocab).astype(np.int64)
        self.first = np.concatenate([[0], np.cumsum(self.unigram)])                     # group of token t: [first[t], first[t+1])
        self.fallback = int(np.argmax(self.unigram))
        self.orders = {n: _LazyOrder(self, n) for n in range(2, n_max + 1)}

    def successors(self, ctx):
        """{x: count} over the windows ctx + (x,) that lie inside one output, counts below p_min dropped."""
        n = len(ctx) + 1
        t0 = ctx[0]
        if t0 < 0 or t0 + 1 >= self.first.shape[0]:
            return {}
        pos = self.by_token[self.first[t0]:self.first[t0 + 1]].astype(np.int64)
        doc_end = self.doc_off[np.searchsorted(self.doc_off, pos, side="right")]        # end of the output holding pos
        pos = pos[pos + n <= doc_end]
        for j in range(1, n - 1):
            pos = pos[self.tokens[pos + j] == ctx[j]]
        succ = Counter(self.tokens[pos + n - 1].tolist())
        return {int(x): int(c) for x, c in succ.items() if c >= self.p_min}


def split_docs(tokens, doc_off):
    return [tokens[doc_off[i]:doc_off[i + 1]] for i in range(len(doc_off) - 1)]


def context_tables(seq, n_max, p_min_ctx):
    """[M]: the prompt drafter "is obtained similarly to p_corp, but it is based on the available
    context": the same construction over the single sequence of available tokens."""
    orders = {n: _tables_from_counts(count_windows([seq], n).items(), n, p_min_ctx) for n in range(2, n_max + 1)}
    return NgramTables(n_max, p_min_ctx, orders, None, None)


def backoff(tables, w):
    """[M]: query (M_n) in descending order of n and take the first match.  Returns (n, successors)
    for the longest suffix of w that is a retained context, or None."""
    for n in range(min(tables.n_max, len(w) + 1), 1, -1):
        succ = tables.orders[n].get(tuple(int(t) for t in w[len(w) - (n - 1):]))
        if succ:
            return n, succ
    return None


def propose(corp, ctx, w, lambda_q16):
    """[M]: p_mixed(x|c) = lambda p_corp(x|c) + (1 - lambda) p_prompt(x|c); the proposal is its argmax.
    With q = lambda * 65536 an integer, the score
        q * C_corp(x) * T_ctx + (65536 - q) * C_ctx(x) * T_corp
    is p_mixed(x|c) times the positive constant 65536 * T_corp * T_ctx, so the argmax is exact.
    A source with weight 0 is left out; with no source matching, the most frequent token."""
    q = int(lambda_q16)
    qb = 65536 - q
    mc = backoff(corp, w) if q > 0 else None
    mx = backoff(ctx, w) if (qb > 0 and ctx is not None) else None
    if mc is None and mx is None:
        return corp.fallback
    if mx is None:
        score = dict(mc[1])
    elif mc is None:
        score = dict(mx[1])
    else:
        sc, sx = mc[1], mx[1]
        tc, tx = sum(sc.values()), sum(sx.values())
        score = {x: q * sc.get(x, 0) * tx + qb * sx.get(x, 0) * tc for x in set(sc) | set(sx)}
    return min(score, key=lambda x: (-score[x], x))


def mixture_probability(corp, ctx, w, lam: Fraction):
    """The mixture formula of [M] evaluated in exact rationals (used by the tests to pin `propose`)."""
    out = {}
    mc, mx = backoff(corp, w), backoff(ctx, w)
    for m, weight in ((mc, lam), (mx, 1 - lam)):
        if m is None:
            continue
        t = sum(m[1].values())
        for x, c in m[1].items():
            out[x] = out.get(x, Fraction(0)) + weight * Fraction(c, t)
    return out


def draft(corp, committed, k, lambda_q16, p_min_ctx=1, use_context=True):
    """k proposals in a row, each appended to the running context ([M]; draft-then-verify of the
    "Speculative Decoding" subsection).  The context statistics cover the committed tokens only."""
    committed = [int(t) for t in committed]
    ctx = context_tables(committed, corp.n_max, p_min_ctx) if use_context else None
    w = list(committed)
    out = []
    for _ in range(k):
        x = propose(corp, ctx, w, lambda_q16)
        out.append(x)
        w.append(x)
    return out
