"""Test oracle (not part of the product path): the model-derived bigram drafter the paper compares against
(Related Work and Results, "TASC-spec": a bigram model that assigns each token its most probable next token
under the given model, obtained by taking the model's conditional distribution for every vocabulary element;
used alone and mixed with the context drafter).

next(x) = argmax_v logits(v | sequence = [x]) with the lowest index on ties: one forward of the one-token
sequence [x] at position 0 per vocabulary element.  As a draft source it is the point mass on next(x) after
context x: an order-2 table with C(x, next(x)) = 1 and T(x) = 1 and no higher orders, which is what the n-gram
counting definition gives for the pseudo-corpus of the V two-token outputs [x, next(x)].
"""
import numpy as np

from . import model as OM
from . import ngram as ON


def model_bigram(model, vocab=None):
    """int64[V]: the model's greedy next token after every single-token sequence."""
    V = model.cfg.vocab if vocab is None else vocab
    out = np.zeros(V, dtype=np.int64)
    for x in range(V):
        cache = model.new_cache(2)
        z = model.forward([x], cache, last_only=True)
        out[x] = int(OM.argmax_lowest(z)[0])
    return out


def bigram_margins(model, vocab=None):
    """float64[V]: gap between the two largest logits after every single-token sequence (tie diagnosis)."""
    V = model.cfg.vocab if vocab is None else vocab
    out = np.zeros(V)
    for x in range(V):
        z = model.forward([x], model.new_cache(2), last_only=True)[0]
        top2 = np.partition(z, -2)[-2:]
        out[x] = top2[1] - top2[0]
    return out


def bigram_tables(next_tok, vocab, n_max):
    """The drafter as tables: order 2 holds (x -> next(x), count 1) for every x; orders 3..n_max are empty
    (the context source still backs off from n_max)."""
    docs = [[x, int(next_tok[x])] for x in range(vocab)]
    return ON.build_tables(docs, vocab, n_max, 1)
