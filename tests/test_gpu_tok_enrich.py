"""tasc_tok_enrich on the GPU against the oracle: merges, frequencies, new ids, corpus lengths, the re-tokenised
corpus and its boundaries, all bit-exact (integers only)."""
import random

import numpy as np
import pytest

import workload as W
from oracle import tok_enrich as OT
from test_oracle_tok_enrich import load_example

pytestmark = pytest.mark.gpu


def _run_and_compare(T, docs, vocab, n_max, budget, device=False):
    import torch
    tokens = np.array([t for d in docs for t in d], dtype=np.int32)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.int64)
    src = torch.from_numpy(tokens).cuda() if device else tokens
    merges, out, out_off, lens = T.tasc_tok_enrich(src, off, vocab, n_max, budget)
    out = out.cpu().numpy() if device else out
    want_m, want_docs, want_l = OT.enrich(docs, vocab, n_max, budget)
    assert merges == want_m
    assert lens.tolist() == want_l
    assert out_off.tolist() == np.cumsum([0] + [len(d) for d in want_docs]).tolist()
    assert out.tolist() == [t for d in want_docs for t in d]
    return merges


def test_worked_example_and_edges():
    import paper_2602_24174_amd as T
    vocab, n_max, budget, docs, merges, lengths, out = load_example()
    assert _run_and_compare(T, docs, vocab, n_max, budget) == merges
    _run_and_compare(T, [[7, 7, 7, 7, 7]], 8, 2, 1)                    # self-overlapping n-gram
    _run_and_compare(T, [[7] * 41, [], [7] * 4, [7, 7, 3, 7, 7, 7]], 8, 3, 4, device=True)
    _run_and_compare(T, [[1, 2], [3]], 4, 3, 10)                       # runs out of n-grams before the budget
    _run_and_compare(T, [[], [5]], 6, 2, 3)                            # nothing to merge
    _run_and_compare(T, [[2, 1, 2, 1, 2, 1, 2], [1, 2, 1, 2, 1]], 3, 8, 3)   # (1,2,1) overlaps itself; n_max 8
    _run_and_compare(T, [[0, 1, 0, 1]], 2, 2, 0)                       # budget 0
    with pytest.raises(T.TascError):
        T.tasc_tok_enrich(np.array([0, 5], dtype=np.int32), np.array([0, 2]), 4, 2, 1)      # token outside the vocabulary
    with pytest.raises(T.TascError):
        T.tasc_tok_enrich(np.array([0, 1], dtype=np.int32), np.array([0, 2]), 1 << 20, 8, 1)  # key too wide


@pytest.mark.parametrize("seed", range(6))
def test_random_corpora(seed):
    import paper_2602_24174_amd as T
    rng = random.Random(40 + seed)
    vocab = rng.choice([2, 3, 7, 50000])
    n_max = rng.choice([2, 3, 4, 6])
    lo = vocab - min(vocab, 4)
    docs = [[lo + rng.randrange(min(vocab, 4)) for _ in range(rng.randint(0, 60))] for _ in range(rng.choice([1, 5, 80]))]
    print(f"seed {seed}: vocab {vocab} n_max {n_max} docs {len(docs)}", flush=True)
    _run_and_compare(T, docs, vocab, n_max, rng.choice([1, 5, 12]), device=bool(seed & 1))


def test_zipf_phrase_corpus_spans_scan_blocks():
    """A config-1-style corpus of about 38,000 tokens (several 4096-element scan blocks, ragged tail), 12 merges."""
    import paper_2602_24174_amd as T
    cfg = W.get_config("cfg1").scaled(n_docs=600)
    tok, off = W.make_corpus(cfg)
    docs = [tok[off[d]:off[d + 1]].tolist() for d in range(cfg.n_docs)]
    merges = _run_and_compare(T, docs, cfg.vocab, 4, 12, device=True)
    print("first merges:", merges[:4], flush=True)
