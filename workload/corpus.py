"""Synthetic task-output corpora and prompts.

A corpus stands in for C_task, the set of expected task outputs (paper,
"Task-Induced n-Grams Concentration"): a few thousand to a million short token
sequences whose n-gram distribution is concentrated on a small typical set.
Recipe: a pool of random phrases; every output is a concatenation of phrases
drawn i.i.d. from a bounded Zipf law over the pool, cut at a uniformly drawn
length; finally each token is replaced by a uniform token with probability
`noise`.
"""
import numpy as np

from .configs import WorkloadConfig

_PURPOSE = {"pool": 1, "doclen": 2, "phrases": 3, "noise": 4, "prompts": 5}


def _rng(seed: int, purpose: str, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | _PURPOSE[purpose], index]))


def make_corpus(cfg: WorkloadConfig):
    """Returns (tokens int32[T], doc_offsets int64[D+1])."""
    V, D = cfg.vocab, cfg.n_docs
    # phrase pool
    g = _rng(cfg.seed, "pool")
    plen = g.integers(cfg.phrase_len_lo, cfg.phrase_len_hi + 1, size=cfg.pool_size)
    poff = np.zeros(cfg.pool_size + 1, dtype=np.int64)
    np.cumsum(plen, out=poff[1:])
    ptok = g.integers(0, V, size=int(poff[-1]), dtype=np.int64).astype(np.int32)
    # bounded Zipf over phrase ranks 1..pool
    w = np.arange(1, cfg.pool_size + 1, dtype=np.float64) ** (-cfg.zipf_s)
    cdf = np.cumsum(w / w.sum())
    cdf[-1] = 1.0
    # document lengths
    dlen = _rng(cfg.seed, "doclen").integers(cfg.doc_len_lo, cfg.doc_len_hi + 1, size=D).astype(np.int64)
    doc_off = np.zeros(D + 1, dtype=np.int64)
    np.cumsum(dlen, out=doc_off[1:])
    T = int(doc_off[-1])
    # Every document draws its own phrases: document i owns the slice
    # [i*m, (i+1)*m) of one long i.i.d. stream of phrase ids, where m phrases
    # always suffice (shortest phrase length * m >= longest document).
    m = -(-cfg.doc_len_hi // cfg.phrase_len_lo)
    tokens = np.empty(T, dtype=np.int32)
    chunk = max(1, (1 << 22) // m)          # documents per batch: bounds the temporaries
    for d0 in range(0, D, chunk):
        d1 = min(D, d0 + chunk)
        nd = d1 - d0
        u = _rng(cfg.seed, "phrases", d0).random(nd * m)
        ids = np.searchsorted(cdf, u, side="left").astype(np.int64).reshape(nd, m)
        ids = np.minimum(ids, cfg.pool_size - 1)
        lens = plen[ids]                                   # [nd, m]
        ends = np.cumsum(lens, axis=1)                     # end offset of each phrase inside its doc
        starts = ends - lens
        want = dlen[d0:d1, None]
        take = np.clip(want - starts, 0, lens)             # tokens used from each phrase (last one truncated)
        flat_take = take.ravel()
        total = int(flat_take.sum())
        assert total == int(dlen[d0:d1].sum())
        # expand: for every used token, its index into the pool
        src0 = np.repeat(poff[ids.ravel()], flat_take)
        first = np.cumsum(flat_take) - flat_take           # output offset of each phrase
        within = np.arange(total, dtype=np.int64) - np.repeat(first, flat_take)
        tokens[doc_off[d0]:doc_off[d1]] = ptok[src0 + within]
    # token noise
    g = _rng(cfg.seed, "noise")
    step = 1 << 24
    for t0 in range(0, T, step):
        t1 = min(T, t0 + step)
        hit = g.random(t1 - t0) < cfg.noise
        rnd = g.integers(0, V, size=t1 - t0, dtype=np.int64).astype(np.int32)
        seg = tokens[t0:t1]
        seg[hit] = rnd[hit]
    return tokens, doc_off


def make_prompts(cfg: WorkloadConfig, batch: int = None, prompt_len: int = None):
    """Uniform random prompts, all of one length.  Returns (tokens int32[B*P], offsets int64[B+1])."""
    B = cfg.batch if batch is None else batch
    P = cfg.prompt_len if prompt_len is None else prompt_len
    toks = _rng(cfg.seed, "prompts").integers(0, cfg.vocab, size=B * P, dtype=np.int64).astype(np.int32)
    offs = np.arange(B + 1, dtype=np.int64) * P
    return toks, offs
