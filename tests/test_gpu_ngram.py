"""GPU n-gram tables and drafts against the CPU oracle: bit-exact."""
import random

import numpy as np
import pytest

import workload as W
from oracle import ngram as ON

pytestmark = pytest.mark.gpu


def _compare_tables(T, ng, ref, n_max, vocab):
    for n in range(2, n_max + 1):
        rows, counts = T.tasc_ngram_export(ng, n)
        want = ref.export(n)
        assert rows.shape[0] == want.shape[0], f"order {n}: {rows.shape[0]} rows, oracle {want.shape[0]}"
        assert (rows.astype(np.int64) == want[:, :n]).all()
        assert (counts.astype(np.int64) == want[:, n]).all()
        ctx, total, top, topc = T.tasc_ngram_export_contexts(ng, n)
        wc = ref.export_contexts(n)
        assert ctx.shape[0] == wc.shape[0]
        assert (ctx.astype(np.int64) == wc[:, :n - 1]).all()
        assert (total.astype(np.int64) == wc[:, n - 1]).all()
        assert (top.astype(np.int64) == wc[:, n]).all()
        assert (topc.astype(np.int64) == wc[:, n + 1]).all()
    fb, uni = T.tasc_ngram_unigram(ng, vocab)
    assert fb == ref.fallback
    assert (uni.astype(np.int64) == ref.unigram).all()


@pytest.mark.parametrize("seed", range(8))
def test_tables_tiny_random_corpora(seed):
    import paper_2602_24174_amd as T
    rng = random.Random(seed)
    vocab = rng.choice([2, 3, 8, 151936])
    n_docs = rng.choice([1, 3, 40])
    docs = [[rng.randrange(min(vocab, 6)) + (vocab - 6 if vocab > 6 and rng.random() < 0.5 else 0)
             for _ in range(rng.randint(0, 14))] for _ in range(n_docs)]
    if not any(docs):
        docs[0] = [1, 1, 1]
    tokens = np.array([t for d in docs for t in d], dtype=np.int32)
    off = np.cumsum([0] + [len(d) for d in docs]).astype(np.int64)
    n_max = rng.choice([2, 3, 5, 7])
    p_min = rng.choice([1, 2, 3])
    print(f"seed {seed} vocab {vocab} docs {n_docs} n_max {n_max} p_min {p_min}", flush=True)
    ng = T.tasc_ngram_build(tokens, off, vocab, n_max, p_min)
    ref = ON.build_tables(docs, vocab, n_max, p_min)
    _compare_tables(T, ng, ref, n_max, vocab)


def test_tables_empty_corpus_and_device_input():
    import torch
    import paper_2602_24174_amd as T
    ng = T.tasc_ngram_build(np.zeros(0, dtype=np.int32), np.zeros(1, dtype=np.int64), 16, 3, 1)
    for n in (2, 3):
        assert T.tasc_ngram_export(ng, n)[0].shape[0] == 0
    # device-resident corpus gives the same tables as a host one
    cfg = W.get_config("cfg1").scaled(n_docs=200)
    tok, off = W.make_corpus(cfg)
    a = T.tasc_ngram_build(tok, off, cfg.vocab, 3, 2)
    b = T.tasc_ngram_build(torch.from_numpy(tok).cuda(), off, cfg.vocab, 3, 2)
    for n in (2, 3):
        ra, ca = T.tasc_ngram_export(a, n)
        rb, cb = T.tasc_ngram_export(b, n)
        assert (ra == rb).all() and (ca == cb).all()


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_tables_full_config(name):
    import paper_2602_24174_amd as T
    cfg = W.get_config(name)
    tok, off = W.make_corpus(cfg)
    print(f"{name}: corpus {tok.shape[0]} tokens", flush=True)
    ng = T.tasc_ngram_build(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    st = T.tasc_ngram_get_stats(ng)
    print(f"build {st.build_ms:.2f} ms, count {st.count_ms:.2f} ms, kept {list(st.kept)[2:cfg.n_max + 1]}", flush=True)
    ref = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    _compare_tables(T, ng, ref, cfg.n_max, cfg.vocab)
    for n in range(2, cfg.n_max + 1):
        assert st.windows[n] == int(np.maximum(np.diff(off) - n + 1, 0).sum())


def test_build_rejects_bad_arguments():
    import paper_2602_24174_amd as T
    tok = np.array([1, 2, 3, 4], dtype=np.int32)
    off = np.array([0, 4], dtype=np.int64)
    for kw in (dict(vocab=8, n_max=1, p_min=1), dict(vocab=8, n_max=9, p_min=1), dict(vocab=8, n_max=3, p_min=0),
               dict(vocab=4, n_max=3, p_min=1),            # token 4 outside [0, 4)
               dict(vocab=1 << 20, n_max=7, p_min=1)):     # 7 x 20 bits > 128
        with pytest.raises(T.TascError) as e:
            T.tasc_ngram_build(tok, off, **kw)
        assert e.value.status == -1
    with pytest.raises(T.TascError):
        T.tasc_ngram_build(tok, np.array([0, 3, 2], dtype=np.int64), 8, 3, 1)


@pytest.mark.parametrize("lam,p_min_ctx", [(49152, 1), (65536, 1), (0, 1), (32768, 2), (9000, 1)])
def test_drafts_match_oracle(lam, p_min_ctx):
    """Drafts for sequences with real structure: corpus documents with noise, fed as 'prompts'."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    cfg = W.get_config("cfg1").scaled(batch=12, gen_len=8)
    rig = Rig(cfg, max_rows=16)
    tok, off = rig.corpus
    ref = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    rng = np.random.default_rng(lam + p_min_ctx)
    prompts = []
    for b in range(cfg.batch):
        d = rng.integers(0, cfg.n_docs)
        p = tok[off[d]:off[d + 1]].copy()[:rng.integers(1, 60)]
        if b % 3 == 0:
            p = np.concatenate([p, p])[:64]            # repeated text: the context source has matches
        if b == 5:
            p = np.full(40, 7, dtype=np.int32)         # one token repeated: the longest successor lists
        prompts.append(p.astype(np.int32))
    flat = np.concatenate(prompts)
    poff = np.cumsum([0] + [len(p) for p in prompts]).astype(np.int64)
    T.tasc_session_prefill(rig.model, rig.session, flat, poff, cfg.gen_len)
    for k in (1, 4, 7):
        params = T.spec_params(k, lam, p_min_ctx, 1)
        drafts = torch.zeros((cfg.batch, k), dtype=torch.int32, device="cuda")
        T.tasc_draft(rig.ng, rig.session, params, drafts)
        got = drafts.cpu().numpy()
        for b in range(cfg.batch):
            committed = T.tasc_session_get_tokens(rig.session, b)
            assert (committed[:len(prompts[b])] == prompts[b]).all() and len(committed) == len(prompts[b]) + 1
            want = ON.draft(ref, committed, k, lam, p_min_ctx)
            assert got[b].tolist() == want, f"sequence {b}, k {k}: {got[b].tolist()} vs oracle {want}"


@pytest.mark.parametrize("lam", [65536, 49152, 16384, 0])
def test_drafts_wide_keys_match_oracle(lam):
    """Vocabulary 151,936 and n_max 5: contexts of 4 tokens are 72-bit keys, full 5-grams 90 bits, so every probe of the
    two highest orders goes through the high key word.  Corpus documents (with noise) as prompts, repeated text, a run
    of one token; drafts bit-exact against the oracle at four mixture weights."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    cfg = W.get_config("cfg1").scaled(vocab=151936, n_max=5, n_docs=3000, batch=12, gen_len=8, prompt_len=96)
    rig = Rig(cfg, max_rows=16)
    tok, off = rig.corpus
    assert int(tok.max()) >= 1 << 17                       # tokens that need all 18 bits
    ref = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    assert len(ref.orders[5]) > 100 and len(ref.orders[4]) > 100
    rng = np.random.default_rng(lam + 17)
    prompts = []
    for b in range(cfg.batch):
        d = rng.integers(0, cfg.n_docs)
        p = tok[off[d]:off[d + 1]].copy()[:rng.integers(6, 90)]
        if b % 3 == 0:
            p = np.concatenate([p, p])[:96]                # repeated text: the context source matches at order 5
        if b == 5:
            p = np.full(50, 151935, dtype=np.int32)        # a run of the largest token id
        if b == 7:
            p = np.concatenate([p[:20], np.array([131072, 151935, 131073, 262143 % 151936], dtype=np.int32), p[:20]])
        prompts.append(p.astype(np.int32))
    flat = np.concatenate(prompts)
    poff = np.cumsum([0] + [len(p) for p in prompts]).astype(np.int64)
    T.tasc_session_prefill(rig.model, rig.session, flat, poff, cfg.gen_len)
    matched_high = 0
    for k in (1, 5, 8):
        params = T.spec_params(k, lam, 1, 1)
        drafts = torch.zeros((cfg.batch, k), dtype=torch.int32, device="cuda")
        T.tasc_draft(rig.ng, rig.session, params, drafts)
        got = drafts.cpu().numpy()
        for b in range(cfg.batch):
            committed = T.tasc_session_get_tokens(rig.session, b)
            want = ON.draft(ref, committed, k, lam, 1)
            assert got[b].tolist() == want, f"lambda {lam} sequence {b}, k {k}: {got[b].tolist()} vs oracle {want}"
            m = ON.backoff(ref, [int(t) for t in committed])
            matched_high += m is not None and m[0] >= 4
    if lam > 0:
        assert matched_high > 0, "no sequence reached a corpus context of 3+ tokens: the wide keys went untested"


def test_drafts_long_single_token_run():
    """A sequence that is one token repeated 3,900 times (every position matches the suffix at every order: the longest
    successor list a sequence can have), one that alternates two tokens, and one long copy of corpus text: drafts equal
    the oracle's."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    cfg = W.get_config("cfg1").scaled(batch=3, gen_len=8, prompt_len=3900, n_max=4)
    rig = Rig(cfg, max_rows=64)
    tok, off = rig.corpus
    ref = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    prompts = [np.full(3900, 11, dtype=np.int32), np.tile(np.array([5, 9], dtype=np.int32), 1950),
               np.tile(tok[off[3]:off[4]], 80)[:3900].astype(np.int32)]
    flat = np.concatenate(prompts)
    poff = np.cumsum([0] + [len(p) for p in prompts]).astype(np.int64)
    T.tasc_session_prefill(rig.model, rig.session, flat, poff, cfg.gen_len)
    for lam, p_min_ctx in ((49152, 1), (0, 1), (32768, 3000)):
        for k in (1, 8):
            drafts = torch.zeros((cfg.batch, k), dtype=torch.int32, device="cuda")
            T.tasc_draft(rig.ng, rig.session, T.spec_params(k, lam, p_min_ctx, 1), drafts)
            got = drafts.cpu().numpy()
            for b in range(cfg.batch):
                committed = T.tasc_session_get_tokens(rig.session, b)
                assert len(committed) == 3901
                want = ON.draft(ref, committed, k, lam, p_min_ctx)
                assert got[b].tolist() == want, f"lambda {lam} p_min_ctx {p_min_ctx} sequence {b} k {k}: {got[b].tolist()} vs {want}"
