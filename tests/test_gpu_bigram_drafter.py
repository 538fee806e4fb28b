"""The model-derived bigram drafter on the GPU against the oracle: next(x) per vocabulary token, the tables built from
it, and draft-then-verify decoding with it alone and mixed with the context statistics."""
import numpy as np
import pytest

import workload as W
from oracle import bigram_drafter as OB
from oracle import model as OM
from oracle import ngram as ON

pytestmark = pytest.mark.gpu


def _bigram_on_gpu(T, model, cfg, batch, max_rows):
    import torch
    max_len = 2 + 2 * max_rows
    sess = T.tasc_session_create(model, batch, max_len, max_rows)
    nxt = torch.full((cfg.vocab,), -1, dtype=torch.int32, device="cuda")
    T.tasc_model_bigram(model, sess, nxt)
    sess.close()
    return nxt


@pytest.mark.parametrize("variant", ["cfg1_f32", "f32_gqa", "bf16_gqa_small", "bf16_gqa_tiled"])
def test_model_bigram_matches_oracle(variant):
    import paper_2602_24174_amd as T
    base = W.get_config("cfg1")
    if variant == "cfg1_f32":
        cfg, batch, max_rows = base, 7, 1                 # 512 tokens in chunks of 7: ragged last chunk
    elif variant == "f32_gqa":
        cfg = base.scaled(n_layers=3, d_model=192, n_heads=6, n_kv_heads=2, head_dim=32, d_ffn=320, vocab=1000, n_docs=1500)
        batch, max_rows = 64, 4                           # padded rows in every chunk
    elif variant == "bf16_gqa_small":
        cfg = base.scaled(dtype="bf16", n_layers=3, d_model=192, n_heads=6, n_kv_heads=2, head_dim=32, d_ffn=320, vocab=1000,
                          n_docs=1500)
        batch, max_rows = 16, 1                           # the persistent small-batch kernel
    else:
        cfg = base.scaled(dtype="bf16", n_layers=2, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=512, vocab=3000,
                          n_docs=3000)
        batch, max_rows = 96, 1                           # the tiled MFMA kernels, 3000 = 31 x 96 + 24
    corpus = W.make_corpus(cfg)
    weights = W.make_model(cfg, corpus)
    model = T.tasc_model_create(cfg, weights, 64)
    print(f"{variant}: vocab {cfg.vocab}, batch {batch}, max_rows {max_rows}", flush=True)
    got = _bigram_on_gpu(T, model, cfg, batch, max_rows).cpu().numpy()
    om = OM.OracleModel(cfg, weights)
    want = OB.model_bigram(om)
    tol = 1e-3 if cfg.dtype == "f32" else 5e-2
    diff = np.flatnonzero(got != want)
    if diff.size:
        # a different argmax is only acceptable where the oracle's two best logits are closer than the logit tolerance
        margins = OB.bigram_margins(om)
        for x in diff:
            z = om.forward([int(x)], om.new_cache(2), last_only=True)[0]
            assert margins[x] < 2 * tol and z.max() - z[got[x]] < 2 * tol, f"token {x}: GPU {got[x]}, oracle {want[x]}, margin {margins[x]:.3e}"
    print(f"{variant}: {diff.size} of {cfg.vocab} successors differ (all within the logit tolerance)", flush=True)
    assert diff.size <= cfg.vocab // 100
    assert (got >= 0).all() and (got < cfg.vocab).all()


def test_bigram_tables_and_decoding():
    """Config 1: the tables built from next(x) equal the oracle's, and decoding with them (alone, and mixed with the
    context statistics at several lambda) reproduces the oracle's drafts, accept lengths and tokens step by step."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    cfg = W.get_config("cfg1")
    rig = Rig(cfg, with_ngram=False)
    om = OM.OracleModel(cfg, rig.weights)
    nxt = _bigram_on_gpu(T, rig.model, cfg, 32, 1)
    nxt_h = nxt.cpu().numpy()
    assert nxt_h.tolist() == OB.model_bigram(om).tolist()
    n_max = 3
    for src in (nxt, nxt_h):                              # device and host input
        ng = T.tasc_ngram_from_bigram(src, cfg.vocab, n_max)
        ref = OB.bigram_tables(nxt_h, cfg.vocab, n_max)
        rows, counts = T.tasc_ngram_export(ng, 2)
        want = ref.export(2)
        assert (rows.astype(np.int64) == want[:, :2]).all() and (counts.astype(np.int64) == want[:, 2]).all()
        assert rows.shape[0] == cfg.vocab and (counts == 1).all()
        assert T.tasc_ngram_export(ng, 3)[0].shape[0] == 0
        fb, uni = T.tasc_ngram_unigram(ng, cfg.vocab)
        assert fb == ref.fallback and (uni.astype(np.int64) == ref.unigram).all()
    rig.ng = ng
    for lam in (1.0, 0.75, 0.25, 0.0):
        q16 = int(round(lam * 65536))
        otrace = []
        want, o_steps = OM.generate(om, rig.prompts, cfg.gen_len, cfg.k, lambda c: ON.draft(ref, c, cfg.k, q16, cfg.p_min_ctx),
                                    trace=otrace, prefill_chunk=rig.max_rows)
        out, st, tr = rig.generate(trace_steps=cfg.gen_len, lambda_q16=q16)
        assert out[0].tolist() == want and st.steps == o_steps
        _, drafts, amax, acc = split_trace(tr[:, 0], cfg.k)
        for s, o in enumerate(otrace):
            assert drafts[s].tolist() == o["drafts"] and acc[s] == o["accept"] and amax[s].tolist() == o["argmax"].tolist()
        print(f"lambda {lam}: {st.steps} steps, accepted {st.accepted} of {st.proposed}", flush=True)
    # a successor outside the vocabulary is rejected
    bad = nxt_h.copy()
    bad[3] = cfg.vocab
    with pytest.raises(T.TascError):
        T.tasc_ngram_from_bigram(bad, cfg.vocab, n_max)
