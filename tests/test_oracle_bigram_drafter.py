"""Pins of the model-derived bigram drafter oracle (CPU only)."""
import numpy as np

import workload as W
from oracle import bigram_drafter as OB
from oracle import model as OM
from oracle import ngram as ON


def _cfg(**kw):
    base = dict(n_docs=120, vocab=96, d_model=32, n_heads=2, n_kv_heads=1, head_dim=16, d_ffn=64, n_layers=2)
    base.update(kw)
    return W.get_config("cfg1").scaled(**base)


def test_zero_layer_model_closed_form():
    """Without layers the next token after [x] is argmax_v W_lm[v] . rmsnorm(embed[x]) (+ bias row x): the
    textbook formula, typed out here with numpy."""
    cfg = _cfg(n_layers=0)
    corpus = W.make_corpus(cfg)
    for with_bias in (False, True):
        w = W.make_model(cfg, corpus if with_bias else None)
        got = OB.model_bigram(OM.OracleModel(cfg, w))
        e = w["embed"].astype(np.float64)
        h = e / np.sqrt((e * e).mean(axis=1, keepdims=True) + cfg.rms_eps) * w["gf"].astype(np.float64)
        z = h @ w["lm_head"].astype(np.float64).T                       # [V(x), V(v)]
        if with_bias:
            b = w["bias"]
            for x in range(cfg.vocab):
                lo, hi = int(b["rowptr"][x]), int(b["rowptr"][x + 1])
                row = np.full(cfg.vocab, float(b["base"][x]))
                row[b["col"][lo:hi]] = b["val"][lo:hi]
                z[x] += row
        assert got.tolist() == z.argmax(axis=1).tolist()


def test_bias_dominated_model_reproduces_corpus_bigrams():
    """With a very strong corpus bias the model's next token after x is the corpus' most frequent successor of x
    (wherever that successor is unique): the model-derived drafter then coincides with the order-2 corpus table."""
    cfg = _cfg(bias_alpha=2000.0)
    tok, off = W.make_corpus(cfg)
    w = W.make_model(cfg, (tok, off))
    nxt = OB.model_bigram(OM.OracleModel(cfg, w))
    pairs = ON.count_windows(ON.split_docs(tok, off), 2)
    checked = 0
    for x in range(cfg.vocab):
        succ = sorted(((c, v) for (u, v), c in pairs.items() if u == x), reverse=True)
        if succ and (len(succ) == 1 or succ[0][0] > succ[1][0]):
            assert nxt[x] == succ[0][1], f"token {x}"
            checked += 1
    assert checked > cfg.vocab // 2


def test_bigram_tables_are_point_masses():
    rng = np.random.default_rng(2)
    V = 40
    nxt = rng.integers(0, V, size=V)
    t = OB.bigram_tables(nxt, V, 4)
    assert t.n_max == 4
    assert sorted(t.orders[2].keys()) == [(x,) for x in range(V)]
    for x in range(V):
        assert t.orders[2][(x,)] == {int(nxt[x]): 1}
    assert t.orders[3] == {} and t.orders[4] == {}
    # alone (lambda = 1) the drafter follows the chain x -> next(x) -> next(next(x)) ...
    seq = [5, 9, 3]
    d = ON.draft(t, seq, 6, 65536)
    want, x = [], seq[-1]
    for _ in range(6):
        x = int(nxt[x])
        want.append(x)
    assert d == want
    # mixed with a context that has seen "3 -> 7" twice: lambda = 0.25 -> the context wins, 0.75 -> the model bigram
    seq = [3, 7, 1, 3, 7, 2, 3]
    nxt[3] = 11
    t = OB.bigram_tables(nxt, V, 2)
    assert ON.draft(t, seq, 1, int(0.25 * 65536)) == [7]
    assert ON.draft(t, seq, 1, int(0.75 * 65536)) == [11]


def test_any_drafter_keeps_greedy_output():
    """Speculative decoding with the model-derived drafter emits exactly the greedy tokens (the method's invariant),
    and accepts every first draft after a token whose bigram successor the full context does not override."""
    cfg = _cfg(gen_len=24, prompt_len=12)
    corpus = W.make_corpus(cfg)
    w = W.make_model(cfg, corpus)
    om = OM.OracleModel(cfg, w)
    nxt = OB.model_bigram(om)
    t = OB.bigram_tables(nxt, cfg.vocab, 3)
    prompt, _ = W.make_prompts(cfg, batch=1)
    greedy, _ = OM.generate(om, prompt, cfg.gen_len, 0, None)
    for lam in (1.0, 0.5):
        out, steps = OM.generate(om, prompt, cfg.gen_len, 3, lambda c: ON.draft(t, c, 3, int(lam * 65536)))
        assert out == greedy and steps < cfg.gen_len - 1
