"""Pins for oracle/model.py: sub-operations against library routines and closed forms, the
KV-cache equivalence, and the invariant that greedy speculative decoding reproduces plain greedy
decoding token for token whatever the drafter proposes."""
import random

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload as W
from oracle import model as OM
from oracle import ngram as ON


def tiny_cfg(**kw):
    base = W.get_config("cfg1").scaled(n_docs=300, gen_len=24, prompt_len=12)
    return base.scaled(**kw)


@pytest.fixture(scope="module")
def tiny():
    cfg = tiny_cfg()
    corpus = W.make_corpus(cfg)
    weights = W.make_model(cfg, corpus)
    return cfg, corpus, weights, OM.OracleModel(cfg, weights)


# ---------------------------------------------------------------- sub-operations
def test_rmsnorm_matches_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(OM.rmsnorm(x, g, 1e-6), want, rtol=1e-12, atol=1e-12)


def test_rope_is_a_rotation_of_pairs():
    rng = np.random.default_rng(1)
    hd = 8
    x = rng.standard_normal((6, 3, hd))
    pos = np.array([0, 1, 2, 5, 17, 400])
    y = OM.rope(x, pos, 10000.0)
    # the pair (i, i + hd/2) as a complex number is multiplied by exp(j * pos * theta^(-2i/hd))
    z = x[..., :hd // 2] + 1j * x[..., hd // 2:]
    ang = pos[:, None] * 10000.0 ** (-2.0 * np.arange(hd // 2) / hd)
    w = z * np.exp(1j * ang)[:, None, :]
    np.testing.assert_allclose(y[..., :hd // 2], w.real, atol=1e-12)
    np.testing.assert_allclose(y[..., hd // 2:], w.imag, atol=1e-12)
    np.testing.assert_allclose(y[0], x[0], atol=0)                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # scores depend on the position difference only
    q, k = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    s1 = (OM.rope(q, [9], 1e4) * OM.rope(k, [4], 1e4)).sum()
    s2 = (OM.rope(q, [105], 1e4) * OM.rope(k, [100], 1e4)).sum()
    np.testing.assert_allclose(s1, s2, rtol=1e-10)


def _torch_forward(cfg, wts, tokens):
    """Independent full-sequence forward built from torch library routines (float64)."""
    def t(a):
        a = W.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a
        return torch.from_numpy(np.ascontiguousarray(a)).double()
    n = len(tokens)
    H, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    x = t(wts["embed"])[torch.tensor(tokens)]
    pos = torch.arange(n).double()
    inv = cfg.rope_theta ** (-2.0 * torch.arange(hd // 2).double() / hd)
    rot = torch.polar(torch.ones(n, hd // 2).double(), pos[:, None] * inv[None, :])   # exp(j*angle)

    def rope(v):                                    # [n, heads, hd]
        z = torch.complex(v[..., :hd // 2], v[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)
    for lw in wts["layers"]:
        h = F.rms_norm(x, (cfg.d_model,), t(lw["g1"]), eps=cfg.rms_eps)
        q = rope(F.linear(h, t(lw["wq"])).view(n, H, hd)).transpose(0, 1)
        k = rope(F.linear(h, t(lw["wk"])).view(n, Hkv, hd)).transpose(0, 1)
        v = F.linear(h, t(lw["wv"])).view(n, Hkv, hd).transpose(0, 1)
        k = k.repeat_interleave(H // Hkv, dim=0)
        v = v.repeat_interleave(H // Hkv, dim=0)
        a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + F.linear(a.transpose(0, 1).reshape(n, H * hd), t(lw["wo"]))
        h = F.rms_norm(x, (cfg.d_model,), t(lw["g2"]), eps=cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t(lw["wg"]))) * F.linear(h, t(lw["wu"])), t(lw["wd"]))
    h = F.rms_norm(x, (cfg.d_model,), t(wts["gf"]), eps=cfg.rms_eps)
    return F.linear(h, t(wts["lm_head"])).numpy()


@pytest.mark.parametrize("variant", ["mha_f32", "gqa_bf16"])
def test_forward_matches_library_composition(variant):
    if variant == "mha_f32":
        cfg = tiny_cfg()
    else:
        cfg = tiny_cfg(dtype="bf16", n_heads=6, n_kv_heads=2, head_dim=16, d_model=96, d_ffn=160, vocab=300)
    wts = W.make_model(cfg, None)
    rng = np.random.default_rng(3)
    for lw in wts["layers"]:                        # non-trivial gains so a dropped gain shows
        lw["g1"] = rng.uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
        lw["g2"] = rng.uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
    wts["gf"] = rng.uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
    tokens = rng.integers(0, cfg.vocab, 21).tolist()
    m = OM.OracleModel(cfg, wts)
    got = m.forward(tokens, m.new_cache(32))
    np.testing.assert_allclose(got, _torch_forward(cfg, wts, tokens), rtol=1e-9, atol=1e-10)


def test_incremental_equals_full_recompute(tiny):
    cfg, corpus, wts, m = tiny
    rng = np.random.default_rng(5)
    tokens = rng.integers(0, cfg.vocab, 30).tolist()
    full = m.forward(tokens, m.new_cache(40))
    cache = m.new_cache(40)
    parts, p = [], 0
    for n in (7, 1, 5, 5, 12):                      # fed k+1 rows at a time
        parts.append(m.forward(tokens[p:p + n], cache))
        cache.length += n
        p += n
    np.testing.assert_allclose(np.concatenate(parts), full, rtol=1e-9, atol=1e-10)
    # a rolled-back cache forgets the rejected rows
    cache.length = 20
    again = m.forward(tokens[20:30], cache)
    np.testing.assert_allclose(again, full[20:30], rtol=1e-9, atol=1e-10)


def test_bias_is_added_for_the_input_token(tiny):
    cfg, corpus, wts, m = tiny
    nb = OM.OracleModel(cfg, dict(wts, bias=None))
    tokens = [3, 200, 77]
    d = m.forward(tokens, m.new_cache(8)) - nb.forward(tokens, nb.new_cache(8))
    raw = ON.build_tables_flat(corpus[0], corpus[1], cfg.vocab, 2, 1)
    for i, u in enumerate(tokens):
        succ = raw.orders[2].get((u,), {})
        c1 = sum(succ.values())
        want = np.array([cfg.bias_alpha * (np.log(succ.get(v, 0) + 1.0) - np.log(c1 + cfg.vocab))
                         for v in range(cfg.vocab)])
        np.testing.assert_allclose(d[i], want, rtol=1e-5, atol=1e-5)


# ---------------------------------------------------------------- the loop
def test_accept_length():
    assert OM.accept_length([], [9]) == 0
    assert OM.accept_length([1, 2, 3], [1, 2, 3, 4]) == 3
    assert OM.accept_length([1, 2, 3], [1, 9, 3, 4]) == 1
    assert OM.accept_length([1, 2, 3], [0, 2, 3, 4]) == 0


def test_speculative_equals_greedy_for_any_drafter(tiny):
    cfg, corpus, wts, m = tiny
    prompt = W.make_prompts(cfg)[0][:cfg.prompt_len]
    G = cfg.gen_len
    greedy, n_greedy = OM.generate(m, prompt, G, 0, None)
    assert n_greedy == G - 1 and len(greedy) == G
    full = list(prompt) + greedy

    def perfect(k):
        return lambda committed: (full[len(committed):len(committed) + k] + [0] * k)[:k]

    def wrong(k):
        return lambda committed: [(full[len(committed)] + 1) % cfg.vocab if len(committed) < len(full) else 0] * k

    rnd = random.Random(0)
    for k in (1, 3, 4):
        out, steps = OM.generate(m, prompt, G, k, perfect(k))
        assert out == greedy and steps == -(-(G - 1) // (k + 1))
        out, steps = OM.generate(m, prompt, G, k, wrong(k))
        assert out == greedy and steps == G - 1
        out, _ = OM.generate(m, prompt, G, k, lambda c: [rnd.randrange(cfg.vocab) for _ in range(k)])
        assert out == greedy
        out, _ = OM.generate(m, prompt, G, k, lambda c: [full[len(c)] if rnd.random() < 0.7 and len(c) < len(full)
                                                          else 0] + [0] * (k - 1), prefill_chunk=5)
        assert out == greedy


def test_ngram_drafter_speeds_up_and_is_exact(tiny):
    cfg, corpus, wts, m = tiny
    tables = ON.build_tables_flat(corpus[0], corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    prompt = W.make_prompts(cfg)[0][:cfg.prompt_len]
    greedy, n_greedy = OM.generate(m, prompt, cfg.gen_len, 0, None)
    trace = []
    out, steps = OM.generate(m, prompt, cfg.gen_len, cfg.k,
                             lambda c: ON.draft(tables, c, cfg.k, cfg.lambda_q16), trace=trace)
    assert out == greedy
    assert steps < n_greedy                          # the bigram-biased target follows the corpus
    assert sum(t["accept"] for t in trace) > 0
