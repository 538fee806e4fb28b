"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (same max_rows, same kernel
family): tables (whole for cfg2; for cfg3-5 every kept n-gram whose first token falls in one residue class, exact for
those keys), step replay of drafts (oracle counts taken on demand from the full corpus) and accept lengths,
speculative == greedy on every sequence, and logits of one sequence for the first verify steps.

Logit tolerance: 5e-2 absolute for cfg2 and cfg3.  For the 1.5B- and 3B-class models that bound is below what bf16
matrix-product inputs cost by themselves (tests/test_bf16_input_rounding.py measures it on the CPU: maximum 0.07 at
28 layers / width 1536, 0.12 at 36 layers / width 2048), so there the tests assert THIS BUILD'S OWN bounds, derived
from that measurement: rms, maximum, the share of logits beyond 5e-2, and that no argmax with a clear margin flips."""
import numpy as np
import pytest

import workload as W
from oracle import model as OM
from oracle import ngram as ON

pytestmark = [pytest.mark.gpu, pytest.mark.slow]


def _sampled_tables(tok, off, n, p_min, mod, rem):
    """Oracle counts restricted to the windows whose first token is = rem (mod `mod`): exact for those keys."""
    starts = ON.window_starts(off, n)
    starts = starts[tok[starts] % mod == rem]
    w, c = ON.count_windows_sorted(tok, off, n, starts=starts)
    keep = c >= p_min
    return w[keep], c[keep]


@pytest.mark.parametrize("name,max_rows,n_steps,sample", [("cfg2", 512, 8, None), ("cfg3", 64, 8, (16, 3))])
def test_full_size_config(name, max_rows, n_steps, sample):
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    from test_gpu_model import _replay
    cfg = W.get_config(name)
    print(f"{name}: building inputs", flush=True)
    rig = Rig(cfg, max_rows=max_rows)
    tok, off = rig.corpus
    # ---- tables
    if sample is None:
        ref = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
        for n in range(2, cfg.n_max + 1):
            rows, counts = T.tasc_ngram_export(rig.ng, n)
            want = ref.export(n)
            assert rows.shape[0] == want.shape[0] and (rows == want[:, :n]).all() and (counts == want[:, n]).all()
    else:
        mod, rem = sample
        for n in range(2, cfg.n_max + 1):
            rows, counts = T.tasc_ngram_export(rig.ng, n)
            sel = rows[:, 0] % mod == rem
            w, c = _sampled_tables(tok, off, n, cfg.p_min, mod, rem)
            assert int(sel.sum()) == w.shape[0], f"order {n}: {int(sel.sum())} sampled rows, oracle {w.shape[0]}"
            assert (rows[sel] == w).all() and (counts[sel] == c).all()
        ref = None
        lazy = ON.LazyTables(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    print("tables ok", flush=True)
    # ---- generation: speculative == greedy on every sequence; replay of drafts / accept lengths
    out, st, tr = rig.generate(trace_steps=cfg.gen_len)
    g_out, g_st, _ = rig.generate(k=0)
    assert (out == g_out).all(), "speculative output differs from the GPU's own greedy decode"
    print(f"steps {st.steps} vs greedy {g_st.steps}; accepted {st.accepted}/{st.proposed}; decode {st.decode_ms:.1f} ms "
          f"(greedy {g_st.decode_ms:.1f} ms)", flush=True)
    if ref is not None:
        for b in range(cfg.batch):
            p = rig.prompts[rig.prompt_off[b]:rig.prompt_off[b + 1]].tolist()
            _replay(cfg, ref, p, tr[:, b], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[b])
    else:
        # every sequence's accept lengths from the GPU's argmax ids; drafts recomputed by the oracle for a spread of
        # sequences over all of their steps (corpus counts on demand from the full corpus)
        n_before, drafts, amax, acc = split_trace(tr, cfg.k)
        for s in range(tr.shape[0]):
            for b in range(cfg.batch):
                if acc[s, b] >= 0:
                    assert acc[s, b] == OM.accept_length(drafts[s, b].tolist(), amax[s, b].tolist())
        for b in range(0, cfg.batch, 4):
            p = rig.prompts[rig.prompt_off[b]:rig.prompt_off[b + 1]].tolist()
            _replay(cfg, lazy, p, tr[:, b], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[b])
        print("draft replay ok", flush=True)
    # ---- logits of sequence 0: prompt forward and the first verify steps
    om = OM.OracleModel(cfg, rig.weights)
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    p0 = rig.prompts[:cfg.prompt_len].tolist()
    cache = om.new_cache(rig.max_len)
    z = om.forward(p0, cache, last_only=True)
    cache.length = len(p0)
    first = int(T.tasc_session_get_tokens(rig.session, 0)[-1])
    top2 = np.sort(z[0])[-2:]
    assert first == int(np.argmax(z[0])) or top2[1] - top2[0] < 0.1
    print("prompt forward ok", flush=True)
    logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    drafts_d = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    worst = 0.0
    for s in range(n_steps):
        T.tasc_draft(rig.ng, rig.session, rig.params(), drafts_d)
        before = T.tasc_session_get_tokens(rig.session, 0)
        T.tasc_verify_step(rig.model, rig.session, drafts_d, cfg.k, None, None, logits)
        got = logits[0].cpu().numpy().astype(np.float64)
        d = drafts_d[0].cpu().numpy().tolist()
        z = om.forward([int(before[-1])] + d, cache)
        worst = max(worst, float(np.abs(got - z).max()))
        cache.length += len(T.tasc_session_get_tokens(rig.session, 0)) - len(before)
    print(f"{name}: max |logit - oracle| over {n_steps} verify steps = {worst:.3e}", flush=True)
    assert worst <= 5e-2


# This build's own logit bounds for the 1.5B- and 3B-class models (see the module docstring): (rms, maximum, share of the
# logits beyond 5e-2).  The CPU measurement of bf16 matrix-product inputs and softmax weights alone, in this test's
# setting (a verify step after a 48-token prompt), gives rms 1.4e-2 / maximum 0.070 / share 3e-4 at 28 layers and width
# 1536, and rms 2.2e-2 / maximum 0.12 / share 2.5e-2 at 36 layers and width 2048; the bounds are about 1.4 times that.
DEEP_BOUNDS = {"cfg4": (2e-2, 1e-1, 2e-3), "cfg5": (3e-2, 1.8e-1, 4e-2)}


def _check_deep_model_logits(name, got, z):
    label = name + " model"
    own_rms, own_max, own_share = DEEP_BOUNDS[name]
    d = np.abs(got - z)
    worst, rms, share = float(d.max()), float(np.sqrt((d ** 2).mean())), float((d > 5e-2).mean())
    top2 = np.sort(z, axis=-1)[:, -2:]
    margin = top2[:, 1] - top2[:, 0]
    flips = [(i, float(margin[i])) for i in range(z.shape[0]) if int(np.argmax(got[i])) != int(np.argmax(z[i]))]
    print(f"{label}: max |logit - oracle| = {worst:.3e}, rms {rms:.3e}, share beyond 5e-2 {share:.2e}, "
          f"smallest top-1 margin {margin.min():.2f}, argmax flips {flips}", flush=True)
    assert rms <= own_rms and worst <= own_max and share <= own_share
    assert all(m <= 0.2 for _, m in flips), "an argmax with a clear margin differs from the oracle's"


def test_cfg4_model_at_its_launch_shapes():
    """The 1.5B-class model with config 4's batch and draft length (576 rows per verify step: the 256 x 192 GEMM tiles,
    head_dim 128 attention in 4 key chunks) on short prompts and a small corpus, so that the oracle can follow a
    sequence: speculative == greedy on all 64 sequences, accept lengths consistent with the GPU's own drafts and argmax
    ids, and the logits of one sequence's prompt forward and first verify step against the oracle."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    cfg = W.get_config("cfg4").scaled(n_docs=3000, prompt_len=48, gen_len=20)
    print("cfg4 model: building inputs", flush=True)
    rig = Rig(cfg, max_rows=64)
    out, st, tr = rig.generate(trace_steps=cfg.gen_len)
    g_out, g_st, _ = rig.generate(k=0)
    assert (out == g_out).all(), "speculative output differs from the GPU's own greedy decode"
    assert g_st.steps == cfg.gen_len - 1
    n_before, drafts, amax, acc = split_trace(tr, cfg.k)
    for s in range(tr.shape[0]):
        for b in range(cfg.batch):
            if acc[s, b] >= 0:
                assert acc[s, b] == OM.accept_length(drafts[s, b].tolist(), amax[s, b].tolist())
    print(f"steps {st.steps} vs greedy {g_st.steps}; accepted {st.accepted}/{st.proposed}", flush=True)
    om = OM.OracleModel(cfg, rig.weights)
    b = 5
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    prompt = rig.prompts[rig.prompt_off[b]:rig.prompt_off[b + 1]].tolist()
    cache = om.new_cache(rig.max_len)
    z = om.forward(prompt, cache, last_only=True)
    cache.length = len(prompt)
    first = int(T.tasc_session_get_tokens(rig.session, b)[-1])
    top2 = np.sort(z[0])[-2:]
    assert first == int(np.argmax(z[0])) or top2[1] - top2[0] < 0.1
    logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    drafts_d = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    T.tasc_draft(rig.ng, rig.session, rig.params(), drafts_d)
    before = T.tasc_session_get_tokens(rig.session, b)
    T.tasc_verify_step(rig.model, rig.session, drafts_d, cfg.k, None, None, logits)
    got = logits[b].cpu().numpy().astype(np.float64)
    z = om.forward([int(before[-1])] + drafts_d[b].cpu().numpy().tolist(), cache)
    _check_deep_model_logits("cfg4", got, z)


def test_cfg5_model_at_its_launch_shapes():
    """Config 5's model at its full depth of 36 layers and its launch shapes (1280 rows per verify step of 256 sequences:
    256 x 256 GEMM tiles, the down projection at its widest row of 2048, head_dim 128 attention in one key chunk,
    16384-row prompt chunks) on short prompts and a small corpus, so that the oracle can follow a sequence: speculative == greedy on all 256 sequences, accept lengths consistent with the GPU's own drafts
    and argmax ids, and the logits of one sequence's prompt forward and first verify step against the oracle."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    cfg = W.get_config("cfg5").scaled(n_docs=3000, prompt_len=48, gen_len=16)
    print("cfg5 model: building inputs", flush=True)
    rig = Rig(cfg, max_rows=64)
    out, st, tr = rig.generate(trace_steps=cfg.gen_len)
    g_out, g_st, _ = rig.generate(k=0)
    assert (out == g_out).all(), "speculative output differs from the GPU's own greedy decode"
    assert g_st.steps == cfg.gen_len - 1
    n_before, drafts, amax, acc = split_trace(tr, cfg.k)
    for s in range(tr.shape[0]):
        for b in range(cfg.batch):
            if acc[s, b] >= 0:
                assert acc[s, b] == OM.accept_length(drafts[s, b].tolist(), amax[s, b].tolist())
    print(f"steps {st.steps} vs greedy {g_st.steps}; accepted {st.accepted}/{st.proposed}", flush=True)
    om = OM.OracleModel(cfg, rig.weights)
    b = 201
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    prompt = rig.prompts[rig.prompt_off[b]:rig.prompt_off[b + 1]].tolist()
    cache = om.new_cache(rig.max_len)
    z = om.forward(prompt, cache, last_only=True)
    cache.length = len(prompt)
    first = int(T.tasc_session_get_tokens(rig.session, b)[-1])
    top2 = np.sort(z[0])[-2:]
    assert first == int(np.argmax(z[0])) or top2[1] - top2[0] < 0.1
    logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    drafts_d = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    T.tasc_draft(rig.ng, rig.session, rig.params(), drafts_d)
    before = T.tasc_session_get_tokens(rig.session, b)
    T.tasc_verify_step(rig.model, rig.session, drafts_d, cfg.k, None, None, logits)
    got = logits[b].cpu().numpy().astype(np.float64)
    z = om.forward([int(before[-1])] + drafts_d[b].cpu().numpy().tolist(), cache)
    _check_deep_model_logits("cfg5", got, z)


@pytest.mark.parametrize("name,mod,rem", [("cfg4", 64, 5), ("cfg5", 64, 37)])
def test_full_size_tables_and_drafts(name, mod, rem):
    """The corpora of the two largest configurations in full (80 M and 160 M tokens, orders up to 5, keys of 90 bits):
    every kept n-gram whose first token is = rem (mod `mod`) equals the oracle's count of exactly those windows, the
    window totals agree, and drafts over these tables equal the oracle's (counts on demand from the full corpus) for
    sequences made of corpus text, at the configuration's mixture weight and with the corpus alone."""
    import torch
    import paper_2602_24174_amd as T
    cfg = W.get_config(name)
    print(f"{name}: building the corpus", flush=True)
    tok, off = W.make_corpus(cfg)
    ng = T.tasc_ngram_build(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    st = T.tasc_ngram_get_stats(ng)
    print(f"{name}: {tok.shape[0]} tokens, build {st.build_ms:.0f} ms, kept {list(st.kept)[2:cfg.n_max + 1]}", flush=True)
    for n in range(2, cfg.n_max + 1):
        assert st.windows[n] == int(np.maximum(np.diff(off) - n + 1, 0).sum())
        rows, counts = T.tasc_ngram_export(ng, n)
        assert rows.shape[0] == st.kept[n]
        sel = rows[:, 0] % mod == rem
        w, c = _sampled_tables(tok, off, n, cfg.p_min, mod, rem)
        assert int(sel.sum()) == w.shape[0], f"order {n}: {int(sel.sum())} sampled rows, oracle {w.shape[0]}"
        assert (rows[sel] == w).all() and (counts[sel] == c).all()
        print(f"order {n}: {w.shape[0]} of {rows.shape[0]} kept n-grams compared", flush=True)
        del rows, counts, w, c
    # ---- drafts: a tiny target with the configuration's vocabulary carries the sequences; the tables are the real ones
    lazy = ON.LazyTables(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    tiny = W.get_config("cfg1").scaled(vocab=cfg.vocab, n_max=cfg.n_max, batch=16, prompt_len=160, gen_len=8, k=cfg.k)
    weights = W.make_model(tiny, (tok, off))       # corpus-biased LM head: the committed first token continues the corpus text
    max_len = 160 + 8 + 32
    model = T.tasc_model_create(tiny, weights, max_len)
    sess = T.tasc_session_create(model, tiny.batch, max_len, 16)
    rng = np.random.default_rng(3)
    prompts = []
    for b in range(tiny.batch):
        d = int(rng.integers(0, cfg.n_docs))
        p = tok[off[d]:off[d + 1]].copy()[:int(rng.integers(8, 150))]
        if b % 4 == 1:
            p = np.concatenate([p[:70], p[:70]])                       # repeated text: both sources match
        if b % 4 == 2:
            p[rng.integers(0, len(p), 3)] = rng.integers(0, cfg.vocab, 3)   # extra noise: forces back-off
        prompts.append(p.astype(np.int32))
    flat = np.concatenate(prompts)
    poff = np.cumsum([0] + [len(p) for p in prompts]).astype(np.int64)
    T.tasc_session_prefill(model, sess, flat, poff, tiny.gen_len)
    high = 0
    for lam in (cfg.lambda_q16, 65536):
        drafts = torch.zeros((tiny.batch, cfg.k), dtype=torch.int32, device="cuda")
        T.tasc_draft(ng, sess, T.spec_params(cfg.k, lam, cfg.p_min_ctx, 1), drafts)
        got = drafts.cpu().numpy()
        for b in range(tiny.batch):
            committed = T.tasc_session_get_tokens(sess, b)
            want = ON.draft(lazy, committed, cfg.k, lam, cfg.p_min_ctx)
            assert got[b].tolist() == want, f"{name} lambda {lam} sequence {b}: {got[b].tolist()} vs oracle {want}"
            m = ON.backoff(lazy, [int(t) for t in committed])
            high += m is not None and m[0] >= 4
    assert high > 0, "no sequence matched a corpus context of 3+ tokens"
    print(f"{name}: drafts ok ({high} high-order corpus matches)", flush=True)
