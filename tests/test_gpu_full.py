"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (same max_rows, same kernel
family): tables (whole for cfg2, a 1/16 sample of the windows for cfg3), step replay of drafts and accept lengths,
speculative == greedy on every sequence, and logits of sequence 0 for the first verify steps."""
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


@pytest.mark.parametrize("name,max_rows,n_steps,sample", [("cfg2", 512, 8, None), ("cfg3", 64, 2, (16, 3))])
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
        # accept lengths from the GPU's own drafts and argmax ids (integers only; no oracle tables at this size)
        n_before, drafts, amax, acc = split_trace(tr, cfg.k)
        for s in range(tr.shape[0]):
            for b in range(cfg.batch):
                if acc[s, b] >= 0:
                    assert acc[s, b] == OM.accept_length(drafts[s, b].tolist(), amax[s, b].tolist())
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
    worst = float(np.abs(got - z).max())
    rms = float(np.sqrt(((got - z) ** 2).mean()))
    print(f"cfg4 model: max |logit - oracle| = {worst:.3e}, rms {rms:.3e}", flush=True)
    # 28 layers of width 1536 with bf16 activations between the kernels: the rounding of the GEMM inputs alone gives an
    # rms error of 1.2e-2 - 1.3e-2 on logits of standard deviation 1.0 in BOTH kernel families (type-generic and MFMA;
    # they differ from each other by as much), and the largest of 1.4 M logits then lies near 5.4 sigma = 0.07.  The 5e-2
    # bound of the smaller configurations is therefore checked here on the rms, and the maximum against 1e-1.
    assert rms <= 2e-2 and worst <= 1e-1


def test_cfg5_launch_shapes():
    """Config 5's per-layer launch shapes (1280 rows per verify step of 256 sequences: 256 x 256 GEMM tiles, the down
    projection in 6 k-slices with the fused reduction + norm at its widest row of 2048, head_dim 128 attention in one key
    chunk, 16384-row prompt chunks) on the first 6 of its 36 layers, short prompts and a small corpus, so that the oracle
    can follow a sequence: speculative == greedy on all 256 sequences, accept lengths consistent with the GPU's own drafts
    and argmax ids, and the logits of one sequence's prompt forward and first verify step against the oracle."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    cfg = W.get_config("cfg5").scaled(n_layers=6, n_docs=3000, prompt_len=48, gen_len=16)
    print("cfg5 shapes: building inputs", flush=True)
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
    worst = float(np.abs(got - z).max())
    rms = float(np.sqrt(((got - z) ** 2).mean()))
    print(f"cfg5 shapes: max |logit - oracle| = {worst:.3e}, rms {rms:.3e}", flush=True)
    # width 2048 with bf16 activations between the kernels: rms 1.1e-2 on logits of standard deviation 1.0 already at 6
    # layers, the largest of 0.76 M logits near 4.7 sigma = 0.05; same bound as for the 1.5B-class model above
    assert rms <= 2e-2 and worst <= 1e-1
