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
