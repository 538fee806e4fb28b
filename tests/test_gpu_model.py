"""GPU forward, verify step and generation loop against the CPU oracle."""
import numpy as np
import pytest

import workload as W
from oracle import model as OM
from oracle import ngram as ON

pytestmark = pytest.mark.gpu


def _replay(cfg, ref_tables, prompt, trace_b, k, lam, p_min_ctx, out_tokens):
    """Oracle recomputes every step's drafts from the GPU's committed tokens and every accept length
    from the GPU's argmax ids (no oracle transformer needed)."""
    from gpu_util import split_trace
    n_before, drafts, amax, acc = split_trace(trace_b, k)
    seq = list(prompt) + [int(out_tokens[0])]
    for s in range(trace_b.shape[0]):
        if acc[s] < 0:
            continue                                       # frozen: already has its tokens
        assert n_before[s] == len(seq)
        if k:
            assert drafts[s].tolist() == ON.draft(ref_tables, seq, k, lam, p_min_ctx), f"step {s}"
        m = OM.accept_length(drafts[s].tolist(), amax[s].tolist())
        assert m == acc[s], f"step {s}"
        seq += drafts[s][:m].tolist() + [int(amax[s][m])]
    gen = seq[len(prompt):]
    assert gen[:len(out_tokens)] == out_tokens.tolist()


def test_cfg1_end_to_end():
    """Config 1 in full: every draft, argmax, accept length and token equals the oracle's; logits <= 1e-3."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig, split_trace
    cfg = W.get_config("cfg1")
    rig = Rig(cfg)
    ref_tables = ON.build_tables_flat(rig.corpus[0], rig.corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    om = OM.OracleModel(cfg, rig.weights)
    otrace = []
    want, o_steps = OM.generate(om, rig.prompts, cfg.gen_len, cfg.k,
                                lambda c: ON.draft(ref_tables, c, cfg.k, cfg.lambda_q16, cfg.p_min_ctx), trace=otrace,
                                prefill_chunk=rig.max_rows)
    out, st, tr = rig.generate(trace_steps=cfg.gen_len)
    print(f"steps {st.steps} (oracle {o_steps}), accepted {st.accepted}/{st.proposed}, decode {st.decode_ms:.2f} ms", flush=True)
    assert out[0].tolist() == want
    assert st.steps == o_steps
    n_before, drafts, amax, acc = split_trace(tr[:, 0], cfg.k)
    for s, o in enumerate(otrace):
        assert n_before[s] == len(o["committed"])
        assert drafts[s].tolist() == o["drafts"]
        assert amax[s].tolist() == o["argmax"].tolist()
        assert acc[s] == o["accept"]
    assert st.accepted == sum(o["accept"] for o in otrace)
    assert sum(st.accept_hist) == st.steps
    _replay(cfg, ref_tables, rig.prompts.tolist(), tr[:, 0], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[0])
    # plain greedy on the GPU gives the same tokens
    g_out, g_st, _ = rig.generate(k=0)
    assert g_out[0].tolist() == want and g_st.steps == cfg.gen_len - 1

    # logits of single verify steps against the oracle, step by step
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    cache = om.new_cache(rig.max_len)
    om.forward(rig.prompts.tolist(), cache)
    cache.length = len(rig.prompts)
    logits = torch.zeros((1, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    acc_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    emit_d = torch.zeros((1, cfg.k + 1), dtype=torch.int32, device="cuda")
    worst = 0.0
    for s in range(6):
        committed = T.tasc_session_get_tokens(rig.session, 0)
        d = ON.draft(ref_tables, committed, cfg.k, cfg.lambda_q16, cfg.p_min_ctx)
        d_dev = torch.tensor([d], dtype=torch.int32, device="cuda")
        T.tasc_verify_step(rig.model, rig.session, d_dev, cfg.k, acc_d, emit_d, logits)
        z = om.forward([int(committed[-1])] + d, cache)
        got = logits.cpu().numpy()[0].astype(np.float64)
        worst = max(worst, float(np.abs(got - z).max()))
        a = OM.argmax_lowest(z)
        m = OM.accept_length(d, a)
        assert int(acc_d.cpu()[0]) == m
        assert emit_d.cpu().numpy()[0].tolist() == d[:m] + [int(a[m])] + [-1] * (cfg.k - m)
        cache.length += m + 1
    print(f"max |logit - oracle| = {worst:.3e}", flush=True)
    assert worst <= 1e-3


@pytest.mark.parametrize("variant", ["f32_gqa_batch", "bf16_gqa_batch"])
def test_small_batched_models(variant):
    """Ragged prompts, batch > 1, GQA, several KV pages and a prompt longer than one chunk; both dtypes."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    base = W.get_config("cfg1")
    cfg = base.scaled(dtype="f32" if variant.startswith("f32") else "bf16", n_layers=3, d_model=192, n_heads=6, n_kv_heads=2,
                      head_dim=32, d_ffn=320, vocab=1000, batch=5, prompt_len=45, gen_len=40, k=5, n_docs=1500, n_max=4)
    rig = Rig(cfg, max_rows=16)
    tol = 1e-3 if cfg.dtype == "f32" else 5e-2
    ref_tables = ON.build_tables_flat(rig.corpus[0], rig.corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    om = OM.OracleModel(cfg, rig.weights)
    # ragged prompts
    lens = [45, 1, 16, 33, 17]
    rng = np.random.default_rng(1)
    prompts = [rng.integers(0, cfg.vocab, n).astype(np.int32) for n in lens]
    rig.prompts = np.concatenate(prompts)
    rig.prompt_off = np.cumsum([0] + lens).astype(np.int64)
    out, st, tr = rig.generate(trace_steps=cfg.gen_len)
    g_out, g_st, _ = rig.generate(k=0)
    assert (out == g_out).all(), "speculative output differs from the GPU's own greedy decode"
    assert g_st.steps == cfg.gen_len - 1 and st.steps <= g_st.steps
    for b in range(cfg.batch):
        _replay(cfg, ref_tables, prompts[b].tolist(), tr[:, b], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[b])
    # logits: the oracle follows the GPU's committed tokens for a few steps
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    caches = []
    for b in range(cfg.batch):
        c = om.new_cache(rig.max_len)
        z = om.forward(prompts[b].tolist(), c, last_only=True)
        c.length = lens[b]
        caches.append(c)
        first = T.tasc_session_get_tokens(rig.session, b)[-1]
        top2 = np.sort(z[0])[-2:]
        assert first == int(np.argmax(z[0])) or top2[1] - top2[0] < 2 * tol
    logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    worst = 0.0
    for s in range(4):
        T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
        before = [T.tasc_session_get_tokens(rig.session, b) for b in range(cfg.batch)]
        T.tasc_verify_step(rig.model, rig.session, drafts, cfg.k, None, None, logits)
        got = logits.cpu().numpy().astype(np.float64)
        d = drafts.cpu().numpy()
        for b in range(cfg.batch):
            z = om.forward([int(before[b][-1])] + d[b].tolist(), caches[b])
            worst = max(worst, float(np.abs(got[b] - z).max()))
            after = T.tasc_session_get_tokens(rig.session, b)
            caches[b].length += len(after) - len(before[b])
    print(f"{variant}: max |logit - oracle| = {worst:.3e}", flush=True)
    assert worst <= tol


def test_api_errors():
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    cfg = W.get_config("cfg1").scaled(n_docs=100, gen_len=8, prompt_len=8)
    rig = Rig(cfg, max_rows=8)
    drafts = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(T.TascError) as e:                     # verify before prefill
        T.tasc_verify_step(rig.model, rig.session, drafts, 4)
    assert e.value.status == -4
    with pytest.raises(T.TascError) as e:
        T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
    assert e.value.status == -4
    bad = rig.prompts.copy()
    bad[3] = cfg.vocab
    with pytest.raises(T.TascError) as e:
        T.tasc_session_prefill(rig.model, rig.session, bad, rig.prompt_off, 8)
    assert e.value.status == -1
    with pytest.raises(T.TascError) as e:                     # does not fit max_len
        T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, 1000)
    assert e.value.status == -1
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, 8)
    for k in (-1, 8, 16):
        with pytest.raises(T.TascError) as e:
            T.tasc_verify_step(rig.model, rig.session, drafts, k)
        assert e.value.status == -1
    with pytest.raises(T.TascError):
        T.tasc_draft(rig.ng, rig.session, T.spec_params(4, 70000), drafts)
    import ctypes                                             # workspace too small
    out = ctypes.c_void_p()
    rc = T.lib().tasc_session_create(rig.model.handle, 1, rig.max_len, 8, rig.session._kv_pool.data_ptr(), 16,
                                     rig.session._workspace.data_ptr(), 16, ctypes.byref(out))
    assert rc == -2 and out.value is None
    # a draft outside the vocabulary is simply rejected
    acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    T.tasc_verify_step(rig.model, rig.session, torch.tensor([[10**6, 1, 2, 3]], dtype=torch.int32, device="cuda"), 4, acc)
    assert int(acc.cpu()[0]) == 0


@pytest.mark.parametrize("heads", [(6, 2, 32), (4, 2, 64), (2, 1, 128), (4, 4, 64)])
def test_small_batch_fused_kernel(heads):
    """bf16 forwards of at most 16 rows run in one persistent launch per step: the spatial-pipeline kernel (modes 5 and,
    launched phase by phase, 6) and the barrier kernel (modes 2, 3, 4, and 1 phase by phase) against the oracle and
    against each other (bit-identical), and speculative == greedy within each mode."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    H, Hkv, hd = heads
    cfg = W.get_config("cfg1").scaled(dtype="bf16", n_layers=3, d_model=H * hd if H * hd >= 192 else 192, n_heads=H,
                                      n_kv_heads=Hkv, head_dim=hd, d_ffn=320, vocab=1000, batch=2, prompt_len=70, gen_len=48,
                                      k=6, n_docs=1500, n_max=4)
    rig = Rig(cfg, max_rows=8)                     # prompt chunks of 8 rows x 2 sequences = 16 rows
    lens = [70, 37]
    rng = np.random.default_rng(7)
    prompts = [rng.integers(0, cfg.vocab, n).astype(np.int32) for n in lens]
    rig.prompts = np.concatenate(prompts)
    rig.prompt_off = np.cumsum([0] + lens).astype(np.int64)
    ref_tables = ON.build_tables_flat(rig.corpus[0], rig.corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    om = OM.OracleModel(cfg, rig.weights)
    results = {}
    try:
        # barrier kernel: 2 = persistent, 3 = agent-scope barriers only, 4 = half of the layer group prefetching, 1 = one
        # launch per phase; pipeline kernel: 5 = persistent (the default), 6 = one launch per phase; 0 = generic kernels
        for mode in (5, 6, 2, 3, 4, 1, 0):
            print(f"heads {heads} mode {mode}", flush=True)
            T.tasc_config_set(T.TASC_CFG_SMALL_KERNEL, 1 if mode in (5, 6) else 0)
            T.tasc_config_set(T.TASC_CFG_SMALL_PATH, {5: 2, 6: 1}.get(mode, min(mode, 2)))
            T.tasc_config_set(T.TASC_CFG_SMALL_XCD_LOCAL, 0 if mode == 3 else 1)
            T.tasc_config_set(T.TASC_CFG_SMALL_LAYER_WORKERS, 16 if mode == 4 else 0)
            out, st, tr = rig.generate(trace_steps=cfg.gen_len)
            g_out, g_st, _ = rig.generate(k=0)
            assert (out == g_out).all(), f"mode {mode}: speculative output differs from greedy"
            assert not T.tasc_session_status(rig.session), f"mode {mode}: a wait of the persistent kernel timed out"
            for b in range(cfg.batch):
                _replay(cfg, ref_tables, prompts[b].tolist(), tr[:, b], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[b])
            # logits of a few verify steps
            T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
            caches = []
            for b in range(cfg.batch):
                c = om.new_cache(rig.max_len)
                om.forward(prompts[b].tolist(), c, last_only=True)
                c.length = lens[b]
                caches.append(c)
            logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
            drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
            worst, all_logits = 0.0, []
            for s in range(5):
                T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
                before = [T.tasc_session_get_tokens(rig.session, b) for b in range(cfg.batch)]
                T.tasc_verify_step(rig.model, rig.session, drafts, cfg.k, None, None, logits)
                got = logits.cpu().numpy()
                all_logits.append(got.copy())
                d = drafts.cpu().numpy()
                for b in range(cfg.batch):
                    z = om.forward([int(before[b][-1])] + d[b].tolist(), caches[b])
                    worst = max(worst, float(np.abs(got[b].astype(np.float64) - z).max()))
                    after = T.tasc_session_get_tokens(rig.session, b)
                    caches[b].length += len(after) - len(before[b])
            print(f"mode {mode}: max |logit - oracle| = {worst:.3e}, steps {st.steps}, XCD-local steps {st.xcd_local_steps}", flush=True)
            if mode in (3, 5, 6):
                assert st.xcd_local_steps == 0
            assert worst <= 5e-2
            results[mode] = (out, tr, np.stack(all_logits))
    finally:
        T.tasc_config_set(T.TASC_CFG_SMALL_KERNEL, 1)
        T.tasc_config_set(T.TASC_CFG_SMALL_PATH, 2)
        T.tasc_config_set(T.TASC_CFG_SMALL_XCD_LOCAL, 1)
        T.tasc_config_set(T.TASC_CFG_SMALL_LAYER_WORKERS, 0)
    for other in (6, 2, 1, 3, 4):
        assert (results[other][0] == results[5][0]).all() and (results[other][1] == results[5][1]).all(), f"mode {other}"
        assert (results[other][2] == results[5][2]).all(), f"mode {other}: the pipeline kernel, the barrier kernel (XCD-local " \
            "or agent-scope barriers) and their per-phase launches must be bit-identical"


@pytest.mark.parametrize("heads", [(4, 2, 64), (2, 1, 128), (6, 2, 32)])
def test_tiled_mfma_kernels(heads):
    """bf16 forwards of more than 16 rows run on the LDS-tiled MFMA GEMMs and the MFMA paged attention:
    several row tiles, ragged last tiles, against the oracle and against the type-generic kernels."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    H, Hkv, hd = heads
    cfg = W.get_config("cfg1").scaled(dtype="bf16", n_layers=2, d_model=256 if H * hd == 256 else 192, n_heads=H, n_kv_heads=Hkv,
                                      head_dim=hd, d_ffn=448, vocab=1000, batch=28, prompt_len=40, gen_len=24, k=7,
                                      n_docs=1500, n_max=4)
    rig = Rig(cfg, max_rows=16)                    # prompt chunks: 28 x 16 = 448 rows (256 x 256 tiles), verify: 28 x 8 = 224 rows (128 x 128 tiles)
    lens = [40 - (b * 7) % 30 for b in range(cfg.batch)]
    rng = np.random.default_rng(11)
    prompts = [rng.integers(0, cfg.vocab, n).astype(np.int32) for n in lens]
    rig.prompts = np.concatenate(prompts)
    rig.prompt_off = np.cumsum([0] + lens).astype(np.int64)
    ref_tables = ON.build_tables_flat(rig.corpus[0], rig.corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    om = OM.OracleModel(cfg, rig.weights)
    check = [0, 7, 27]                             # sequences whose logits the oracle follows
    outs = {}
    try:
        for tiled in (1, 0):
            print(f"heads {heads} tiled {tiled}", flush=True)
            T.tasc_config_set(T.TASC_CFG_TILED_PATH, tiled)
            out, st, tr = rig.generate(trace_steps=cfg.gen_len)
            g_out, g_st, _ = rig.generate(k=0)
            assert (out == g_out).all(), f"tiled {tiled}: speculative output differs from greedy"
            for b in range(cfg.batch):
                _replay(cfg, ref_tables, prompts[b].tolist(), tr[:, b], cfg.k, cfg.lambda_q16, cfg.p_min_ctx, out[b])
            T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
            caches = {}
            for b in check:
                c = om.new_cache(rig.max_len)
                om.forward(prompts[b].tolist(), c, last_only=True)
                c.length = lens[b]
                caches[b] = c
            logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
            drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
            worst = 0.0
            for s in range(3):
                T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
                before = {b: T.tasc_session_get_tokens(rig.session, b) for b in check}
                T.tasc_verify_step(rig.model, rig.session, drafts, cfg.k, None, None, logits)
                got = logits.cpu().numpy()
                d = drafts.cpu().numpy()
                for b in check:
                    z = om.forward([int(before[b][-1])] + d[b].tolist(), caches[b])
                    worst = max(worst, float(np.abs(got[b].astype(np.float64) - z).max()))
                    after = T.tasc_session_get_tokens(rig.session, b)
                    caches[b].length += len(after) - len(before[b])
            print(f"tiled {tiled}: max |logit - oracle| = {worst:.3e}, steps {st.steps}", flush=True)
            assert worst <= 5e-2
            outs[tiled] = out
    finally:
        T.tasc_config_set(T.TASC_CFG_TILED_PATH, 1)


def test_tiled_step_graph_and_chains():
    """Verify steps of the tiled kernels replayed from a recorded graph, and the layers run as several chains of
    sequences on streams of their own, give the tokens, accept lengths and counters of plain launches on one stream:
    every replay is checked (the graph is recorded at the second step and replayed from then on, with host reads and
    synchronisations between the steps), then whole generations."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    cfg = W.get_config("cfg1").scaled(dtype="bf16", n_layers=2, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=448,
                                      vocab=1000, batch=28, prompt_len=40, gen_len=40, k=4, n_docs=1500, n_max=4)
    rig = Rig(cfg, max_rows=16)
    drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    emitted = torch.zeros((cfg.batch, cfg.k + 1), dtype=torch.int32, device="cuda")
    runs = {}
    try:
        for graph, chains in ((0, 1), (1, 1), (0, 3), (1, 2), (1, 4)):
            print(f"graph {graph} chains {chains}", flush=True)
            T.tasc_config_set(T.TASC_CFG_STEP_GRAPH, graph)
            T.tasc_config_set(T.TASC_CFG_CHAINS, chains)
            T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
            steps = []
            for s in range(7):
                T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
                T.tasc_verify_step(rig.model, rig.session, drafts, cfg.k, acc, emitted)
                torch.cuda.synchronize()
                steps.append((drafts.cpu().numpy().copy(), acc.cpu().numpy().copy(), emitted.cpu().numpy().copy(),
                              [T.tasc_session_get_tokens(rig.session, b).copy() for b in (0, 13, 27)]))
            out, st, _ = rig.generate()
            g_out, _, _ = rig.generate(k=0)
            assert (out == g_out).all(), f"graph {graph} chains {chains}: speculative output differs from greedy"
            runs[(graph, chains)] = (steps, out, (st.steps, st.accepted, st.proposed, tuple(st.accept_hist)))
    finally:
        T.tasc_config_set(T.TASC_CFG_STEP_GRAPH, 1)
        T.tasc_config_set(T.TASC_CFG_CHAINS, 0)
    ref_steps, ref_out, ref_stats = runs[(0, 1)]
    assert sum(int(a.sum()) for _, a, _, _ in ref_steps) > 0, "no draft was ever accepted: the test would compare nothing"
    for key, (steps, out, stats) in runs.items():
        for s, (a, b) in enumerate(zip(ref_steps, steps)):
            assert (a[0] == b[0]).all() and (a[1] == b[1]).all(), f"{key} step {s}"
            m = a[1]
            for row in range(cfg.batch):
                assert (a[2][row, :m[row] + 1] == b[2][row, :m[row] + 1]).all(), f"{key} step {s} sequence {row}"
            assert all((x == y).all() for x, y in zip(a[3], b[3])), f"{key} step {s}"
        assert (out == ref_out).all() and stats == ref_stats, key


@pytest.mark.parametrize("shape", ["two_row_passes_long_keys", "one_chunk_many_sequences", "hd128_long_keys"])
def test_staged_attention_shapes(shape):
    """The LDS-staged attention at the edges of its launch shapes: more than 64 (row, head) pairs per KV head (two row
    passes), several key tiles per chunk and chunks without tiles, and so many sequences that every KV head runs as one
    chunk (no merge kernel); speculative = greedy and logits against the oracle."""
    import torch
    import paper_2602_24174_amd as T
    from gpu_util import Rig
    base = W.get_config("cfg1")
    if shape == "two_row_passes_long_keys":
        # 14 query heads on 2 KV heads: 7 x 16 prompt rows = 112 pairs per KV head; prompts of up to 700 tokens = 11 key tiles
        cfg = base.scaled(dtype="bf16", n_layers=2, d_model=128, n_heads=14, n_kv_heads=2, head_dim=64, d_ffn=256, vocab=800,
                          batch=3, prompt_len=700, gen_len=20, k=9, n_docs=1200, n_max=3)
        lens, check = [700, 333, 65], [0, 1, 2]
    elif shape == "one_chunk_many_sequences":
        cfg = base.scaled(dtype="bf16", n_layers=1, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=128, vocab=600,
                          batch=140, prompt_len=70, gen_len=12, k=3, n_docs=1200, n_max=3)
        lens, check = [70 - (b * 5) % 66 for b in range(140)], [0, 13, 139]
    else:
        cfg = base.scaled(dtype="bf16", n_layers=2, d_model=128, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=256, vocab=800,
                          batch=2, prompt_len=1100, gen_len=16, k=15, n_docs=1200, n_max=3)
        lens, check = [1100, 129], [0, 1]
    rig = Rig(cfg, max_rows=16)
    rng = np.random.default_rng(23)
    prompts = [rng.integers(0, cfg.vocab, n).astype(np.int32) for n in lens]
    rig.prompts = np.concatenate(prompts)
    rig.prompt_off = np.cumsum([0] + lens).astype(np.int64)
    print(f"{shape}: batch {cfg.batch}, heads {cfg.n_heads}/{cfg.n_kv_heads} x {cfg.head_dim}, longest prompt {max(lens)}", flush=True)
    out, st, _ = rig.generate()
    g_out, g_st, _ = rig.generate(k=0)
    assert (out == g_out).all(), "speculative output differs from greedy"
    assert g_st.steps == cfg.gen_len - 1
    om = OM.OracleModel(cfg, rig.weights)
    T.tasc_session_prefill(rig.model, rig.session, rig.prompts, rig.prompt_off, cfg.gen_len)
    caches = {}
    for b in check:
        c = om.new_cache(rig.max_len)
        z = om.forward(prompts[b].tolist(), c, last_only=True)
        c.length = lens[b]
        caches[b] = c
        first = T.tasc_session_get_tokens(rig.session, b)[-1]
        top2 = np.sort(z[0])[-2:]
        assert first == int(np.argmax(z[0])) or top2[1] - top2[0] < 0.1
    logits = torch.zeros((cfg.batch, cfg.k + 1, cfg.vocab), dtype=torch.float32, device="cuda")
    drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    worst = 0.0
    for s in range(2):
        T.tasc_draft(rig.ng, rig.session, rig.params(), drafts)
        before = {b: T.tasc_session_get_tokens(rig.session, b) for b in check}
        T.tasc_verify_step(rig.model, rig.session, drafts, cfg.k, None, None, logits)
        got = logits.cpu().numpy()
        d = drafts.cpu().numpy()
        for b in check:
            z = om.forward([int(before[b][-1])] + d[b].tolist(), caches[b])
            worst = max(worst, float(np.abs(got[b].astype(np.float64) - z).max()))
            after = T.tasc_session_get_tokens(rig.session, b)
            caches[b].length += len(after) - len(before[b])
    print(f"{shape}: max |logit - oracle| = {worst:.3e}", flush=True)
    assert worst <= 5e-2
