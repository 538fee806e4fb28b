#!/usr/bin/env python3
"""Benchmark of the TASC-spec hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: corpus n-gram table build
(tasc_ngram_build, corpus resident in HBM) followed by tasc_generate (prompt forward, then draft /
verify / accept until every sequence has its tokens).  The headline value is emitted tokens per second
of the decode loop (accepted drafts + bonus tokens, first max_new per sequence) on the 135M-class
bf16, batch-1 workload; the whole step's time is ms_per_step.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def algorithmic_bytes_verify(cfg, mean_cached_len):
    """Bytes one verify step has to move (per launch of the whole step): every weight once, the live
    KV once per KV head, the k+1 new KV rows written.  Activations and logits are not counted."""
    es = 2 if cfg.dtype == "bf16" else 4
    hd_q, hd_kv = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    per_layer = cfg.d_model * (hd_q + 2 * hd_kv) + hd_q * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn
    weights = (cfg.n_layers * per_layer + cfg.vocab * cfg.d_model) * es
    kv_tok = cfg.n_layers * 2 * hd_kv * es
    kv_read = cfg.batch * mean_cached_len * kv_tok
    kv_write = cfg.batch * (cfg.k + 1) * kv_tok
    return weights + kv_read + kv_write, {"weights": weights, "kv_read": kv_read, "kv_write": kv_write}


def cpu_baseline(cfg, corpus, weights, prompts, max_steps):
    """The CPU oracle as it stands, timed on this host: table build, prompt forward of sequence 0 and
    up to `max_steps` draft/verify steps.  Reported as emitted tokens per second of the decode loop."""
    from oracle import model as OM
    from oracle import ngram as ON
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.time()
    tables = ON.build_tables_flat(corpus[0], corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    t_build = time.time() - t0
    om = OM.OracleModel(cfg, weights)
    prompt = [int(t) for t in prompts[:cfg.prompt_len]]
    cache = om.new_cache(cfg.prompt_len + cfg.gen_len + 2 * (cfg.k + 1))
    t0 = time.time()
    z = om.forward(prompt, cache, last_only=True)
    cache.length = len(prompt)
    t_prefill = time.time() - t0
    out = [int(np.argmax(z[0]))]
    t0 = time.time()
    steps = 0
    while len(out) < cfg.gen_len and steps < max_steps:
        d = ON.draft(tables, prompt + out, cfg.k, cfg.lambda_q16, cfg.p_min_ctx)
        z = om.forward([out[-1]] + d, cache)
        a = OM.argmax_lowest(z)
        m = OM.accept_length(d, a)
        out += d[:m] + [int(a[m])]
        cache.length += m + 1
        steps += 1
    t_decode = time.time() - t0
    emitted = min(len(out), cfg.gen_len) - 1
    return {"value": emitted / t_decode if t_decode > 0 else None, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{cfg.name} sequence 0: full table build ({t_build:.2f} s), full prompt forward ({t_prefill:.2f} s), "
                      f"{steps} draft+verify steps emitting {emitted} tokens in {t_decode:.2f} s (decode loop only in value)",
            "build_s": t_build, "prefill_s": t_prefill, "decode_s": t_decode, "steps": steps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--cpu-steps", type=int, default=24, help="draft+verify steps of the CPU oracle sample (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB plain copy kernel 4 times (reference for rocprofv3 byte counters)")
    ap.add_argument("--max-rows", type=int, default=0, help="rows per sequence and forward (prompt chunk length); 0 = default")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus {args.gpus} is not supported",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workload as W
    import paper_2602_24174_amd as T

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    T.lib()

    def note(msg):                                  # progress on stderr: the one JSON line stays alone on stdout
        print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

    cfg = W.get_config(args.config)
    note(f"{cfg.name}: generating corpus")
    corpus = W.make_corpus(cfg)
    note(f"corpus {corpus[0].shape[0]} tokens; generating weights")
    weights = W.make_model(cfg, corpus)
    note("weights done")
    prompts, poff = W.make_prompts(cfg)
    max_rows = args.max_rows or max(cfg.k + 1, 512 if cfg.batch == 1 else 64)
    max_len = cfg.prompt_len + cfg.gen_len + 2 * max_rows
    small = cfg.batch * min(max_rows, 16) <= 16   # decode steps then run on the persistent fused kernel
    model = T.tasc_model_create(cfg, weights, max_len)
    session = T.tasc_session_create(model, cfg.batch, max_len, max_rows)
    d_corpus = torch.from_numpy(corpus[0]).cuda()           # inputs resident in HBM before the timed region
    d_prompts = torch.from_numpy(prompts).cuda()
    out = torch.zeros((cfg.batch, cfg.gen_len), dtype=torch.int32, device="cuda")
    params = T.spec_params(cfg.k, cfg.lambda_q16, cfg.p_min_ctx, 1)
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        ng = T.tasc_ngram_build(d_corpus, corpus[1], cfg.vocab, cfg.n_max, cfg.p_min, stream)
        st = T.tasc_generate(model, ng, session, d_prompts, poff, cfg.gen_len, params, out, None, 0, stream)
        bs = T.tasc_ngram_get_stats(ng)
        ng.close()
        return st, bs

    note("model and session on the device; warm-up")
    for _ in range(args.warmup):
        step()
    note("timed region")
    T.tasc_profile_enable(["layers" if small else "verify"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = [step() for _ in range(args.steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = T.tasc_profile_read()
    T.tasc_profile_enable([])
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    decode_ms = sum(s.decode_ms for s, _ in stats)
    prefill_ms = sum(s.prefill_ms for s, _ in stats) / args.steps
    build_ms = sum(b.build_ms for _, b in stats) / args.steps
    tokens = sum(s.emitted for s, _ in stats)
    value = tokens / (decode_ms / 1e3)
    vsteps = sum(s.steps for s, _ in stats)
    accepted = sum(s.accepted for s, _ in stats)
    proposed = sum(s.proposed for s, _ in stats)
    hist = [sum(s.accept_hist[i] for s, _ in stats) for i in range(cfg.k + 1)]
    spec_tokens = out.cpu().numpy().copy()

    # the GPU's own plain greedy decode: speed-up ratio and the token-identity check
    g_stats = T.tasc_generate(model, None, session, d_prompts, poff, cfg.gen_len, T.spec_params(0), out, None, 0, stream)
    identical = bool((out.cpu().numpy() == spec_tokens).all())
    greedy_tps = g_stats.emitted / (g_stats.decode_ms / 1e3)

    # roofline of the dominant kernel: the verify step (weights + live KV streamed once per step)
    # (the event pairs also bracket the 32 prompt-chunk launches of the same kernel: identical weight traffic)
    ver_ms, ver_n = prof.get("layers" if small else "verify", (0.0, 0))
    mean_len = cfg.prompt_len + cfg.gen_len / 2.0
    alg_bytes, parts = algorithmic_bytes_verify(cfg, mean_len)
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy kernel);
    # a separate profiler run, so the figure comes from its committed summary and only for the workload it covers
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "cfg2_k_small_step_hbm_traffic.txt")
    if small and cfg.name == "cfg2" and os.path.exists(tpath):
        for ln in open(tpath):
            if ln.startswith("traffic_bytes_per_launch:"):
                traffic = int(ln.split(":")[1])
    roofline = None
    if ver_n:
        avg_ms = ver_ms / ver_n
        achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": traffic, "kernel": ("k_small_step (persistent fused forward: all layers + LM head + argmax + accept in one launch)" if small
                               else "verify step (all kernels of one target forward + accept)"),
                    "avg_launch_ms": avg_ms, "launches": ver_n, "algorithmic_bytes": alg_bytes, "bytes_breakdown": parts}

    note("timed region done")
    if args.calibrate_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            T.tasc_calibration_copy(dst, src, stream)
        torch.cuda.synchronize()
        del src, dst
    cpu = None
    if args.cpu_steps > 0:
        cpu = cpu_baseline(cfg, corpus, weights, prompts, args.cpu_steps)

    line = {
        "metric": "accepted tokens/s/GPU + verify-step HBM GB/s (fraction of peak)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}-layer d{cfg.d_model} {cfg.n_heads}/{cfg.n_kv_heads} heads ffn{cfg.d_ffn} "
                               f"vocab{cfg.vocab} {cfg.dtype}; corpus {cfg.n_docs} outputs ({corpus[0].shape[0]} tokens); "
                               f"n_max {cfg.n_max}, k {cfg.k}, p_min {cfg.p_min}, lambda {cfg.lam}; batch {cfg.batch}, "
                               f"prompt {cfg.prompt_len}, generate {cfg.gen_len}",
                   "batch": cfg.batch, "k": cfg.k, "n_max": cfg.n_max, "prompt_len": cfg.prompt_len, "gen_len": cfg.gen_len},
        "value_basis": "emitted tokens (accepted drafts + bonus) / decode-loop device time; the step also holds build and prefill",
        "phases_ms": {"ngram_build": build_ms, "prefill": prefill_ms, "decode": decode_ms / args.steps},
        "verify_steps_per_generate": vsteps / args.steps,
        "xcd_local_steps_per_generate": sum(s.xcd_local_steps for s, _ in stats) / args.steps,
        "mean_accept_len": accepted / max(1, vsteps * cfg.batch),
        "accepted_draft_tokens_per_s": accepted / (decode_ms / 1e3),
        "accept_hist": hist, "proposed": proposed,
        "greedy_tokens_per_s": greedy_tps, "speedup_vs_gpu_greedy": value / greedy_tps, "spec_equals_greedy": identical,
        "build_Mwindows_per_s": (sum(stats[0][1].windows) / 1e6) / (stats[0][1].count_ms / 1e3) if stats[0][1].count_ms else None,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
