#!/usr/bin/env python3
"""Benchmark of the TASC-spec hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: corpus n-gram table build
(tasc_ngram_build, corpus resident in HBM) followed by tasc_generate (prompt forward, then draft /
verify / accept until every sequence has its tokens).  The headline is the largest single-GPU
workload (the 3B-class bf16 model, 256 sequences): `value` = emitted tokens per second of its decode
loop (accepted drafts + bonus tokens, first max_new per sequence, all sequences), `roofline` = the
matrix-product rate of its verify step against the bf16 MFMA peak, with the HBM figure beside it.
`per_config` carries the same figures for all five workloads (tokens/s, median verify-step latency,
HBM and MFMA fractions, speculative == greedy), one of them also with a weak LM-head bias so that
few drafts are accepted.

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

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
# HBM bytes of one verify step from rocprofv3 hardware counters (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter
# reads for a plain copy kernel of known size); bench.py cannot collect counters itself, so the figure of the committed
# counter runs is carried here, for the workload they were taken on only
MEASURED_TRAFFIC = {"cfg5": 29473969869}
MEASURED_TRAFFIC_SOURCE = "profiles/cfg5_verify_step_hbm_traffic.txt (bytes per verify step: every kernel of the step)"
MFMA_PEAK_TFLOPS = 2500.0    # MI355X published dense bf16 matrix rate
FP32_PEAK_TFLOPS = 157.3     # fp32 vector rate (the fp32 configuration runs on the type-generic kernels)


def note(msg):                                  # progress on stderr: the one JSON line stays alone on stdout
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes_verify(cfg, mean_cached_len):
    """Bytes one verify step has to move: every weight once, the live KV once per KV head, the k+1 new
    KV rows written.  Activations and logits are not counted."""
    es = 2 if cfg.dtype == "bf16" else 4
    hd_q, hd_kv = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    per_layer = cfg.d_model * (hd_q + 2 * hd_kv) + hd_q * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn
    weights = (cfg.n_layers * per_layer + cfg.vocab * cfg.d_model) * es
    kv_tok = cfg.n_layers * 2 * hd_kv * es
    kv_read = cfg.batch * mean_cached_len * kv_tok
    kv_write = cfg.batch * (cfg.k + 1) * kv_tok
    return weights + kv_read + kv_write, {"weights": weights, "kv_read": kv_read, "kv_write": kv_write}


def algorithmic_flops_verify(cfg, mean_cached_len):
    """Matrix-product flops of one verify step: 2 x parameters x rows (layers and LM head), and beside it the two
    attention products over the live keys."""
    hd_q, hd_kv = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    per_layer = cfg.d_model * (hd_q + 2 * hd_kv) + hd_q * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn
    rows = cfg.batch * (cfg.k + 1)
    gemm = 2.0 * (cfg.n_layers * per_layer + cfg.vocab * cfg.d_model) * rows
    attn = 4.0 * cfg.n_layers * rows * hd_q * mean_cached_len
    return gemm, attn


def run_config(T, torch, W, cfg, steps, warmup, corpus=None, weights=None, label=None):
    """Builds the workload, runs `warmup` + `steps` whole steps, returns (figures, corpus, weights, prompts)."""
    label = label or cfg.name
    if corpus is None:
        note(f"{label}: generating corpus")
        corpus = W.make_corpus(cfg)
    if weights is None:
        note(f"{label}: corpus {corpus[0].shape[0]} tokens; generating weights")
        weights = W.make_model(cfg, corpus)
    prompts, poff = W.make_prompts(cfg)
    max_rows = max(cfg.k + 1, 512 if cfg.batch == 1 else 64)
    max_len = cfg.prompt_len + cfg.gen_len + 2 * max_rows
    small = cfg.dtype == "bf16" and cfg.batch * min(max_rows, 16) <= 16      # decode steps on the persistent kernel
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

    note(f"{label}: model and session on the device; {warmup} warm-up + {steps} timed steps")
    for _ in range(warmup):
        step()
    # Timed region: event pairs around every verify step and draft call only (and around the one kernel of a small-batch
    # step).  Brackets around single kernels of the tiled step would switch its graph replay off and put an event between
    # every two launches, so the largest kernel's own duration is taken in one extra, untimed generate afterwards.
    classes = ["verify", "draft"] + (["layers"] if small else [])
    T.tasc_profile_enable(classes)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = [step() for _ in range(steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dur = {c: T.tasc_profile_durations(c) for c in classes}
    T.tasc_profile_read()
    T.tasc_profile_enable([])
    if not small:
        T.tasc_profile_enable(["gemm_gu"])
        step()
        torch.cuda.synchronize()
        dur["gemm_gu"] = T.tasc_profile_durations("gemm_gu")
        T.tasc_profile_read()
        T.tasc_profile_enable([])
    ms_per_step = (t1 - t0) * 1e3 / steps
    decode_ms = sum(s.decode_ms for s, _ in stats)
    tokens = sum(s.emitted for s, _ in stats)
    vsteps = sum(s.steps for s, _ in stats)
    accepted = sum(s.accepted for s, _ in stats)
    spec_tokens = out.cpu().numpy().copy()

    # the GPU's own plain greedy decode: speed-up ratio and the token-identity check
    g = T.tasc_generate(model, None, session, d_prompts, poff, cfg.gen_len, T.spec_params(0), out, None, 0, stream)
    identical = bool((out.cpu().numpy() == spec_tokens).all())
    greedy_tps = g.emitted / (g.decode_ms / 1e3)

    mean_len = cfg.prompt_len + cfg.gen_len / 2.0
    alg_bytes, parts = algorithmic_bytes_verify(cfg, mean_len)
    gemm_flops, attn_flops = algorithmic_flops_verify(cfg, mean_len)
    med_verify = float(np.median(dur["verify"])) if dur["verify"].size else None
    fig = {
        "config": cfg.name if label == cfg.name else label,
        "workload": f"{cfg.n_layers}-layer d{cfg.d_model} {cfg.n_heads}/{cfg.n_kv_heads} heads ffn{cfg.d_ffn} vocab{cfg.vocab} {cfg.dtype}; "
                    f"corpus {cfg.n_docs} outputs ({corpus[0].shape[0]} tokens); n_max {cfg.n_max}, k {cfg.k}, p_min {cfg.p_min}, "
                    f"lambda {cfg.lam}, LM-head bias {cfg.bias_alpha}; batch {cfg.batch}, prompt {cfg.prompt_len}, generate {cfg.gen_len}",
        "dtype": cfg.dtype, "rows_per_verify_step": cfg.batch * (cfg.k + 1),
        "tokens_per_s": tokens / (decode_ms / 1e3), "accepted_draft_tokens_per_s": accepted / (decode_ms / 1e3),
        "ms_per_step": ms_per_step,
        "phases_ms": {"ngram_build": sum(b.build_ms for _, b in stats) / steps, "prefill": sum(s.prefill_ms for s, _ in stats) / steps,
                      "decode": decode_ms / steps},
        "verify_steps_per_generate": vsteps / steps,
        "verify_step_ms_median": med_verify,
        "verify_step_ms_mean": float(dur["verify"].mean()) if dur["verify"].size else None,
        "draft_call_us_median": float(np.median(dur["draft"])) * 1e3 if dur["draft"].size else None,
        "mean_accept_len": accepted / max(1, vsteps * cfg.batch),
        "accept_hist": [sum(s.accept_hist[i] for s, _ in stats) for i in range(cfg.k + 1)],
        "greedy_tokens_per_s": greedy_tps, "speedup_vs_gpu_greedy": (tokens / (decode_ms / 1e3)) / greedy_tps,
        "spec_equals_greedy": identical,
        "build_Mwindows_per_s": (sum(stats[0][1].windows) / 1e6) / (stats[0][1].count_ms / 1e3) if stats[0][1].count_ms else None,
        "algorithmic_bytes_per_verify_step": alg_bytes, "bytes_breakdown": parts,
        "algorithmic_gemm_flops_per_verify_step": gemm_flops, "attention_flops_per_verify_step": attn_flops,
    }
    if med_verify:
        peak_tf = MFMA_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_PEAK_TFLOPS
        fig["hbm_gbs"] = alg_bytes / (med_verify * 1e-3) / 1e9
        fig["hbm_frac"] = fig["hbm_gbs"] / HBM_PEAK_GBS
        fig["gemm_tflops"] = gemm_flops / (med_verify * 1e-3) / 1e12
        fig["mfma_frac"] = fig["gemm_tflops"] / peak_tf
        fig["matrix_peak_tflops"] = peak_tf
    if small and dur["layers"].size:
        # the one kernel of the small-batch verify step: every layer, the LM head, the argmax and the accept in one launch
        k_ms = float(np.median(dur["layers"]))
        fig["step_kernel"] = {"name": "k_pipe_step (one persistent launch per verify step)", "median_launch_ms": k_ms,
                              "mean_launch_ms": float(dur["layers"].mean()), "launches": int(dur["layers"].size),
                              "hbm_gbs": alg_bytes / (k_ms * 1e-3) / 1e9, "hbm_frac": alg_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if not small and dur["gemm_gu"].size:
        # the largest kernel of the tiled verify step: gate/up projection + SwiGLU (one launch per layer; prompt chunks of
        # other row counts are bracketed too, so only the launches of the verify shape are taken: the most frequent duration class)
        gu = np.sort(dur["gemm_gu"])
        gu = gu[: max(1, int(gu.size * 0.9))] if cfg.prompt_len > 0 else gu
        flops = 2.0 * 2 * cfg.d_ffn * cfg.d_model * cfg.batch * (cfg.k + 1)
        k_ms = float(np.median(gu))
        fig["largest_kernel"] = {"name": "k_gemm_tiled (gate/up projection + SwiGLU)", "median_launch_ms": k_ms, "launches": int(dur["gemm_gu"].size),
                                 "measured": "HIP event pairs around each launch, in one extra untimed generate (plain launches; the pair itself adds a few us)",
                                 "tflops": flops / (k_ms * 1e-3) / 1e12, "mfma_frac": flops / (k_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS}
    del model, session, d_corpus, d_prompts, out
    torch.cuda.empty_cache()
    return fig, corpus, weights, prompts


def cpu_baseline(W, cfg, corpus, weights, prompts, prompt_tokens, doc_share):
    """The CPU oracle as it stands, timed on this host, on a bounded sample of the headline workload: tables from the
    first 1/doc_share of the corpus, sequence 0 with its prompt cut to `prompt_tokens`, one draft + verify step."""
    from oracle import model as OM
    from oracle import ngram as ON
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_docs = max(1, cfg.n_docs // doc_share)
    off = corpus[1][:n_docs + 1]
    tok = corpus[0][:off[-1]]
    t0 = time.time()
    tables = ON.build_tables_flat(tok, off, cfg.vocab, cfg.n_max, cfg.p_min)
    t_build = time.time() - t0
    om = OM.OracleModel(cfg, weights)
    prompt = [int(t) for t in prompts[:prompt_tokens]]
    cache = om.new_cache(prompt_tokens + 2 * (cfg.k + 1))
    t0 = time.time()
    z = om.forward(prompt, cache, last_only=True)
    cache.length = len(prompt)
    t_prefill = time.time() - t0
    out = [int(np.argmax(z[0]))]
    t0 = time.time()
    d = ON.draft(tables, prompt + out, cfg.k, cfg.lambda_q16, cfg.p_min_ctx)
    z = om.forward([out[-1]] + d, cache)
    a = OM.argmax_lowest(z)
    m = OM.accept_length(d, a)
    t_step = time.time() - t0
    return {"value": (m + 1) / t_step, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{cfg.name}, sequence 0 only: tables from the first {n_docs} of {cfg.n_docs} outputs ({t_build:.1f} s), prompt cut to "
                      f"{prompt_tokens} tokens ({t_prefill:.1f} s), ONE draft + verify step of {cfg.k + 1} rows emitting {m + 1} tokens in "
                      f"{t_step:.1f} s; value = those tokens / that step (the GPU figure covers {cfg.batch} sequences)",
            "build_s": t_build, "prefill_s": t_prefill, "verify_step_s": t_step, "emitted": m + 1}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg5", help="the headline workload")
    ap.add_argument("--others", default="cfg1,cfg2,cfg3,cfg4", help="workloads reported in per_config beside the headline ('' = none)")
    ap.add_argument("--low-accept", default="cfg3", help="workload that is also run with LM-head bias 1 (few drafts accepted; '' = none)")
    ap.add_argument("--cpu", type=int, default=1, help="1: time the CPU oracle on a bounded sample of the headline workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB plain copy kernel 4 times (the known-size reference for rocprofv3 byte counters)")
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

    per_config = []
    others = [n for n in args.others.split(",") if n and n != args.config]
    for name in others:
        cfg = W.get_config(name)
        fig, corpus, weights, _ = run_config(T, torch, W, cfg, 2, 1)
        per_config.append(fig)
        if name == args.low_accept:
            # same corpus and matrices, LM-head bias strength 1 instead of 8: the target no longer follows the corpus'
            # bigram chain, so acceptance falls with the draft position as in the paper's experiments
            low = cfg.scaled(bias_alpha=1.0)
            w2 = dict(weights)
            w2["bias"] = W.model.bigram_bias_csr(corpus[0], corpus[1], low.vocab, low.bias_alpha)
            fig2, _, _, _ = run_config(T, torch, W, low, 2, 1, corpus=corpus, weights=w2, label=f"{name} with LM-head bias 1 (low acceptance)")
            per_config.append(fig2)
        del corpus, weights

    cfg = W.get_config(args.config)
    head, corpus, weights, prompts = run_config(T, torch, W, cfg, args.steps, args.warmup)
    per_config.append(head)
    note("timed region done")
    if args.calibrate_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            T.tasc_calibration_copy(dst, src, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del src, dst
    cpu = None
    if args.cpu:
        note("CPU oracle sample")
        cpu = cpu_baseline(W, cfg, corpus, weights, prompts, 16, 16)
        note("CPU oracle sample done")

    bf16 = cfg.dtype == "bf16"
    compute_bound = cfg.batch * (cfg.k + 1) >= 310        # rows above the ridge of 2.5 PFLOP/s over 8 TB/s
    med = head["verify_step_ms_median"]
    hbm = {"bound": "hbm", "achieved": head.get("hbm_gbs"), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head.get("hbm_frac"),
           "algorithmic_bytes": head["algorithmic_bytes_per_verify_step"], "bytes_breakdown": head["bytes_breakdown"]}
    mfma = {"bound": "mfma", "achieved": head.get("gemm_tflops"), "peak": head.get("matrix_peak_tflops"), "unit": "TFLOP/s",
            "frac": head.get("mfma_frac"), "algorithmic_flops": head["algorithmic_gemm_flops_per_verify_step"]}
    roofline = dict(mfma if (compute_bound and bf16) else hbm)
    roofline.update({"traffic": MEASURED_TRAFFIC.get(cfg.name), "traffic_source": MEASURED_TRAFFIC_SOURCE if cfg.name in MEASURED_TRAFFIC else None,
                     "kernel": "verify step: every kernel of one target forward over batch x (k+1) rows, the LM head with argmax, and the accept "
                               "(HIP events around each step on the launch stream; median over the timed region)",
                     "median_launch_ms": med, "launches": int(head["verify_steps_per_generate"] * args.steps),
                     "other_bound": hbm if (compute_bound and bf16) else mfma})
    for k in ("largest_kernel", "step_kernel"):
        if k in head:
            roofline[k] = head[k]

    line = {
        "metric": "accepted tokens/s/GPU + verify-step HBM GB/s (fraction of peak)",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {head['workload']}", "batch": cfg.batch, "k": cfg.k, "n_max": cfg.n_max,
                   "prompt_len": cfg.prompt_len, "gen_len": cfg.gen_len},
        "value_basis": "emitted tokens (accepted drafts + bonus, all sequences) / decode-loop device time; one step = table build + prompt forward + decode",
        "phases_ms": head["phases_ms"], "verify_steps_per_generate": head["verify_steps_per_generate"],
        "verify_step_ms_median": med, "mean_accept_len": head["mean_accept_len"], "accept_hist": head["accept_hist"],
        "accepted_draft_tokens_per_s": head["accepted_draft_tokens_per_s"],
        "greedy_tokens_per_s": head["greedy_tokens_per_s"], "speedup_vs_gpu_greedy": head["speedup_vs_gpu_greedy"],
        "spec_equals_greedy": head["spec_equals_greedy"], "build_Mwindows_per_s": head["build_Mwindows_per_s"],
        "roofline": roofline, "cpu_baseline": cpu, "per_config": per_config,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
