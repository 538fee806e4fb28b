"""A bare loop of draft + verify steps on one workload, for profilers and counter runs: no events, no host reads
between the steps, nothing but the hot path's own kernels after the set-up.

    python -m paper_2602_24174_amd.verify_loop [--config cfg5] [--docs 2000] [--steps 12] [--max-rows 64]

    rocprofv3 --kernel-trace --stats -- python -m paper_2602_24174_amd.verify_loop --config cfg5
    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum -- python -m paper_2602_24174_amd.verify_loop --config cfg5

Set-up (untimed): synthetic corpus (--docs outputs: the tables only shape the drafts, so a small corpus does for
kernel profiles of the verify step), tables, model, session, prompt prefill.  Then --steps times tasc_draft +
tasc_verify_step at the configuration's batch and draft length, one synchronisation at the end, and the mean wall time
of a step.  In a trace the verify-step launches are told from the prefill's by their grid size.
"""
import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--docs", type=int, default=2000, help="corpus size (0 = the configuration's)")
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--max-rows", type=int, default=64, help="rows per sequence of a prompt chunk")
    ap.add_argument("--chains", type=int, default=0, help="sequence ranges whose layers run side by side (0 = the library's rule)")
    ap.add_argument("--graph", type=int, default=1, help="1: the step is recorded into a graph and replayed (the library's default), 0: plain launches")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB plain copy kernel 4 times (the known-size reference for rocprofv3 byte counters)")
    ap.add_argument("--progress", action="store_true", help="synchronise and print after every step (for slow counter runs)")
    ap.add_argument("--warm", type=int, default=0, help="untimed steps before the timed ones")
    args = ap.parse_args()
    import torch
    import workload as W
    import paper_2602_24174_amd as T
    cfg = W.get_config(args.config)
    if args.docs:
        cfg = cfg.scaled(n_docs=args.docs)
    corpus = W.make_corpus(cfg)
    weights = W.make_model(cfg, corpus)
    max_rows = max(args.max_rows, cfg.k + 1)
    max_len = cfg.prompt_len + cfg.gen_len + 2 * max_rows
    model = T.tasc_model_create(cfg, weights, max_len)
    table = T.tasc_ngram_build(corpus[0], corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    session = T.tasc_session_create(model, cfg.batch, max_len, max_rows)
    prompts, prompt_off = W.make_prompts(cfg)
    print(f"{cfg.name}: set-up done, prompt forward", flush=True)
    T.tasc_session_prefill(model, session, prompts, prompt_off, cfg.gen_len)
    torch.cuda.synchronize()
    print(f"{cfg.name}: prompt forward done", flush=True)
    params = T.spec_params(cfg.k, cfg.lambda_q16, cfg.p_min_ctx, 1)
    drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    steps = min(args.steps, (cfg.gen_len - 1) // (cfg.k + 1) - args.warm)      # stay inside the session's generation budget
    T.tasc_config_set(T.TASC_CFG_CHAINS, args.chains)
    T.tasc_config_set(T.TASC_CFG_STEP_GRAPH, args.graph)
    for _ in range(args.warm):
        T.tasc_draft(table, session, params, drafts)
        T.tasc_verify_step(model, session, drafts, cfg.k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        T.tasc_draft(table, session, params, drafts)
        T.tasc_verify_step(model, session, drafts, cfg.k)
        if args.progress:
            torch.cuda.synchronize()
            print(f"step {i + 1} of {steps} done", flush=True)
    t_host = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if args.calibrate_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            T.tasc_calibration_copy(dst, src, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    import zlib
    digest = zlib.crc32(b"".join(T.tasc_session_get_tokens(session, b).tobytes() for b in range(cfg.batch)))
    print(f"{cfg.name}: {steps} draft + verify steps of {cfg.batch} x {cfg.k + 1} rows, chains {args.chains}, graph {args.graph}, {dt / steps * 1e3:.3f} ms per step, "
          f"the host's share (enqueueing) {t_host / steps * 1e3:.3f} ms "
          f"(without --warm the first steps include one-off set-up of the kernels); crc32 of all sequences' tokens {digest:08x}", flush=True)


if __name__ == "__main__":
    main()
