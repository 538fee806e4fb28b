"""Per-phase timing report of the persistent small-batch step kernel (tasc_profile_phases).

    python -m paper_2602_24174_amd.phase_report [--config cfg2] [--grid G] [--layer-wgs N] [--layer-stride S]

Builds the named workload (--docs N shrinks the corpus, and with it the LM-head bias table), prefills, runs a few warm verify steps, then one verify step with the per-phase wall-clock stamps
on, and prints per layer-phase medians: the longest workgroup's work, the span from the first begin to the
last end, and the barrier gap to the next phase.
"""
import argparse
import os
import sys
import warnings

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pipeline_report(cfg, ts, n_wg):
    """Stamps of the spatial-pipeline kernel: per workgroup and phase (inputs complete, outputs stored); a workgroup
    only has stamps for the phases of its role."""
    warnings.simplefilter("ignore", RuntimeWarning)              # phase 0 (the embedding) has no stamps: all-NaN columns
    L = cfg.n_layers
    have = ts[:, :, 1] > 0
    ready = np.where(have, ts[:, :, 0], np.nan)
    done = np.where(have, ts[:, :, 1], np.nan)
    lay = slice(1, 1 + 5 * L)
    first_ready, last_ready = np.nanmin(ready, axis=0), np.nanmax(ready, axis=0)
    last_done = np.nanmax(done, axis=0)
    work = np.nanmax(done - ready, axis=0)                       # inputs complete -> outputs stored, slowest workgroup
    hop = last_ready[2:] - last_done[1:-1]                       # outputs stored -> the next phase's slowest workgroup has its inputs
    per = lambda v: np.round(np.nanmedian(np.asarray(v)[:5 * L].reshape(L, 5), axis=0), 2)
    t0 = np.nanmin(ready[:, 1])
    n_role = [int(have[:, 1 + r].sum()) for r in range(5)]
    print(f"{cfg.name}: grid {n_wg} workgroups; workgroups per role (qkv, attention, o-proj, gate/up, down) {n_role}; k = {cfg.k}, "
          f"cached length about {cfg.prompt_len + 6 * (cfg.k + 1)}")
    print(f"whole step {np.nanmax(done) - t0:.1f} us from the first layer's inputs; layers {last_done[5 * L] - t0:.1f} us "
          f"({(last_done[5 * L] - t0) / L:.2f} us per layer); LM head {last_done[-2] - first_ready[-2]:.1f} us "
          f"(inputs at the last workgroup {last_ready[-2] - last_done[5 * L]:.2f} us after the last layer); accept ends "
          f"{last_done[-1] - last_done[-2]:.1f} us after the last strip")
    print("per-layer medians over the layers (us)                         qkv    attn   o-proj  gate/up  down")
    print("  inputs complete -> outputs stored, slowest workgroup       ", per(work[lay]))
    print("  outputs stored -> inputs complete at the next phase        ", per(np.append(hop[:5 * L - 1], np.nan)))
    print("  spread of 'inputs complete' over the phase's workgroups    ", per((last_ready - first_ready)[lay]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--layer-wgs", type=int, default=0)
    ap.add_argument("--layer-stride", type=int, default=0)
    ap.add_argument("--max-rows", type=int, default=16)
    ap.add_argument("--workers", type=int, default=0, help="computing members of the layer group in XCD-local mode (0 = half)")
    ap.add_argument("--docs", type=int, default=0, help="corpus size (0 = the configuration's; it sets the size of the LM-head bias table)")
    ap.add_argument("--agent-barriers", action="store_true", help="agent-scope barriers only (no XCD-local mode)")
    ap.add_argument("--barrier-kernel", action="store_true", help="the barrier kernel instead of the spatial pipeline")
    ap.add_argument("--share", type=int, default=1, help="tiles per workgroup and layer of the pipeline kernel (1..3)")
    ap.add_argument("--dump", default="", help="also save the raw stamps [workgroup][phase][2] (microseconds) as a .npy file")
    args = ap.parse_args()
    import torch
    import workload as W
    import paper_2602_24174_amd as T

    cfg = W.get_config(args.config)
    if args.docs:
        cfg = cfg.scaled(n_docs=args.docs)
    if cfg.batch * args.max_rows > 16:
        sys.exit("the persistent kernel only serves sessions with batch * max_rows <= 16")
    corpus = W.make_corpus(cfg)
    weights = W.make_model(cfg, corpus)
    prompts, poff = W.make_prompts(cfg)
    max_len = cfg.prompt_len + cfg.gen_len + 2 * args.max_rows
    model = T.tasc_model_create(cfg, weights, max_len)
    ng = T.tasc_ngram_build(corpus[0], corpus[1], cfg.vocab, cfg.n_max, cfg.p_min)
    sess = T.tasc_session_create(model, cfg.batch, max_len, args.max_rows)
    T.tasc_config_set(T.TASC_CFG_SMALL_KERNEL, 0 if args.barrier_kernel else 1)
    T.tasc_config_set(T.TASC_CFG_PIPE_SHARE, args.share)
    T.tasc_config_set(T.TASC_CFG_SMALL_XCD_LOCAL, 0 if args.agent_barriers else 1)
    T.tasc_config_set(T.TASC_CFG_SMALL_LAYER_WORKERS, args.workers)
    T.tasc_config_set(T.TASC_CFG_SMALL_GRID, args.grid)
    T.tasc_config_set(T.TASC_CFG_SMALL_LAYER_WGS, args.layer_wgs)
    T.tasc_config_set(T.TASC_CFG_SMALL_LAYER_STRIDE, args.layer_stride)
    T.tasc_session_prefill(model, sess, prompts, poff, cfg.gen_len)
    params = T.spec_params(cfg.k, cfg.lambda_q16, cfg.p_min_ctx, 1)
    drafts = torch.zeros((cfg.batch, cfg.k), dtype=torch.int32, device="cuda")
    n_ph = 3 + 5 * cfg.n_layers
    n_wg = args.grid or torch.cuda.get_device_properties(0).multi_processor_count
    buf = torch.zeros(n_wg * n_ph * 2, dtype=torch.int64, device="cuda")
    for _ in range(5):
        T.tasc_draft(ng, sess, params, drafts)
        T.tasc_verify_step(model, sess, drafts, cfg.k)
    T.tasc_profile_phases(buf)
    T.tasc_draft(ng, sess, params, drafts)
    T.tasc_verify_step(model, sess, drafts, cfg.k)
    torch.cuda.synchronize()
    T.tasc_profile_phases(None)

    ts = buf.cpu().numpy().reshape(n_wg, n_ph, 2).astype(np.float64) / 100.0      # microseconds (100 MHz clock)
    if args.dump:
        np.save(args.dump, ts)
    if not args.barrier_kernel:
        return pipeline_report(cfg, ts, n_wg)
    one_xcd = not args.agent_barriers and n_wg >= 256            # the library's defaults
    stride = args.layer_stride or (8 if one_xcd else 1)
    lg = args.layer_wgs or (32 if one_xcd and not args.layer_stride else 48)
    members = [w for w in range(n_wg) if w % stride == 0 and w // stride < lg]
    n_work = (args.workers or lg) if one_xcd else lg
    pre = ts[members[n_work:]][:, :1 + 5 * cfg.n_layers]
    lay = ts[members[:n_work]][:, :1 + 5 * cfg.n_layers]
    begin, end = lay[:, :, 0], lay[:, :, 1]
    work = (end - begin).max(axis=0)
    span = end.max(axis=0) - begin.min(axis=0)
    gap = np.append(begin.min(axis=0)[1:] - end.max(axis=0)[:-1], 0.0)
    per = lambda v: np.round(np.median(v[1:].reshape(cfg.n_layers, 5), axis=0), 2)
    t0 = begin.min()
    print(f"{cfg.name}: grid {n_wg} workgroups, layer group {len(members)} (stride {stride}), {n_work} of them computing; k = {cfg.k}, cached length "
          f"about {cfg.prompt_len + 6 * (cfg.k + 1)}")
    print(f"whole step {ts[:, :, 1].max() - t0:.1f} us; embedding + layers {end.max() - t0:.1f} us; "
          f"LM head {ts[:, -2, 1].max() - ts[:, -2, 0].min():.1f} us; accept {ts[0, -1, 1] - ts[0, -1, 0]:.1f} us")
    print("per-layer medians over the layers (us)        qkv    attn   o-proj  gate/up  down")
    print("  longest workgroup's work                 ", per(work))
    print("  first begin .. last end                  ", per(span))
    print("  barrier: last end -> next phase's begin  ", per(gap))
    if len(pre):
        print(f"  prefetchers ({len(pre)}): longest fetch-ahead      ", per((pre[:, :, 1] - pre[:, :, 0]).max(axis=0)))


if __name__ == "__main__":
    main()
