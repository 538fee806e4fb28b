"""Typical-set statistics of a workload's corpus tables (tasc_ngram_entropy), per n-gram order.

    python -m paper_2602_24174_amd.table_report [--config cfg2] [--docs N] [--p-min 1] [--coverage 0.8]

Prints, for the token distribution (order 1) and every order up to n_max: distinct entries, Shannon and Renyi-2
entropy (nats), exp(H) (the paper's estimate of the typical-set size) and the number of n-grams that reach the given
share of the mass (paper, "Task-Induced n-Grams Concentration").  p_min = 1 keeps the corpus' full distribution.
"""
import argparse
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--docs", type=int, default=0)
    ap.add_argument("--p-min", type=int, default=1)
    ap.add_argument("--coverage", type=float, default=0.8)
    args = ap.parse_args()
    import torch
    import workload as W
    import paper_2602_24174_amd as T
    cfg = W.get_config(args.config)
    if args.docs:
        cfg = cfg.scaled(n_docs=args.docs)
    tok, off = W.make_corpus(cfg)
    d_tok = torch.from_numpy(tok).cuda()
    ng = T.tasc_ngram_build(d_tok, off, cfg.vocab, cfg.n_max, args.p_min)
    ppm = int(round(args.coverage * 1e6))
    print(f"{cfg.name}: corpus {cfg.n_docs} outputs, {tok.shape[0]} tokens, vocab {cfg.vocab}, p_min {args.p_min}")
    print(f"{'order':>5s} {'entries':>12s} {'windows':>12s} {'H nats':>9s} {'H2 nats':>9s} {'exp(H)':>12s} {'cover ' + str(args.coverage):>12s} {'share':>7s} {'ms':>7s}")
    for n in range(1, cfg.n_max + 1):
        T.tasc_ngram_entropy(ng, n, ppm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g = T.tasc_ngram_entropy(ng, n, ppm)
        ms = (time.perf_counter() - t0) * 1e3
        share = g.n_cover / g.n_entries if g.n_entries else 0.0
        print(f"{n:5d} {g.n_entries:12d} {g.total:12d} {g.shannon:9.4f} {g.renyi2:9.4f} {math.exp(g.shannon):12.0f} {g.n_cover:12d} {share:7.3f} {ms:7.2f}")


if __name__ == "__main__":
    main()
