"""Tokenizer enrichment on a workload's corpus (tasc_tok_enrich): compression and token-entropy effect.

    python -m paper_2602_24174_amd.tok_enrich_report [--config cfg2] [--docs N] [--budget 100,1000] [--n-max 4]

For every budget M: the corpus length before and after M merges (the paper's output compression rate), the time per
merge, the first merges, and the token distribution's entropy before and after, plain and normalised by ln of the
vocabulary size (paper, "Enriching the Tokenizer": collapsing typical n-grams into tokens makes the token distribution
less peaked; Appendix, Renyi entropy of the augmented vocabulary as a predictor).
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
    ap.add_argument("--budget", default="100,1000")
    ap.add_argument("--n-max", type=int, default=0)
    args = ap.parse_args()
    import torch
    import workload as W
    import paper_2602_24174_amd as T
    cfg = W.get_config(args.config)
    if args.docs:
        cfg = cfg.scaled(n_docs=args.docs)
    n_max = args.n_max or cfg.n_max
    tok, off = W.make_corpus(cfg)
    d_tok = torch.from_numpy(tok).cuda()

    def token_entropy(tokens, offsets, vocab):
        ng = T.tasc_ngram_build(tokens, offsets, vocab, 2, 1)
        g = T.tasc_ngram_entropy(ng, 1, 800000)
        ng.close()
        return g

    g0 = token_entropy(d_tok, off, cfg.vocab)
    print(f"{cfg.name}: corpus {cfg.n_docs} outputs, {tok.shape[0]} tokens, vocab {cfg.vocab}, n_max {n_max}")
    print(f"  base tokenisation: token entropy {g0.shannon:.4f} nats (normalised {g0.shannon / math.log(cfg.vocab):.4f}), "
          f"Renyi-2 {g0.renyi2:.4f}, {g0.n_entries} tokens in use")
    for m in [int(x) for x in args.budget.split(",")]:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        merges, out, out_off, lens = T.tasc_tok_enrich(d_tok, off, cfg.vocab, n_max, m)
        dt = time.perf_counter() - t0
        g = token_entropy(out, out_off, cfg.vocab + m)
        by_n = {}
        for gram, _, _ in merges:
            by_n[len(gram)] = by_n.get(len(gram), 0) + 1
        print(f"  budget {m}: {len(merges)} merges in {dt:.2f} s ({dt / max(1, len(merges)) * 1e3:.1f} ms per merge); corpus {lens[0]} -> {lens[-1]} tokens "
              f"(x{lens[0] / max(1, lens[-1]):.3f} shorter); merged n-gram lengths {dict(sorted(by_n.items()))}")
        print(f"    token entropy {g.shannon:.4f} nats (normalised {g.shannon / math.log(cfg.vocab + m):.4f}), Renyi-2 {g.renyi2:.4f}, "
              f"{g.n_entries} tokens in use; first merges: " + ", ".join(f"{gram} x{f}" for gram, f, _ in merges[:3]))


if __name__ == "__main__":
    main()
