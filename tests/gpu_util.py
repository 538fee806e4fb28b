"""Shared set-up for the GPU parity tests (inputs only; no arithmetic of the method)."""
import numpy as np

import workload as W


class Rig:
    """Corpus, weights, GPU model / tables / session of one configuration."""

    def __init__(self, cfg, max_rows=None, with_ngram=True, batch=None):
        import paper_2602_24174_amd as T
        self.T = T
        self.cfg = cfg
        self.batch = batch or cfg.batch
        self.corpus = W.make_corpus(cfg)
        self.weights = W.make_model(cfg, self.corpus)
        self.max_rows = max_rows or max(cfg.k + 1, 16)
        self.max_len = cfg.prompt_len + cfg.gen_len + 2 * self.max_rows
        self.model = T.tasc_model_create(cfg, self.weights, self.max_len)
        self.ng = T.tasc_ngram_build(self.corpus[0], self.corpus[1], cfg.vocab, cfg.n_max, cfg.p_min) if with_ngram else None
        self.session = T.tasc_session_create(self.model, self.batch, self.max_len, self.max_rows)
        self.prompts, self.prompt_off = W.make_prompts(cfg, batch=self.batch)

    def params(self, k=None, lambda_q16=None, p_min_ctx=None):
        c = self.cfg
        return self.T.spec_params(c.k if k is None else k, c.lambda_q16 if lambda_q16 is None else lambda_q16,
                                  c.p_min_ctx if p_min_ctx is None else p_min_ctx, 1)

    def generate(self, k=None, trace_steps=0, max_new=None, **kw):
        import torch
        c = self.cfg
        p = self.params(k, **kw)
        G = max_new or c.gen_len
        out = torch.zeros((self.batch, G), dtype=torch.int32, device="cuda")
        trace = None
        if trace_steps:
            trace = torch.full((trace_steps, self.batch, 2 * p.k + 3), -7, dtype=torch.int32, device="cuda")
        st = self.T.tasc_generate(self.model, self.ng if p.k > 0 else None, self.session, self.prompts, self.prompt_off, G, p,
                                  out, trace, trace_steps)
        return out.cpu().numpy(), st, (trace.cpu().numpy()[:st.steps] if trace is not None else None)


def split_trace(tr, k):
    """trace row -> (committed length, drafts[k], argmax[k+1], accept)."""
    return tr[..., 0], tr[..., 1:1 + k], tr[..., 1 + k:2 * k + 2], tr[..., 2 * k + 2]
