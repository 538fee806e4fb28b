"""Acceptance sweeps on the GPU against the oracle: at every sweep point of a config-1-sized workload the accept-length
histogram, the step count and the emitted tokens that tasc_generate reports equal the oracle's draft-then-verify run,
and the per-position rates derived from them agree."""
import numpy as np
import pytest

import workload as W
from oracle import acceptance as OA
from oracle import model as OM
from oracle import ngram as ON

pytestmark = pytest.mark.gpu

POINTS = [  # (k, lambda, p_min, alpha)
    (4, 0.75, 5, 8.0),      # the configuration's defaults
    (1, 0.75, 5, 8.0),
    (8, 0.75, 5, 8.0),
    (15, 0.75, 5, 8.0),     # the longest draft the library takes
    (4, 0.0, 5, 8.0),       # context statistics alone
    (4, 1.0, 5, 8.0),       # corpus tables alone
    (4, 0.25, 1, 8.0),      # unpruned tables
    (4, 0.75, 50, 8.0),     # heavy pruning
    (4, 0.75, 5, 1.0),      # a target the corpus predicts less well
    (4, 0.75, 5, 0.0),      # a target that ignores the corpus (no bias table at all)
]


def test_sweep_points_match_oracle():
    import torch
    import paper_2602_24174_amd as T
    from paper_2602_24174_amd.acceptance_sweeps import SweepRig, position_rates
    cfg = W.get_config("cfg1").scaled(gen_len=48)
    rig = SweepRig(cfg)
    tables = {}
    alpha_now = cfg.bias_alpha
    om = OM.OracleModel(cfg, rig.weights)
    for (k, lam, p_min, alpha) in POINTS:
        print(f"sweep point k={k} lambda={lam} p_min={p_min} alpha={alpha}", flush=True)
        if alpha != alpha_now:
            rig.set_bias(alpha)
            om = OM.OracleModel(cfg, rig.weights)
            alpha_now = alpha
        if p_min not in tables:
            tables[p_min] = ON.build_tables_flat(rig.corpus[0], rig.corpus[1], cfg.vocab, cfg.n_max, p_min)
        q16 = int(round(lam * 65536))
        otrace = []
        want, o_steps = OM.generate(om, rig.prompts, cfg.gen_len, k,
                                    lambda c: ON.draft(tables[p_min], c, k, q16, cfg.p_min_ctx), trace=otrace,
                                    prefill_chunk=rig.max_rows, max_len=rig.max_len)
        lens = [o["accept"] for o in otrace]
        r = rig.run(k=k, lam=lam, p_min=p_min)
        assert rig.out.cpu().numpy()[0].tolist() == want
        assert r["equals_greedy"]
        assert r["steps"] == o_steps
        assert r["hist"] == OA.histogram(lens, k)
        assert np.allclose(r["rate"], [float(x) for x in OA.acceptance_by_position(lens, k)], atol=1e-12)
        assert abs(r["mean_accept"] - float(OA.mean_accept(lens))) < 1e-12
