"""What the bf16 storage of activations between the GEMMs costs on the logits, measured on the CPU with no GPU code.

The oracle keeps every activation in float64.  A path that feeds bf16 operands to its matrix products ("bf16 in, fp32
accumulate") must round, at the least, the normalised activations, q / k / v, the attention output, the SwiGLU output
and the final normalised row.  This test runs the float64 forward twice over the same weights, once exact and once
with exactly those roundings (and a third time with the softmax weights rounded as well, which an MFMA attention adds),
at the depth and width of the 1.5B-class and 3B-class workload models, and records the logit error that rounding
alone produces.  It is the yardstick for the logit tolerance of the GPU parity tests of those two configurations: an
error of the GPU path at this level is inherent in the storage type, anything well above it is the kernels' own.

The forward below is written for this measurement only (whole prompt in one chunk, weights drawn layer by layer so
that the 3B-class model never sits in memory; activations float64, each matrix product taken in float32 on the exact
bf16 weight values, whose own rounding, 2^-24, is 2^-15 of the one under study); it is pinned to the oracle's float64
forward on a small model first."""
import numpy as np
import pytest

import workload as W
from oracle import model as OM
from workload.model import to_bf16_bits, bf16_bits_to_f32


def _bf16(x):
    """float64 -> nearest bf16 (ties to even), back in float64."""
    return bf16_bits_to_f32(to_bf16_bits(x.astype(np.float32))).astype(np.float64)


def _mm(a, w):
    """a [n, K] float64 times w [N, K]^T float32, product in float32, result float64."""
    return (a.astype(np.float32) @ w.T).astype(np.float64)


def _forward(cfg, tokens, layer_fn, embed, lm_head, rnd, rnd_p):
    """Logits [n, V] of `tokens` at positions 0..n-1.  rnd(x) is applied to every matrix-product / attention input,
    rnd_p to the softmax weights; the identity gives the oracle's arithmetic."""
    n, H, Hkv, hd = len(tokens), cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    pos = np.arange(n)
    e0 = embed[np.asarray(tokens)]
    xs = [(OM._to_f64(e0) if e0.dtype == np.uint16 else e0.astype(np.float64)) for _ in rnd]
    mask = pos[None, :] > pos[:, None]
    for l in range(cfg.n_layers):
        w = {k: (bf16_bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in layer_fn(l).items()}
        for i, (r, rp) in enumerate(zip(rnd, rnd_p)):
            x = xs[i]
            h = r(OM.rmsnorm(x, w["g1"], cfg.rms_eps))
            q = r(OM.rope(_mm(h, w["wq"]).reshape(n, H, hd), pos, cfg.rope_theta))
            k = r(OM.rope(_mm(h, w["wk"]).reshape(n, Hkv, hd), pos, cfg.rope_theta))
            v = r(_mm(h, w["wv"]).reshape(n, Hkv, hd))
            att = np.zeros((n, H, hd))
            for j in range(H):
                g = (j * Hkv) // H
                s = np.where(mask, -np.inf, (q[:, j] @ k[:, g].T) / np.sqrt(hd))
                e = np.exp(s - s.max(axis=-1, keepdims=True))
                p = rp(e)                                   # an MFMA attention rounds the unnormalised weights ...
                att[:, j] = (p @ v[:, g]) / p.sum(axis=-1, keepdims=True)      # ... and normalises with their sum
            x = x + _mm(r(att.reshape(n, H * hd)), w["wo"])
            h = r(OM.rmsnorm(x, w["g2"], cfg.rms_eps))
            gate, up = _mm(h, w["wg"]), _mm(h, w["wu"])
            x = x + _mm(r((gate / (1.0 + np.exp(-gate))) * up), w["wd"])
            xs[i] = x
    lm = bf16_bits_to_f32(lm_head) if lm_head.dtype == np.uint16 else lm_head
    return [_mm(r(OM.rmsnorm(x, np.ones(cfg.d_model), cfg.rms_eps)), lm) for x, r in zip(xs, rnd)]


IDENT = lambda x: x  # noqa: E731


class _Weights:
    """i.i.d. N(0, 0.02^2) matrices with bf16 values held as float32, drawn into buffers that are reused from layer to
    layer (the statistics of the workload models; not their bit patterns, which this measurement does not need)."""

    THREADS = 8

    def __init__(self, cfg, seed):
        from concurrent.futures import ThreadPoolExecutor
        self.cfg = cfg
        self.rngs = [np.random.Generator(np.random.SFC64([seed, t])) for t in range(self.THREADS)]
        self.pool = ThreadPoolExecutor(self.THREADS)
        self.buf = {}

    def _fill(self, job):
        t, part = job                                   # every thread owns one generator and one slice of the matrix
        self.rngs[t].standard_normal(out=part, dtype=np.float32)
        part *= np.float32(0.02)
        b = part.view(np.uint32)
        b += np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))      # round to nearest even at bit 16
        b &= np.uint32(0xFFFF0000)

    def matrix(self, name, shape):
        w = self.buf.get((name, shape))
        if w is None:
            w = self.buf[(name, shape)] = np.empty(shape, dtype=np.float32)
        flat = w.reshape(-1)
        cuts = np.linspace(0, flat.size, self.THREADS + 1).astype(np.int64)
        list(self.pool.map(self._fill, [(t, flat[cuts[t]:cuts[t + 1]]) for t in range(self.THREADS)]))
        return w

    def layer(self, l):
        c = self.cfg
        d, H, Hkv, hd, F = c.d_model, c.n_heads, c.n_kv_heads, c.head_dim, c.d_ffn
        out = {n: self.matrix(n, s) for n, s in (("wq", (H * hd, d)), ("wk", (Hkv * hd, d)), ("wv", (Hkv * hd, d)),
                                                 ("wo", (d, H * hd)), ("wg", (F, d)), ("wu", (F, d)), ("wd", (d, F)))}
        out["g1"] = out["g2"] = np.ones(d)
        return out


def test_measurement_forward_equals_oracle_forward():
    cfg = W.get_config("cfg1").scaled(dtype="bf16", n_layers=3, d_model=64, n_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96,
                                      vocab=300)
    weights = W.make_model(cfg)
    toks = [5, 17, 299, 0, 42, 17, 8]
    om = OM.OracleModel(cfg, weights)
    want = om.forward(toks, om.new_cache(16))
    got = _forward(cfg, toks, lambda l: weights["layers"][l], weights["embed"], weights["lm_head"], [IDENT], [IDENT])[0]
    assert np.abs(got - want).max() < 2e-6          # float32 products against float64 ones


CONTEXT = 48          # prompt length of the GPU parity tests of the two deep models (tests/test_gpu_full.py)


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_logit_error_of_bf16_inputs_alone(name):
    """The rows of one verify step (k + 1 of them) after a 48-token context, as the GPU tests of these models score
    them; the error is taken over those rows (it grows with the context: with 5 rows and no context the 3B-class
    figures are rms 1.6e-2 / maximum 0.09, with the context 2.2e-2 / 0.12)."""
    cfg = W.get_config(name)
    rows = cfg.k + 1
    rng = np.random.default_rng(11)
    toks = rng.integers(0, cfg.vocab, CONTEXT + rows).tolist()
    gen = _Weights(cfg, 5)
    embed = gen.matrix("embed", (cfg.vocab, cfg.d_model)).copy()
    lm_head = gen.matrix("lm_head", (cfg.vocab, cfg.d_model))
    exact, inputs, inputs_p = _forward(cfg, toks, gen.layer, embed, lm_head, [IDENT, _bf16, _bf16], [IDENT, IDENT, _bf16])
    out = {}
    exact = exact[-rows:]
    for label, z in (("inputs", inputs), ("inputs + softmax weights", inputs_p)):
        d = np.abs(z[-rows:] - exact)
        out[label] = (float(d.max()), float(np.sqrt((d ** 2).mean())), float((d > 5e-2).mean()))
        print(f"{name} ({cfg.n_layers} layers, d {cfg.d_model}, {rows} rows x {cfg.vocab} logits), bf16 {label}: "
              f"max |delta| {out[label][0]:.4f}, rms {out[label][1]:.4f}, share beyond 5e-2 {out[label][2]:.2e}; "
              f"logit std {exact.std():.3f}", flush=True)
    worst, rms, share = out["inputs + softmax weights"]
    # The finding this test records (the draws are seeded, so the figures repeat).  0.5B-class model: the rounding stays
    # well inside the 5e-2 logit tolerance.  1.5B- and 3B-class models: rounding the inputs alone passes it, which is why
    # the GPU parity tests of those two hold the path to bounds derived from here, about 1.4 times these figures
    # (tests/test_gpu_full.py: DEEP_BOUNDS).
    if name == "cfg3":
        assert worst < 4e-2 and rms < 8e-3
    if name == "cfg4":
        assert 5e-2 < worst < 1e-1 and 1e-2 < rms < 1.7e-2 and share < 1e-3
    if name == "cfg5":
        assert 5e-2 < worst < 1.6e-1 and 1.7e-2 < rms < 2.7e-2 and share < 3.5e-2
