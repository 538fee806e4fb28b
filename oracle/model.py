"""CPU oracle for the target forward and the draft-then-verify loop.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; it shares no code with the HIP library.

The paper (section "Speculative Decoding") fixes the loop: a drafter proposes
gamma tokens, the target scores them in ONE forward pass, a prefix of k <= gamma
tokens is accepted; with beam size 1 (Results, TASC-spec subsection) this is
greedy decoding, whose output speculative decoding must reproduce token for
token.  The target itself is a black box in the paper; its architecture here
(pre-norm RMSNorm, RoPE with rotate-half pairing, grouped-query attention,
SwiGLU, untied LM head, sparse bigram bias on the logits) comes from the
workload configurations, so the architecture constants are "parity unpinned"
by the paper.  What IS pinned (tests/test_oracle_model.py): the sub-operations
against library routines, incremental-with-cache == full recompute, and
speculative == plain greedy for arbitrary drafters.

All floating point is float64 on the bf16- (or fp32-) rounded weights, so a
difference to the GPU measures the GPU's activation rounding only.
"""
import numpy as np


def _to_f64(w):
    """Weights arrive as float32 arrays or as uint16 arrays of bf16 bit patterns."""
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


def rmsnorm(x, g, eps):
    """x * g / sqrt(mean(x^2) + eps), row-wise."""
    return x * g / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing: dims (i, i + hd/2) of every head are rotated by the
    angle pos * theta^(-2i/hd).  x: [n, heads, hd], pos: [n]."""
    hd = x.shape[-1]
    half = hd // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(s):
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


class KVCache:
    """Contiguous per-layer cache of one sequence; `length` = number of valid positions."""

    def __init__(self, n_layers, n_kv_heads, head_dim, max_len):
        self.k = np.zeros((n_layers, max_len, n_kv_heads, head_dim))
        self.v = np.zeros((n_layers, max_len, n_kv_heads, head_dim))
        self.length = 0


class OracleModel:
    def __init__(self, cfg, weights, cache_weights=None):
        self.cfg = cfg
        self.w = weights
        n_params = cfg.n_layers * (2 * cfg.d_model * cfg.n_heads * cfg.head_dim
                                   + 2 * cfg.d_model * cfg.n_kv_heads * cfg.head_dim
                                   + 3 * cfg.d_model * cfg.d_ffn)
        self._cache_on = (n_params < 2.5e8) if cache_weights is None else cache_weights
        self._cache = {}
        self.lm_head = _to_f64(weights["lm_head"])
        self.bias = weights.get("bias")

    def _layer(self, l, name):
        if not self._cache_on:
            return _to_f64(self.w["layers"][l][name])
        key = (l, name)
        if key not in self._cache:
            self._cache[key] = _to_f64(self.w["layers"][l][name])
        return self._cache[key]

    def new_cache(self, max_len):
        c = self.cfg
        return KVCache(c.n_layers, c.n_kv_heads, c.head_dim, max_len)

    def hidden(self, tokens, cache):
        """Final-norm hidden states [n, d] of `tokens` placed at positions cache.length ...; K and V
        of these positions are appended to the cache (cache.length is NOT advanced: the caller commits)."""
        c = self.cfg
        tokens = np.asarray(tokens, dtype=np.int64)
        n = tokens.shape[0]
        p0 = cache.length
        pos = np.arange(p0, p0 + n)
        H, Hkv, hd = c.n_heads, c.n_kv_heads, c.head_dim
        x = _to_f64(self.w["embed"][tokens])
        for l in range(c.n_layers):
            h = rmsnorm(x, _to_f64(self.w["layers"][l]["g1"]), c.rms_eps)
            q = (h @ self._layer(l, "wq").T).reshape(n, H, hd)
            k = (h @ self._layer(l, "wk").T).reshape(n, Hkv, hd)
            v = (h @ self._layer(l, "wv").T).reshape(n, Hkv, hd)
            q = rope(q, pos, c.rope_theta)
            k = rope(k, pos, c.rope_theta)
            cache.k[l, p0:p0 + n] = k
            cache.v[l, p0:p0 + n] = v
            att = np.zeros((n, H, hd))
            for j in range(H):
                g = (j * Hkv) // H                      # query head j reads KV head floor(j * Hkv / H)
                kk = cache.k[l, :p0 + n, g]             # [p0+n, hd]
                vv = cache.v[l, :p0 + n, g]
                s = (q[:, j] @ kk.T) / np.sqrt(hd)      # [n, p0+n]
                mask = np.arange(p0 + n)[None, :] > pos[:, None]
                s = np.where(mask, -np.inf, s)
                att[:, j] = softmax(s) @ vv
            x = x + att.reshape(n, H * hd) @ self._layer(l, "wo").T
            h = rmsnorm(x, _to_f64(self.w["layers"][l]["g2"]), c.rms_eps)
            gate = h @ self._layer(l, "wg").T
            up = h @ self._layer(l, "wu").T
            x = x + ((gate / (1.0 + np.exp(-gate))) * up) @ self._layer(l, "wd").T
        return rmsnorm(x, _to_f64(self.w["gf"]), c.rms_eps)

    def logits_from_hidden(self, h, tokens):
        """h W_lm^T + bias(u, .), u = the input token of the row."""
        z = h @ self.lm_head.T
        if self.bias is not None:
            b = self.bias
            for i, u in enumerate(np.asarray(tokens, dtype=np.int64)):
                lo, hi = int(b["rowptr"][u]), int(b["rowptr"][u + 1])
                cols = b["col"][lo:hi]
                dense = z[i, cols].copy()
                z[i] += float(b["base"][u])
                z[i, cols] = dense + b["val"][lo:hi].astype(np.float64)
        return z

    def forward(self, tokens, cache, last_only=False):
        h = self.hidden(tokens, cache)
        if last_only:
            return self.logits_from_hidden(h[-1:], np.asarray(tokens)[-1:])
        return self.logits_from_hidden(h, tokens)


def argmax_lowest(z):
    """Row-wise argmax, lowest index among equal maxima (numpy's argmax returns the first)."""
    return np.argmax(z, axis=-1)


def accept_length(drafts, a):
    """Longest m with drafts[i] == a[i] for all i < m  (a[i] = target argmax after row i; row 0 is
    the pending token, row i >= 1 the i-th draft)."""
    m = 0
    while m < len(drafts) and int(drafts[m]) == int(a[m]):
        m += 1
    return m


def generate(model, prompt, gen_len, k, drafter, max_len=None, prefill_chunk=None, trace=None):
    """Greedy draft-then-verify decoding of one sequence.  k = 0 is plain greedy decoding.

    drafter(committed_tokens) -> k proposed tokens.  Emits exactly gen_len tokens.  `trace`, if a
    list, receives one dict per verify step (committed, drafts, argmax, accept, logits, margin)."""
    prompt = [int(t) for t in prompt]
    max_len = max_len or (len(prompt) + gen_len + k + 1)
    cache = model.new_cache(max_len)
    step = prefill_chunk or len(prompt)
    z = None
    for p0 in range(0, len(prompt), step):
        chunk = prompt[p0:p0 + step]
        z = model.forward(chunk, cache, last_only=True)
        cache.length += len(chunk)
    pending = int(argmax_lowest(z)[0])
    out = [pending]
    n_steps = 0
    while len(out) < gen_len:
        committed = prompt + out
        drafts = [int(t) for t in drafter(committed)] if k > 0 else []
        assert len(drafts) == k
        rows = [pending] + drafts
        z = model.forward(rows, cache)
        a = argmax_lowest(z)
        m = accept_length(drafts, a)
        emitted = drafts[:m] + [int(a[m])]
        if trace is not None:
            top2 = np.partition(z, -2, axis=-1)[:, -2:]
            trace.append({"committed": committed, "drafts": drafts, "argmax": a.copy(), "accept": m,
                          "logits": z, "margin": top2[:, 1] - top2[:, 0], "cached_len": cache.length})
        cache.length += 1 + m                            # rejected positions are dead, overwritten later
        pending = emitted[-1]
        out.extend(emitted)
        n_steps += 1
    return out[:gen_len], n_steps
