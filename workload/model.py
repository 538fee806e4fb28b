"""Random-init decoder-only target models (stand-ins for the fine-tuned targets).

The paper treats the target as a black box; its architecture here is the
pre-norm RMSNorm / RoPE / GQA / SwiGLU decoder the workload configurations
name.  All matrices are i.i.d. N(0, 0.02^2), all norm gains are 1, the LM head
is its own draw (untied).  A sparse additive LM-head bias
alpha * log P_bigram(v | u), add-one smoothed and taken from the corpus, makes
the target behave like the task distribution so that drafts get accepted.

Canonical tensor layout (what both the oracle and the library's model_create
receive): every linear weight is [out_features, in_features], row-major.
For bf16 configurations the tensors are uint16 arrays holding bf16 bit patterns.
"""
import numpy as np

from .configs import WorkloadConfig

_TENSOR_ID = {"embed": 1, "lm_head": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6, "wg": 7, "wu": 8, "wd": 9}


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(cfg, tensor, layer, shape):
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 8) | 0x40 | _TENSOR_ID[tensor], layer]))
    w = g.standard_normal(size=shape, dtype=np.float32)
    w *= np.float32(0.02)
    return to_bf16_bits(w) if cfg.dtype == "bf16" else w


def make_layer(cfg: WorkloadConfig, layer: int) -> dict:
    d, H, Hkv, hd, F = cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn
    return {
        "wq": _normal(cfg, "wq", layer, (H * hd, d)),
        "wk": _normal(cfg, "wk", layer, (Hkv * hd, d)),
        "wv": _normal(cfg, "wv", layer, (Hkv * hd, d)),
        "wo": _normal(cfg, "wo", layer, (d, H * hd)),
        "wg": _normal(cfg, "wg", layer, (F, d)),
        "wu": _normal(cfg, "wu", layer, (F, d)),
        "wd": _normal(cfg, "wd", layer, (d, F)),
        "g1": np.ones(d, dtype=np.float32),
        "g2": np.ones(d, dtype=np.float32),
    }


def make_model(cfg: WorkloadConfig, corpus=None, layers: bool = True) -> dict:
    """Returns {"embed", "lm_head", "gf", "layers": [..], "bias": csr dict or None}."""
    m = {
        "embed": _normal(cfg, "embed", 0, (cfg.vocab, cfg.d_model)),
        "lm_head": _normal(cfg, "lm_head", 0, (cfg.vocab, cfg.d_model)),
        "gf": np.ones(cfg.d_model, dtype=np.float32),
        "layers": [make_layer(cfg, l) for l in range(cfg.n_layers)] if layers else [],
        "bias": None,
    }
    if corpus is not None:
        m["bias"] = bigram_bias_csr(corpus[0], corpus[1], cfg.vocab, cfg.bias_alpha)
    return m


def bigram_bias_csr(tokens: np.ndarray, doc_off: np.ndarray, vocab: int, alpha: float) -> dict:
    """LM-head bias table: bias(u, v) = alpha * (ln(c2(u,v) + 1) - ln(c1(u) + V)).

    c2 = raw count of the adjacent pair (u, v) inside one document, c1(u) = sum_v c2(u, v).
    Stored as CSR over the seen pairs (value = the full bias of that pair) plus
    `base[u]` = the bias of every unseen pair of row u.  Computed in float64, stored fp32.
    """
    T = tokens.shape[0]
    a = tokens[:-1].astype(np.int64)
    b = tokens[1:].astype(np.int64)
    keep = np.ones(max(T - 1, 0), dtype=bool)
    ends = doc_off[1:-1] - 1                    # last token of every document but the final one
    ends = ends[(ends >= 0) & (ends < T - 1)]
    keep[ends] = False                          # the pair (last of doc i, first of doc i+1) is not a bigram
    # documents of length 0 make ends repeat or point at another document's last token: still correct,
    # because the boundary sits between ends and ends+1 either way.
    key = a[keep] * vocab + b[keep]
    uk, cnt = np.unique(key, return_counts=True)
    row = uk // vocab
    col = (uk % vocab).astype(np.int32)
    c1 = np.bincount(row, weights=cnt.astype(np.float64), minlength=vocab)
    rowptr = np.zeros(vocab + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=vocab), out=rowptr[1:])
    lognorm = np.log(c1 + float(vocab))
    val = alpha * (np.log(cnt.astype(np.float64) + 1.0) - lognorm[row])
    base = -alpha * lognorm
    return {"rowptr": rowptr, "col": col, "val": val.astype(np.float32), "base": base.astype(np.float32)}

