"""The five synthetic workload configurations (stand-ins for the paper's task
corpora and fine-tuned target models, which are not available).

Method hyper-parameters the paper fixes (Results, TASC-spec subsection):
p_min = 5 and lambda = 0.75, greedy (beam size 1).  Draft length k, n_max,
model shapes, batch, prompt and generation lengths are this build's choices.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    dtype: str            # "f32" or "bf16": storage type of weights and KV cache
    # model
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    bias_alpha: float     # logits += alpha * log P_bigram(. | input token)
    rope_theta: float
    rms_eps: float
    # corpus
    n_docs: int
    doc_len_lo: int
    doc_len_hi: int
    pool_size: int        # number of phrases in the pool
    phrase_len_lo: int
    phrase_len_hi: int
    zipf_s: float
    noise: float
    # drafting and decode
    n_max: int
    k: int
    batch: int
    prompt_len: int
    gen_len: int
    kv_block: int         # tokens per KV page
    p_min: int = 5
    p_min_ctx: int = 1
    lam: float = 0.75
    seed: int = 0

    @property
    def lambda_q16(self) -> int:
        return int(round(self.lam * 65536))

    @property
    def max_len(self) -> int:
        """Largest number of cached positions a sequence can reach."""
        return self.prompt_len + self.gen_len + self.k + 1

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


def _cfg(name, dtype, L, d, H, Hkv, hd, F, V, docs, lo, hi, pool, noise, n_max, k, B, P, G):
    return WorkloadConfig(
        name=name, dtype=dtype, n_layers=L, d_model=d, n_heads=H, n_kv_heads=Hkv, head_dim=hd,
        d_ffn=F, vocab=V, bias_alpha=8.0, rope_theta=10000.0, rms_eps=1e-6,
        n_docs=docs, doc_len_lo=lo, doc_len_hi=hi, pool_size=pool, phrase_len_lo=2, phrase_len_hi=8,
        zipf_s=1.1, noise=noise, n_max=n_max, k=k, batch=B, prompt_len=P, gen_len=G, kv_block=16)


CONFIGS = {
    # tiny fp32 model the CPU oracle runs end to end in seconds
    "cfg1": _cfg("cfg1", "f32", 2, 128, 4, 4, 32, 512, 512, 2_000, 32, 96, 200, 0.10, 3, 4, 1, 64, 64),
    # 135M-class bf16, batch 1: weight-streaming verify step
    "cfg2": _cfg("cfg2", "bf16", 30, 576, 9, 3, 64, 1536, 49_152, 50_000, 64, 256, 5_000, 0.10, 4, 8, 1, 512, 256),
    # 0.5B-class bf16, batch 32
    "cfg3": _cfg("cfg3", "bf16", 24, 896, 14, 2, 64, 4864, 151_936, 200_000, 64, 256, 5_000, 0.10, 4, 6, 32, 1024, 256),
    # 1.5B-class bf16, batch 64
    "cfg4": _cfg("cfg4", "bf16", 28, 1536, 12, 2, 128, 8960, 151_936, 500_000, 64, 256, 5_000, 0.10, 5, 8, 64, 2048, 256),
    # 3B-class bf16, batch 256
    "cfg5": _cfg("cfg5", "bf16", 36, 2048, 16, 2, 128, 11008, 151_936, 1_000_000, 64, 256, 20_000, 0.05, 5, 4, 256, 512, 128),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]
