"""Seeded synthetic inputs: task corpora, prompts and random-init target models.

This package only *generates data*.  It holds none of the method's arithmetic
(no n-gram table, no drafting, no transformer math): the CPU oracle and the HIP
library both receive what is generated here as plain arrays.  Every draw comes
from a Philox counter-based generator keyed by (seed, purpose, index), so any
tensor or corpus can be regenerated on its own.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .corpus import make_corpus, make_prompts  # noqa: F401
from .model import make_model, bigram_bias_csr, to_bf16_bits, bf16_bits_to_f32  # noqa: F401
