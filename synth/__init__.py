"""Seeded synthetic inputs for the frequency-ranked draft LM head.

This package only *produces bytes*: bf16 weight / hidden-state arrays and a
frequency-ranked id list with the long-tail shape the paper measures on its
corpus (Section 3.2, "Corpus-Level Token Statistics").  It holds none of the
method's arithmetic (no gather, no logits, no softmax, no top-k) so that the
CPU oracle and the HIP library can both be fed from it without sharing code.
"""

from .gen import (  # noqa: F401
    BASE_SEED,
    CONFIGS,
    DraftHeadConfig,
    SWEEP_V_SUB,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_exact_case,
    make_hidden,
    make_weights,
    zipf_ranking,
)
