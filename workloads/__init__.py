"""Seeded synthetic inputs for the AudioKV eviction path.

This package only draws random tensors of the shapes and statistics of an
audio-language-model prefill (AR(1) keys, spike tokens, text spans, Dirichlet
head weights). It contains none of the method's arithmetic and is the one
module that both the CPU oracle's tests and the HIP path's tests may import.
"""

from .gen import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f64,
    f64_to_bf16_bits,
    gen_item,
    gen_lengths,
    gen_weights,
    get_config,
)
