"""Seeded synthetic inputs for the batched heterogeneous-rank LoRA apply.

This module only *draws inputs* (token activations, adapter weights, request
lengths, adapter popularity) and converts number formats.  It holds none of the
method's arithmetic: no shrink, no expand, no indexing.  Both the CPU oracle's
tests and the GPU tests take their inputs from here so that both sides see the
same bits.

The instances stand in for the serving workloads of the paper's evaluation
(section 5.1: five adapter ranks 8..128, N_a adapters, power-law adapter
popularity, production-trace prompt lengths), none of which ship with the
paper's text.
"""
from .gen import (  # noqa: F401
    Instance,
    Projection,
    bf16_round,
    bf16_bits,
    bf16_from_bits,
    make_instance,
    tiny,
    decode,
    decode_heavy,
    decode_paper,
    decode_qkv,
    prefill,
    mixed,
    stress,
    small_mixed,
    CONFIGS,
)
