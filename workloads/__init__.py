"""Seeded synthetic inputs for the target-side verification step.

This package only *draws inputs* (hidden states, LM-head weights, draft logits,
drafted ids, vocabulary maps, n-gram caches, temperatures, Philox keys).  It
holds none of the verification arithmetic and is the one module that both the
CPU oracle's tests and the HIP path's tests/bench consume.
"""
from .synth import (  # noqa: F401
    VerifyCase,
    CaseSpec,
    make_case,
    baseline_spec,
    baseline_case,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
)
