"""Seeded synthetic workloads shared by the tests, the CPU oracle and the GPU path.

This package holds shapes and random input buffers only.  It contains none of
the method's arithmetic (no layer math, no graph construction, no memory
planning): both sides receive the very same host buffers from here.
"""
from .synth import (  # noqa: F401
    LlamaConfig,
    CONFIGS,
    config,
    normal,
    to_bf16_bits,
    bf16_bits_to_f32,
    make_llama_inputs,
    make_lora_inputs,
    random_dag,
)
