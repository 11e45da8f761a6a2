"""Seeded synthetic inputs for the sparse-attention hot path.

This package only draws random numbers and moves bytes (page scatter, table
permutation).  It holds none of the method's arithmetic, so that both the CPU
oracle's tests and the HIP path's tests can take their inputs from it without
sharing any code of the computation itself.
"""
from .generate import (  # noqa: F401
    Workload,
    DecodeInputs,
    PrefillInputs,
    CONFIGS,
    get_config,
    make_decode_inputs,
    make_prefill_inputs,
    scatter_prefill_kv_to_pages,
)
