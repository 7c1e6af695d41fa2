"""Seeded synthetic inputs for choreographed attention.

This package only draws random numbers and lays out selection lists.  It
holds none of the method's arithmetic (no RoPE, no softmax, no slot
allocation): both the CPU oracle and the GPU tests consume the plain arrays
it returns.
"""
from .generators import (  # noqa: F401
    POS_AUTO,
    Call,
    Event,
    Workload,
    round_to_bf16,
    make_workload,
    tiny_fp32,
    single_prefill,
    parallel_decode,
    multi_agent_rounds,
    long_context,
    decode_loop,
    prefix_cache_baseline_rounds,
    small_random,
)
