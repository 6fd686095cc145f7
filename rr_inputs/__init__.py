"""Seeded synthetic long-context attention inputs.

This package only draws random tensors with a documented structure.  It holds
none of the method's arithmetic (no sampling rule, no scores, no softmax, no
selection) so that both the CPU oracle's tests and the GPU harness can take
their inputs from it without sharing any code of the method itself.
"""
from .workloads import (  # noqa: F401
    Workload,
    CONFIGS,
    get_config,
    custom,
    generate,
    bf16_round,
    bf16_bits,
    bf16_from_bits,
)
