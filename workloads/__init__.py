"""Seeded synthetic inputs and workload shapes for the ST3 hot path.

This package holds data only: tensor shapes, token counts, seeds, and the
random-number recipe that turns a seed into Q/K/V tensors.  It contains none
of the method's arithmetic (no attention, no ranking, no retention schedule),
so both the CPU oracle and the HIP path may import it without sharing code
that decides a result.
"""
from .configs import WORKLOADS, Workload, get_workload  # noqa: F401
from .synth import (  # noqa: F401
    bf16_bits_to_f64,
    bf16_round_bits,
    decode_qkv,
    normal_block,
    prefill_qkv,
)
