"""Seeded synthetic router inputs shared by the tests, the benchmark and the CPU checker.

Holds random-number recipes only: none of the routing method's arithmetic lives here.
"""
from .synth import (CONFIGS, RouterInputs, bf16_round, bf16_bits, bf16_from_bits,
                    make_inputs, make_logits, capacity)

__all__ = ["CONFIGS", "RouterInputs", "bf16_round", "bf16_bits", "bf16_from_bits",
           "make_inputs", "make_logits", "capacity"]
