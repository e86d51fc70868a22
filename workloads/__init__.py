"""Seeded synthetic inputs for sliced, asymmetric-unit causal attention.

This module draws sample lengths and q/k/v/dO values and names, as plain data,
which grouping policy each workload uses for its forward and backward unit
lists.  It holds none of the method's arithmetic: no attention, no slice or
unit construction, no cost model.  Both the CPU oracle's tests and the HIP
path's tests/benchmarks draw their inputs here so that both see identical
host arrays.

Length mixes follow the shape the paper reports for its corpora (most samples
short, a sub-percent tail carrying about half of the work; "Skewed Data
Distributions" in the Background section); the corpora themselves are not
reproduced.
"""
from .mixes import (WORKLOADS, Workload, draw_lengths, draw_values, to_bf16_bits,
                    bf16_bits_to_f32, bf16_round, SEEDS)

__all__ = ["WORKLOADS", "Workload", "draw_lengths", "draw_values", "to_bf16_bits",
           "bf16_bits_to_f32", "bf16_round", "SEEDS"]
