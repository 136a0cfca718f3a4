"""Seeded synthetic inputs for KCache decode attention.

This package only manufactures data: query vectors, K and V caches and
sequence lengths with LLaMA-class shapes.  It holds none of the method's
arithmetic (no scores, softmax, selection or weighted sum) and is the one
module that both the CPU oracle's tests and the GPU path's tests may import.

Every value is a pure function of (seed, tensor, layer, sequence, head,
position, channel): a counter-based integer hash picks one of 65 536 standard
normal quantiles from a table computed once on the host.  The same torch
integer ops run on the CPU and on the GPU, so the big configurations can be
generated directly in HBM while the oracle regenerates any single unit on the
host with identical bits.
"""
from .gen import (CONFIGS, Workload, config, normal_table, gen_q, gen_kv_units, gen_layer,
                  gen_unit, pivot_positions, torch_dtype, as_bits)

__all__ = ["CONFIGS", "Workload", "config", "normal_table", "gen_q", "gen_kv_units", "gen_layer",
           "gen_unit", "pivot_positions", "torch_dtype", "as_bits"]
