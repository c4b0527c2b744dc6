"""Seeded synthetic inputs for the sparsified-FFN step; shared by tests, smoke and bench.
Holds no arithmetic of the method itself (no pruning, packing, activation or GEMM)."""
from .synth import (bf16_bits_from_f32, make_ffn_inputs, make_moe_segments, make_moe_inputs, make_router_inputs, make_ffn_sweep, CONFIGS,
                    Z_FOR_ZERO_FRACTION)
