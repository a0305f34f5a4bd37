"""Seeded synthetic ARMT workloads (shapes, weights, embeddings).

This module serves both the CPU oracle's tests and the HIP path's tests / bench.
It holds NO arithmetic of the method itself: only shape bookkeeping, a seeded
normal generator and fp32 -> bf16 rounding of the generated values.

Workload shapes follow the LLaMA-3-family models the paper evaluates (Section 4,
Table 1 and the appendix tables) and the ARMT settings it states for the 1B model
(segment 1024, 16 memory tokens, associative hidden size 64; Appendix A).
Values are i.i.d. normal: the paper's pretrained weights and token streams are
not available, so these stand in for them.
"""
from .workloads import (ArmtShape, CONFIGS, get_shape, make_weights, make_embeddings,
                        round_to_bf16, bf16_bits, from_bf16_bits, LAYER_FIELDS, make_token_ends, LLAMA3_VOCAB,
                        describe_workload)

__all__ = ["ArmtShape", "CONFIGS", "get_shape", "make_weights", "make_embeddings",
           "round_to_bf16", "bf16_bits", "from_bf16_bits", "LAYER_FIELDS", "make_token_ends", "LLAMA3_VOCAB",
           "describe_workload"]
