"""Seeded synthetic inputs for the dKV-Cache hot path.

This module serves both the CPU oracle and the HIP path with the same bytes.
It holds no arithmetic of the method: only workload descriptors, counter-based
random draws, and the storage-format rounding of generated data.
"""
from .configs import ModelShape, RunShape, CONFIGS, model_run
from .rng import normal_f32, uniform_ids, permutation, bf16_round, bf16_bits, bits_to_f32
from .weights import SynthWeights
from .workloads import (prompt_tokens, random_block_order, attn_update_case,
                        AttnUpdateShape, CONFIG1_SHAPE, CONFIG1_ACTIVE_SIZES)
