"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This package holds shapes, seeds and random draws only: none of the method's
arithmetic (no norm, no attention, no LoRA, no allocator logic) lives here.
"""
from .synth import (  # noqa: F401
    ModelCfg, LoraCfg, DecodeCfg, FinetuneCfg, Workload, CONFIGS, workload,
    rng_for, bf16_round, bf16_bits, bf16_from_bits,
    make_layer_weights, make_lora, make_decode_inputs, make_finetune_inputs,
    make_model_extras, draw_lengths, page_order, make_token_ids, make_arrivals, LORA_TARGETS,
)
