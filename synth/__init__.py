"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This package draws random numbers and converts them to bf16 bit patterns.  It
holds none of the method's arithmetic (no projection, norm, rotation, layout
change or selection): those live, separately, in the CPU oracle and in the HIP
library, which share no code with each other.
"""
from .inputs import (  # noqa: F401
    CONFIGS,
    Config,
    SEED_BASE,
    bf16_bits_to_f32,
    config_seed,
    f32_to_bf16_bits,
    make_layer_inputs,
    make_v_pair,
    perturb_tiles,
    sample_token_ids,
)
