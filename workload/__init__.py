"""Seeded synthetic input generators shared by the CPU oracle's tests and the HIP path.

This package holds NO arithmetic of the scoring / SubSample method: only counter-based
pseudo-random draws (weights, token ids, prefix lengths, page permutations, uniforms) and
the shape presets of the five benchmark configurations.
"""
from .rng import (stream_key, raw_u32, normal_table, normal_tensor, uniform_f64,
                  zipf_tokens, uniform_tokens, permutation, bf16_round_f32)
from .configs import ModelDesc, Workload, CONFIGS, get_config, weight_shapes
