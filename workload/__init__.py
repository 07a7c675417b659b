"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check."""
from .gen import (BF16_NAN, CONFIGS, E4M3_NAN, PAGE, PrefillBatch, Problem, build_prefill, make_prefill, bf16_bits_to_f32, build_problem, e4m3_encode,
                  f32_to_bf16_bits, make_pool, make_problem, normal_bf16, response_lengths)

__all__ = ["BF16_NAN", "CONFIGS", "E4M3_NAN", "PAGE", "PrefillBatch", "Problem", "build_prefill", "make_prefill", "bf16_bits_to_f32", "build_problem",
           "e4m3_encode", "f32_to_bf16_bits", "make_pool", "make_problem", "normal_bf16", "response_lengths"]
