"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path.

This package holds input generation only: a counter-based random generator,
the decoder shapes of the five workloads, and the token / length / block-table
recipes.  None of the transformer arithmetic lives here.
"""
from .gen import uniform_bits, uniform01, normal, randint, permutation  # noqa: F401
from .configs import (  # noqa: F401
    DecoderShape, TINY, LLAMA7B, LLAMA13B, MISTRAL7B, make_weights, SEED_BASE,
)
