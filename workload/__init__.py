"""Seeded synthetic inputs shared by the oracle-side and GPU-side tests and benchmarks.

Holds only input generation (shapes, random weights, random prompts); none of
the decoding method's arithmetic lives here.
"""
from .configs import CONFIGS, TINY, get_config  # noqa: F401
from .generate import make_weights, make_prompts, round_to_bf16  # noqa: F401
