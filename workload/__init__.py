"""Seeded synthetic inputs (weights, prompts) for the early-exit decode path.

This module serves both the CPU oracle and the HIP library and therefore holds
none of the method's arithmetic: it only turns (seed, tensor id, element index)
into numbers.  See ``gen.py``.
"""
from .gen import (  # noqa: F401
    CONFIGS,
    ModelShape,
    TABLE4_EXIT_HEAD_SCALE,
    TensorKind,
    gaussian_tensor,
    model_tensor,
    model_tensor_list,
    prompt_tokens,
    prompt_lengths,
    to_numpy,
    write_weight_file,
)
