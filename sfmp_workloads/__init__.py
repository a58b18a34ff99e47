"""Seeded synthetic inputs for the SFMP mixed-precision GEMM/GEMV path.

This module only *produces inputs* (weights, activations, bitmaps,
permutations and the quantised codes / scales / zero-points derived from
them).  It holds none of the arithmetic of the inference path (no packing, no
unpacking, no dequantisation, no matmul): those live, separately, in the CPU
oracle and in the HIP library, and both consume what is generated here.

Shapes are the LLaMA-3.1 8B / 70B linear-layer shapes the paper evaluates
(Section 4, experimental setup; Section 3.5 names the 4096x4096 q_proj).  The
paper's real checkpoints, Fisher statistics and bitmaps are not available, so
every tensor is drawn from a seeded numpy PCG64 generator.
"""
from .generators import (  # noqa: F401
    TILE,
    GROUP,
    SHAPES_8B,
    SHAPES_70B,
    LAYER_8B,
    LAYER_70B,
    CONFIGS,
    Problem,
    make_bitmap,
    block_bitmap,
    to_bf16,
    param_bits,
    clustered_bitmap,
    make_weights,
    make_activations,
    make_perm,
    quantize_minmax,
    random_quantized,
    make_problem,
    with_activations,
    config_cases,
    algorithmic_bytes,
    metadata_bits_per_weight,
)
from . import allocation  # noqa: E402,F401
