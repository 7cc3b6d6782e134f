"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no rescale, no quantisation, no pruning, no coding): those
live, separately and independently, in the CPU oracle and in the HIP library.
"""
from .gen import (  # noqa: F401
    MatrixSpec,
    LLAMA7B_LAYER,
    LLAMA13B_LAYER,
    matrix_seed,
    gen_weight,
    gen_act_absmax,
    gen_activation_bf16,
    layer_specs,
)
