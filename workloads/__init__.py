"""Seeded synthetic inputs shared by the CPU oracle and the HIP library.

This package describes *what is fed in*: operator graphs with symbolic input
dims, weight tensors and per-call symbol draws.  It performs none of the
method's arithmetic (no shape inference, no planning, no operator maths); every
intermediate tensor is left with an undeclared shape so that each consumer has
to infer it on its own.
"""
from .graphdesc import GraphDesc, TensorDesc, OpDesc, GraphBuilder  # noqa: F401
from .rng import normal, uniform, randint, to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from . import configs  # noqa: F401
