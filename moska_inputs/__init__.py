"""Seeded synthetic inputs for the MoSKA decode-attention path.

This package only *describes* problems and *draws* their tensors.  It holds none
of the method's arithmetic (no routing, no softmax, no merge) and imports neither
the CPU oracle nor the HIP library: both are fed from here by the tests and the
benchmark.
"""
from .problem import Problem, DTYPE_CODES, torch_dtype, CONFIGS, config
from .generate import Inputs, generate

__all__ = ["Problem", "DTYPE_CODES", "torch_dtype", "CONFIGS", "config", "Inputs", "generate"]
