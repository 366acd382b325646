"""Seeded synthetic inputs for the KurTail rotation-learning step.

This module holds none of the method's arithmetic: it only draws activations X
shaped like the stored MHSA/FFN block inputs of a Llama-family model (a Gaussian
or heavy-tailed bulk, a few outlier channels, optional Student-t spikes) and
starting rotations R (identity or Haar-like orthogonal).  Both the HIP path and
the CPU oracle are fed from here so that they see identical bytes.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    make_x,
    make_problem,
    random_orthogonal,
    bf16_round,
    to_f64,
)
