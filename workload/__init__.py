"""Seeded synthetic inputs for the MoE-layer hot path.

This package holds only input generation: a counter-based pseudo-random
generator, Gaussian weights, AR(1) hidden-state sequences and the table of
benchmark configurations.  It contains none of the method's arithmetic (no
router, no expert evaluation, no cache statistics) and imports neither the CPU
oracle nor the HIP library; both consume the tensors it produces as plain data.
"""
from .configs import CONFIGS, MoEConfig, get_config  # noqa: F401
from .gen import (  # noqa: F401
    hidden_states,
    TENSOR_IDS,
    ar1_hidden_states,
    gaussian,
    layer_weights,
    random_trace,
)
