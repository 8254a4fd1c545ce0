"""Seeded synthetic inputs and parameter sets shared by the oracle-side tests and the HIP-side
tests / benchmark.

Nothing in this package performs the method's arithmetic (no NTT, no key switching, no
encoding): it only chooses parameters (primes, roots of unity as plain number-theory facts) and
draws seeded random tensors with the shapes and value ranges of the batched-CNN workloads.
"""
from .params import CkksParams, make_params, CONFIGS  # noqa: F401
from .tensors import (  # noqa: F401
    MASTER_SEED,
    sub_seed,
    image_batch,
    conv_weights,
    rotation_offsets,
    uniform_residues,
    conv_tap_offsets,
)
