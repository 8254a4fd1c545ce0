"""Seeded synthetic tensors standing in for the paper's CIFAR images and trained, BN-folded
ResNet weights (Experiments section), which are not available: same shapes, same value ranges.

Every object gets its own sub-seed derived from the master seed and a label, so that the oracle
side and the HIP side of a test can regenerate identical inputs independently.
"""
from __future__ import annotations

import hashlib
from typing import List, Sequence

import numpy as np

MASTER_SEED = 0x260416834


def sub_seed(label: str, seed: int = MASTER_SEED) -> int:
    h = hashlib.sha256(f"{seed}:{label}".encode()).digest()
    return int.from_bytes(h[:8], "little")


def _rng(label: str, seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(sub_seed(label, seed)))


def image_batch(batch: int, channels: int, height: int, width: int, seed: int = MASTER_SEED) -> np.ndarray:
    """Pixels uniform in [-1, 1], shape [batch, channels, height, width], float64."""
    return _rng("images", seed).uniform(-1.0, 1.0, size=(batch, channels, height, width))


def conv_weights(c_out: int, c_in: int, ksize: int = 3, seed: int = MASTER_SEED,
                 dist: str = "he_normal") -> np.ndarray:
    """3x3 kernels, shape [c_out, c_in, k, k].  ``he_normal``: N(0, 2/(k*k*c_in)) as for a
    ReLU network at initialisation; ``uniform``: U[-0.5, 0.5] (the single-channel case)."""
    r = _rng("weights", seed)
    if dist == "uniform":
        return r.uniform(-0.5, 0.5, size=(c_out, c_in, ksize, ksize))
    std = (2.0 / (ksize * ksize * c_in)) ** 0.5
    return r.normal(0.0, std, size=(c_out, c_in, ksize, ksize))


def rotation_offsets(count: int, slots: int, seed: int = MASTER_SEED) -> List[int]:
    """``count`` distinct rotation amounts drawn from [1, slots-1]."""
    r = _rng("offsets", seed)
    return sorted(int(x) for x in r.choice(np.arange(1, slots), size=count, replace=False))


def uniform_residues(shape: Sequence[int], moduli: Sequence[int], label: str,
                     seed: int = MASTER_SEED) -> np.ndarray:
    """uint64 array of the given shape whose second-to-last axis runs over ``moduli``: entry
    [..., t, :] is uniform in [0, moduli[t])."""
    shape = tuple(shape)
    assert shape[-2] == len(moduli)
    r = _rng(label, seed)
    out = np.empty(shape, dtype=np.uint64)
    for t, q in enumerate(moduli):
        out[..., t, :] = r.integers(0, q, size=shape[:-2] + shape[-1:], dtype=np.uint64)
    return out


def conv_tap_offsets(width: int) -> List[int]:
    """Slot offsets of the nine taps of a 3x3 window in row-major (dy, dx) order for images
    flattened row by row: dy*W + dx for dy, dx in {-1, 0, 1}."""
    return [dy * width + dx for dy in (-1, 0, 1) for dx in (-1, 0, 1)]
