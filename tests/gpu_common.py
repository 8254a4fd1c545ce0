"""Helpers shared by the GPU parity tests: seeded operands and oracle-made keys/ciphertexts."""
import numpy as np


def rand_poly(rng, moduli, n):
    """[len(moduli)][n] uniform residues."""
    return np.stack([rng.integers(0, q, size=n, dtype=np.uint64) for q in moduli])


def rand_ct(rng, moduli, level, n):
    return np.stack([rand_poly(rng, moduli[:level + 1], n) for _ in range(2)])


def w_residues(w_int, moduli, level):
    """[C_out][C_in][9] signed integers -> residues [C_out][C_in][9][level+1]."""
    co, ci, nt = w_int.shape
    out = np.empty((co, ci, nt, level + 1), dtype=np.uint64)
    for i in range(level + 1):
        q = int(moduli[i])
        out[..., i] = np.mod(w_int.astype(object), q).astype(np.uint64)
    return out
