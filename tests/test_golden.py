"""Stored oracle outputs (tests/golden/, written by make_golden.py from the oracle alone) checked
against the oracle as it is now and against independent Python-integer evaluations of the definitions."""
import os

import numpy as np

from oracle import Oracle
from workloads.params import make_params
from helpers import brv, crt, centred

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rows(name):
    return [list(map(int, line.split())) for line in open(os.path.join(GOLD, name)) if line.strip() and not line.startswith("#")]


def test_ntt_fixture():
    (q, psi), a, want = rows("ntt_n16.txt")
    p = make_params(4, 2, 1, 1, bits=20)
    assert (q, psi) == (p.moduli[0], p.psi[0])
    assert Oracle(p).ntt_fwd(np.array(a, dtype=np.uint64), 0).tolist() == want
    assert [sum(ai * pow(psi, (2 * brv(k, 4) + 1) * i, q) for i, ai in enumerate(a)) % q for k in range(16)] == want


def test_rescale_fixture():
    r = rows("rescale_n16.txt")
    (q0, q1, psi0, psi1), ins, outs = r[0], r[1:5], r[5:7]
    p = make_params(4, 2, 1, 1, bits=20)
    assert (q0, q1, psi0, psi1) == (p.moduli[0], p.moduli[1], p.psi[0], p.psi[1])
    o = Oracle(p)
    ct = np.array(ins, dtype=np.uint64).reshape(2, 2, 16)
    got = o.rescale(ct, 1)
    assert got[:, 0].tolist() == outs
    # independent: coefficient form, CRT, round(c / q1), back to evaluation form by the definition
    for comp in range(2):
        c0, c1 = o.ntt_inv(ct[comp, 0], 0), o.ntt_inv(ct[comp, 1], 1)
        coeffs = [centred(crt([int(x), int(y)], [q0, q1]), q0 * q1) for x, y in zip(c0, c1)]
        rounded = [(2 * c + q1) // (2 * q1) % q0 for c in coeffs]
        want = [sum(ai * pow(psi0, (2 * brv(k, 4) + 1) * i, q0) for i, ai in enumerate(rounded)) % q0 for k in range(16)]
        assert want == outs[comp]
