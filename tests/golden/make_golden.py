#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ by calling ONLY the CPU oracle.

The paper prints no numeric example of a transform, key switch or ciphertext, so these files are
regression anchors of the oracle itself (each is also checked against an independent Python-integer
evaluation of its definition in tests/test_golden.py), not values quoted from the paper.
Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import Oracle  # noqa: E402
from workloads.params import make_params  # noqa: E402


def main():
    p = make_params(4, 2, 1, 1, bits=20)       # N = 16, two 20-bit chain primes, one special prime
    o = Oracle(p)
    a = np.arange(1, o.N + 1, dtype=np.uint64) * 12345 % p.moduli[0]
    with open(os.path.join(HERE, "ntt_n16.txt"), "w") as f:
        f.write("# negacyclic NTT, N = 16 (Background: RNS Decomposition and NTT Optimization); oracle output\n")
        f.write("# q psi\n%d %d\n# input coefficients\n%s\n# out[k] = a(psi^(2*bitrev(k)+1))\n%s\n"
                % (p.moduli[0], p.psi[0], " ".join(map(str, a.tolist())), " ".join(map(str, o.ntt_fwd(a, 0).tolist()))))
    # rescale of a fixed two-limb ciphertext component pair
    ct = np.stack([[(np.arange(o.N, dtype=np.uint64) * (7 + 3 * i + c) + 5) % p.moduli[i] for i in range(2)] for c in range(2)])
    out = o.rescale(ct, 1)
    with open(os.path.join(HERE, "rescale_n16.txt"), "w") as f:
        f.write("# rescale from level 1 to level 0, N = 16 (Experiments: HE Security Parameters); oracle output\n")
        f.write("# q0 q1 psi0 psi1\n%d %d %d %d\n" % (p.moduli[0], p.moduli[1], p.psi[0], p.psi[1]))
        for c in range(2):
            for i in range(2):
                f.write("# in comp %d limb %d\n%s\n" % (c, i, " ".join(map(str, ct[c, i].tolist()))))
        for c in range(2):
            f.write("# out comp %d\n%s\n" % (c, " ".join(map(str, out[c, 0].tolist()))))


if __name__ == "__main__":
    main()
