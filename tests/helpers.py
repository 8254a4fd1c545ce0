"""Exact big-integer helpers for the oracle pins (Python integers, no shared code with either
implementation)."""
from math import prod


def crt(residues, moduli):
    """The integer in [0, prod(moduli)) with the given residues."""
    Q = prod(moduli)
    x = 0
    for r, q in zip(residues, moduli):
        Qi = Q // q
        x += int(r) * Qi * pow(Qi, -1, q)
    return x % Q


def centred(x, Q):
    x %= Q
    return x - Q if x > Q // 2 else x


def brv(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2) if bits else 0
