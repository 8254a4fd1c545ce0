"""Pins for the oracle's negacyclic NTT and automorphisms: the O(N^2) definition, closed forms
on monomials, the convolution theorem against the schoolbook negacyclic product, round trips."""
import numpy as np
import pytest

from oracle import Oracle
from workloads.params import make_params
from helpers import brv


@pytest.mark.parametrize("log_n", [2, 5, 10])
def test_fast_ntt_equals_definition(log_n):
    p = make_params(log_n, 2, 0, 1, bits=30)
    o = Oracle(p)
    rng = np.random.default_rng(log_n)
    for t, q in enumerate(p.moduli):
        a = rng.integers(0, q, size=o.N, dtype=np.uint64)
        assert np.array_equal(o.ntt_fwd(a, t), o.ntt_definition(a, t))


@pytest.mark.parametrize("log_n", [3, 6])
def test_ntt_of_monomial_closed_form(log_n):
    """NTT(X^i)[k] = psi^((2 brv(k)+1) i), computed here with Python integers."""
    p = make_params(log_n, 1, 0, 1, bits=40)
    o = Oracle(p)
    q, psi, N = p.moduli[0], p.psi[0], o.N
    for i in (0, 1, N // 2 + 1, N - 1):
        a = np.zeros(N, dtype=np.uint64)
        a[i] = 7
        want = [7 * pow(psi, (2 * brv(k, log_n) + 1) * i, q) % q for k in range(N)]
        assert o.ntt_fwd(a, 0).tolist() == want


@pytest.mark.parametrize("log_n", [4, 12, 16])
def test_ntt_round_trip(log_n):
    p = make_params(log_n, 2, 1, 1)
    o = Oracle(p)
    rng = np.random.default_rng(1)
    for t, q in enumerate(p.moduli):
        a = rng.integers(0, q, size=o.N, dtype=np.uint64)
        a[:3] = (0, 1, q - 1)
        assert np.array_equal(o.ntt_inv(o.ntt_fwd(a, t), t), a)
        assert np.array_equal(o.ntt_fwd(o.ntt_inv(a, t), t), a)


@pytest.mark.parametrize("log_n", [3, 8])
def test_convolution_theorem_vs_schoolbook(log_n):
    p = make_params(log_n, 1, 0, 1)
    o = Oracle(p)
    q = p.moduli[0]
    rng = np.random.default_rng(2)
    a = rng.integers(0, q, size=o.N, dtype=np.uint64)
    b = rng.integers(0, q, size=o.N, dtype=np.uint64)
    prod_ntt = o.mul(o.ntt_fwd(a, 0)[None], o.ntt_fwd(b, 0)[None], [0])[0]
    assert np.array_equal(o.ntt_inv(prod_ntt, 0), o.schoolbook(q, a, b))


def test_schoolbook_is_negacyclic():
    """X^(N-1) * X = X^N = -1."""
    p = make_params(3, 1, 0, 1, bits=20)
    o = Oracle(p)
    q = p.moduli[0]
    a = np.zeros(8, dtype=np.uint64); a[7] = 1
    b = np.zeros(8, dtype=np.uint64); b[1] = 1
    want = np.zeros(8, dtype=np.uint64); want[0] = q - 1
    assert np.array_equal(o.schoolbook(q, a, b), want)


def test_ntt_many_matches_single():
    p = make_params(6, 3, 2, 1)
    o = Oracle(p)
    rng = np.random.default_rng(3)
    idx = [0, 2, 4, 3]
    polys = np.stack([[rng.integers(0, p.moduli[t], size=o.N, dtype=np.uint64) for t in idx] for _ in range(3)])
    fwd = o.ntt_many(polys, idx)
    for b in range(3):
        for a, t in enumerate(idx):
            assert np.array_equal(fwd[b, a], o.ntt_fwd(polys[b, a], t))
    assert np.array_equal(o.ntt_many(fwd, idx, inverse=True), polys)


@pytest.mark.parametrize("log_n", [4, 9])
def test_automorphism_forms_agree(log_n):
    """Gather in evaluation form == index map with sign in coefficient form, through the NTT."""
    p = make_params(log_n, 1, 0, 1)
    o = Oracle(p)
    q = p.moduli[0]
    rng = np.random.default_rng(4)
    a = rng.integers(0, q, size=o.N, dtype=np.uint64)
    for r in (1, 3, o.n - 1):
        g = o.galois(r)
        assert np.array_equal(o.automorph_ntt(o.ntt_fwd(a, 0), g), o.ntt_fwd(o.automorph_coeff(a, 0, g), 0))
    g = 2 * o.N - 1  # conjugation X -> X^-1 is an automorphism too
    assert np.array_equal(o.automorph_ntt(o.ntt_fwd(a, 0), g), o.ntt_fwd(o.automorph_coeff(a, 0, g), 0))


def test_automorphism_monomial_closed_form():
    """sigma_g(X^i) = X^(i g mod 2N) with X^N = -1."""
    p = make_params(4, 1, 0, 1, bits=20)
    o = Oracle(p)
    q, N = p.moduli[0], 16
    g = 5
    for i in range(N):
        a = np.zeros(N, dtype=np.uint64); a[i] = 3
        e = i * g % (2 * N)
        want = np.zeros(N, dtype=np.uint64)
        want[e % N] = 3 if e < N else q - 3
        assert np.array_equal(o.automorph_coeff(a, 0, g), want)


def test_automorphism_composition():
    p = make_params(7, 1, 0, 1)
    o = Oracle(p)
    q = p.moduli[0]
    a = np.random.default_rng(5).integers(0, q, size=o.N, dtype=np.uint64)
    g1, g2 = o.galois(3), o.galois(11)
    assert np.array_equal(o.automorph_ntt(o.automorph_ntt(a, g1), g2), o.automorph_ntt(a, o.galois(14)))
    assert np.array_equal(o.automorph_ntt(o.automorph_ntt(a, g1), o.galois(-3)), a)
