"""The double-precision modular arithmetic of the HIP library (csrc/f64mod.h: the butterflies', the basis
conversions' and the fused inner products' one copy of it) against 128-bit integers, on the CPU.

The header compiles for the host as it does for the GPU; tests/f64mod_check.cpp wraps it and also holds the
judges (signed 128-bit integer arithmetic), which the GPU test of the same routines reuses.  Cases: more than
10^7 seeded random ones, and the boundaries the random ones do not reach: multiplicands at 0, 1, q/2, q-1,
2q-1 and 2^51-1 in both signs, multipliers 0, 1, q-1, products whose quotient by q is within a rounding of a
tie (results at +-q/2), sums of the stated numbers of terms at their largest, for the benchmark's primes (the
largest NTT-friendly primes below 2^50), the largest primes below 2^50 of any kind and small ones."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from workloads.params import CONFIGS, is_prime, ntt_primes

HERE = os.path.dirname(os.path.abspath(__file__))


def build_checker(out_dir):
    so = os.path.join(str(out_dir), "libf64mod_check.so")
    cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-shared", "-fPIC", "-o", so, os.path.join(HERE, "f64mod_check.cpp")]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    lib = ctypes.CDLL(so)
    lib.chk_product.restype = ctypes.c_long
    lib.chk_reduce.restype = ctypes.c_long
    lib.chk_canonical.restype = ctypes.c_long
    lib.chk_centre.restype = ctypes.c_long
    lib.chk_dot.restype = ctypes.c_long
    lib.chk_fold.restype = ctypes.c_long
    lib.run_fwd_round.restype = ctypes.c_double
    lib.run_fwd_round_any.restype = ctypes.c_double
    lib.run_inv_round.restype = ctypes.c_double
    lib.run_inv_round_any.restype = ctypes.c_double
    return lib


@pytest.fixture(scope="module")
def lib(tmp_path_factory):
    return build_checker(tmp_path_factory.mktemp("f64mod"))


def ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def largest_primes_below(bound, count):
    out, c = [], bound - 1
    while len(out) < count:
        if is_prime(c):
            out.append(c)
        c -= 1
    return out


def primes_under_test():
    cfg = CONFIGS["cfg5_resnet20_stage3"].params().moduli
    ps = [cfg[0], cfg[-1], cfg[len(cfg) // 2]]             # the benchmark's chain and special primes
    ps += largest_primes_below(1 << 50, 2)                 # the largest moduli the arithmetic admits
    ps += ntt_primes(13, 1, bits=36) + ntt_primes(12, 1, bits=20) + [12289]
    return ps


PRIMES = primes_under_test()


def boundary_multiplicands(q, limit):
    """Signed multiplicands at the edges of the admitted range |y| < limit."""
    vals = [0, 1, 2, q // 2, q // 2 + 1, q - 1, q, q + 1, 2 * q - 1, 2 * q, (1 << 51) - 1, (1 << 50), (1 << 50) - 1, limit - 1]
    vals = sorted({v for v in vals if 0 <= v < limit})
    return np.array(vals + [-v for v in vals], dtype=np.int64)


def near_tie_pairs(q, rng, count, limit):
    """(y, w) with y*w = +-(q-1)/2 + t (mod q), |t| <= 2: the quotient y*w/q is within a few units of q of a tie."""
    w = rng.integers(1, q, size=count, dtype=np.uint64)
    ys = []
    for wi in w.tolist():
        t = int(rng.integers(-2, 3))
        target = ((q - 1) // 2 + t) % q if rng.integers(0, 2) else ((q + 1) // 2 + t) % q
        y = target * pow(wi, -1, q) % q                      # y in [0, q)
        y += q * int(rng.integers(0, max(1, (limit - y) // q)))   # any admitted representative
        if rng.integers(0, 2):
            y = y - q * ((y // q) + 1) if y - q * ((y // q) + 1) > -limit else y   # a negative representative
        ys.append(y)
    return np.array(ys, dtype=np.int64), w


def check_product(lib, run, y, w, q, num, den):
    y = np.ascontiguousarray(y, dtype=np.int64)
    w = np.ascontiguousarray(w, dtype=np.uint64)
    r = np.empty(len(y), dtype=np.float64)
    run(ptr(y), ptr(w), ctypes.c_uint64(q), ptr(r), ctypes.c_size_t(len(y)))
    worst = ctypes.c_double(0)
    bad = lib.chk_product(ptr(y), ptr(w), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(y)), num, den, ctypes.byref(worst))
    assert bad < 0, f"q={q}: y={int(y[bad])} w={int(w[bad])} gave {r[bad]!r}"
    return worst.value


@pytest.mark.parametrize("q", PRIMES)
def test_mulmod_precomputed_quotient(lib, q):
    """mulmod: |y| < 2^51, 0 <= w < q: exact, at most (1/2 + |y| / 2^53) q < 3/4 q; below 0.57 q for reduced multiplicands."""
    rng = np.random.default_rng(q % 1000003)
    limit = 1 << 51
    edge_y = boundary_multiplicands(q, limit)
    edge_w = np.array(sorted({0, 1, 2, q // 2, (q + 1) // 2, q - 2, q - 1}), dtype=np.uint64)
    yy, ww = np.meshgrid(edge_y, edge_w)
    check_product(lib, lib.run_mulmod, yy.ravel(), ww.ravel(), q, 3, 4)
    n = 1_000_000
    y = rng.integers(-(limit - 1), limit, size=n, dtype=np.int64)
    w = rng.integers(0, q, size=n, dtype=np.uint64)
    worst = check_product(lib, lib.run_mulmod, y, w, q, 3, 4)
    assert worst > 0.49                                      # the quotient is rounded, not truncated
    y, w = near_tie_pairs(q, rng, 20000, limit)
    check_product(lib, lib.run_mulmod, y, w, q, 3, 4)
    half = q // 2 + 1                                        # what a reduction leaves
    y = rng.integers(-half, half + 1, size=n, dtype=np.int64)
    check_product(lib, lib.run_mulmod, y, rng.integers(0, q, size=n, dtype=np.uint64), q, 57, 100)
    y, w = near_tie_pairs(q, rng, 20000, half)
    check_product(lib, lib.run_mulmod, y, w, q, 57, 100)


@pytest.mark.parametrize("q", PRIMES)
def test_mulmod_data_multiplier(lib, q):
    """mulmod_any (quotient from the rounded product): |y| < q, 0 <= w < q: exact, at most (1/2 + |y| / 2^52) q < 3/4 q;
    below 0.63 q for reduced multiplicands; exact and at most q for |y| < 2q."""
    rng = np.random.default_rng(q % 1000003 + 1)
    edge_y = boundary_multiplicands(q, q)
    edge_w = np.array(sorted({0, 1, 2, q // 2, (q + 1) // 2, q - 2, q - 1}), dtype=np.uint64)
    yy, ww = np.meshgrid(edge_y, edge_w)
    check_product(lib, lib.run_mulmod_any, yy.ravel(), ww.ravel(), q, 3, 4)
    n = 1_000_000
    y = rng.integers(-(q - 1), q, size=n, dtype=np.int64)
    w = rng.integers(0, q, size=n, dtype=np.uint64)
    check_product(lib, lib.run_mulmod_any, y, w, q, 3, 4)
    y, w = near_tie_pairs(q, rng, 20000, q)
    check_product(lib, lib.run_mulmod_any, y, w, q, 3, 4)
    half = q // 2 + 1
    y = rng.integers(-half, half + 1, size=n, dtype=np.int64)
    w = rng.integers(0, q, size=n, dtype=np.uint64)
    check_product(lib, lib.run_mulmod_any, y, w, q, 63, 100)
    y, w = near_tie_pairs(q, rng, 20000, half)
    check_product(lib, lib.run_mulmod_any, y, w, q, 63, 100)
    # as a butterfly's twiddle product (the lo passes hold a twiddle's value alone): multiplicands up to 2q, at most q
    wide = 2 * q
    yy, ww = np.meshgrid(boundary_multiplicands(q, wide), edge_w)
    check_product(lib, lib.run_mulmod_any, yy.ravel(), ww.ravel(), q, 1, 1)
    y = rng.integers(-(wide - 1), wide, size=n, dtype=np.int64)
    check_product(lib, lib.run_mulmod_any, y, rng.integers(0, q, size=n, dtype=np.uint64), q, 1, 1)
    y, w = near_tie_pairs(q, rng, 20000, wide)
    check_product(lib, lib.run_mulmod_any, y, w, q, 1, 1)


@pytest.mark.parametrize("q", PRIMES)
def test_reduce_and_canonical(lib, q):
    """reduce: integer |v| < 2^53 -> |r| <= q/2 + 1; canonical(reduce(v)) = v mod q."""
    rng = np.random.default_rng(q % 1000003 + 2)
    lim = 1 << 53
    edges = [0, 1, q // 2, q // 2 + 1, q - 1, q, q + 1, lim - 1, lim - 2]
    edges += [k * q + d for k in (1, 2, 3, 7, (lim - 1) // q) for d in (-1, 0, 1, q // 2, q // 2 + 1) if k * q + d < lim]
    edges = np.array(edges + [-e for e in edges], dtype=np.int64)
    v = np.concatenate([edges, rng.integers(-(lim - 1), lim, size=500_000, dtype=np.int64),
                        rng.integers(-4 * q, 4 * q, size=200_000, dtype=np.int64)])
    r = np.empty(len(v), dtype=np.float64)
    lib.run_reduce(ptr(v), ctypes.c_uint64(q), ptr(r), ctypes.c_size_t(len(v)))
    bad = lib.chk_reduce(ptr(v), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(v)))
    assert bad < 0, f"q={q}: reduce({int(v[bad])}) = {r[bad]!r}"
    c = np.empty(len(v), dtype=np.uint64)
    lib.run_canonical(ptr(v), ctypes.c_uint64(q), ptr(c), ctypes.c_size_t(len(v)))
    bad = lib.chk_canonical(ptr(v), ptr(c), ctypes.c_uint64(q), ctypes.c_size_t(len(v)))
    assert bad < 0, f"q={q}: canonical({int(v[bad])}) = {int(c[bad])}"


def test_u64_double_round_trip(lib):
    rng = np.random.default_rng(7)
    v = np.concatenate([np.array([0, 1, 2, (1 << 50) - 1, 1 << 50, (1 << 52) - 1], dtype=np.uint64),
                        rng.integers(0, 1 << 52, size=200_000, dtype=np.uint64)])
    r = np.empty_like(v)
    lib.run_from_to_u64(ptr(v), ptr(r), ctypes.c_size_t(len(v)))
    assert np.array_equal(v, r)


@pytest.mark.parametrize("q", PRIMES[:5])
def test_centred_scaled_store(lib, q):
    """What the inverse transform leaves in front of a basis conversion: v * k mod q as the centred residue."""
    rng = np.random.default_rng(q % 1000003 + 3)
    for k in (1, q - 1, (q + 1) // 2, int(rng.integers(2, q))):
        v = np.concatenate([boundary_multiplicands(q, 2 * q), rng.integers(-(2 * q - 1), 2 * q, size=200_000, dtype=np.int64)])
        # values that land next to +-q/2 after the multiplication
        kinv = pow(k, -1, q)
        near = [(((q - 1) // 2 + t) * kinv) % q for t in range(-2, 4)]
        v = np.concatenate([v, np.array(near + [x - q for x in near], dtype=np.int64)])
        r = np.empty(len(v), dtype=np.float64)
        lib.run_centre(ptr(v), ctypes.c_uint64(k), ctypes.c_uint64(q), ptr(r), ctypes.c_size_t(len(v)))
        bad = lib.chk_centre(ptr(v), ctypes.c_uint64(k), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(v)))
        assert bad < 0, f"q={q} k={k}: v={int(v[bad])} gave {r[bad]!r}"


@pytest.mark.parametrize("nd", [1, 4, 8, 9, 12, 16])
@pytest.mark.parametrize("q", PRIMES)
def test_conversion_sums(lib, q, nd):
    """The basis-conversion sum of nd centred source residues times constants below q (their centred representatives): exact
    although a chain of eight products reaches 2^101; inputs at their largest (|y| = 2^49 source residues of a 50-bit modulus
    against the constants of largest magnitude, all of one sign and alternating), constants q - 1, powers of two that put
    every product half way between two multiples of 2^50 (the chain's rounding ties), rows whose every product is congruent
    to about +-q/2, and random."""
    rng = np.random.default_rng(q % 1000003 + nd)
    half_src = (1 << 49) - 1                                  # centred residues of a source modulus below 2^50
    n = 100_000
    y = rng.integers(-half_src, half_src + 1, size=(n, nd), dtype=np.int64)
    y[0] = half_src
    y[1] = -half_src
    y[2, ::2], y[2, 1::2] = half_src, -half_src
    y[40:2000] = 4 * rng.integers(-(half_src // 4), half_src // 4, size=(1960, nd), dtype=np.int64) + 2    # y = 2 mod 4
    mixed = rng.integers(0, q, size=nd, dtype=np.uint64)
    mixed[::2] = (q + 1) // 2                                  # centred -(q - 1) / 2 next to random constants
    tie = min(1 << 48, 1 << (q.bit_length() - 2))              # y * 2^48 = 2^49 mod 2^50 for y = 2 mod 4
    for cw in (rng.integers(0, q, size=nd, dtype=np.uint64), np.full(nd, q - 1, dtype=np.uint64), np.full(nd, (q + 1) // 2, dtype=np.uint64),
               np.full(nd, (q - 1) // 2, dtype=np.uint64), np.full(nd, tie, dtype=np.uint64), mixed):
        cw = np.ascontiguousarray(cw)
        yy = y.copy()
        # rows whose every product is congruent to about +q/2: the sum of the per-term results is as large as it gets
        for row in range(3, 40):
            for a in range(nd):
                c = int(cw[a])
                if c:
                    t = ((q - 1) // 2 - int(rng.integers(0, 3))) * pow(c, -1, q) % q
                    yy[row, a] = t if t <= half_src else t - q if q - t <= half_src else yy[row, a]
        r = np.empty(n, dtype=np.float64)
        assert lib.run_dot(ptr(yy), ptr(cw), nd, ctypes.c_uint64(q), ptr(r), ctypes.c_size_t(n)) == 0
        bad = lib.chk_dot(ptr(yy), ptr(cw), nd, ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(n))
        assert bad < 0, f"q={q} nd={nd}: row {yy[bad].tolist()} gave {r[bad]!r}"


@pytest.mark.parametrize("fn", ["run_fwd_round", "run_fwd_round_any"])
@pytest.mark.parametrize("q", PRIMES[:5])
def test_forward_round_of_three_stages(lib, q, fn):
    """Three butterfly stages on reduced inputs and the reduction that ends the round, as the transforms chain them:
    every multiplicand stays below 2q (so below 2^51), the results match exact integer butterflies.  With the twiddle's
    quotient precomputed, and with the twiddle's value alone (the fused inner-product pass)."""
    rng = np.random.default_rng(q % 1000003 + 5)
    half = q // 2 + 1
    worst = 0.0
    for trial in range(20000):
        if trial < 64:                                       # all inputs and all twiddles at their extremes
            v = np.array([half if (trial >> j) & 1 else -half for j in range(6)] + [half, -half], dtype=np.int64)
            tw = np.array([q - 1, 1, q - 1, (q + 1) // 2, (q - 1) // 2, q - 2, 2], dtype=np.uint64)
        else:
            v = rng.integers(-half, half + 1, size=8, dtype=np.int64)
            tw = rng.integers(0, q, size=7, dtype=np.uint64)
        want = np.empty(8, dtype=np.uint64)
        lib.ref_fwd_round(ptr(v), ptr(tw), ctypes.c_uint64(q), ptr(want))
        got = v.copy()
        worst = max(worst, getattr(lib, fn)(ptr(got), ptr(tw), ctypes.c_uint64(q)))
        assert np.all(np.abs(got) <= half), (q, trial)
        assert np.array_equal(np.mod(got, q).astype(np.uint64), want), (q, trial)
    assert worst < 2 * q


@pytest.mark.parametrize("fn", ["run_inv_round", "run_inv_round_any"])
@pytest.mark.parametrize("q", PRIMES[:5])
def test_inverse_round_of_three_stages(lib, q, fn):
    """Three inverse butterfly stages (sum re-centred, difference times the twiddle) chained as the inverse transforms chain
    them, from reduced inputs and from inputs as large as a previous round's products leave them (below q): every
    multiplicand stays below 2q, every value that enters the next round stays below q, the results match exact integer
    butterflies.  With the twiddle's quotient precomputed, and with the twiddle's value alone (the inverse lo pass)."""
    rng = np.random.default_rng(q % 1000003 + 6)
    worst = 0.0
    for bound in (q // 2 + 1, q - 1):
        for trial in range(10000):
            if trial < 64:
                v = np.array([bound if (trial >> j) & 1 else -bound for j in range(6)] + [bound, -bound], dtype=np.int64)
                tw = np.array([q - 1, 1, q - 1, (q + 1) // 2, (q - 1) // 2, q - 2, 2], dtype=np.uint64)
            else:
                v = rng.integers(-bound, bound + 1, size=8, dtype=np.int64)
                tw = rng.integers(0, q, size=7, dtype=np.uint64)
            want = np.empty(8, dtype=np.uint64)
            lib.ref_inv_round(ptr(v), ptr(tw), ctypes.c_uint64(q), ptr(want))
            got = v.copy()
            worst = max(worst, getattr(lib, fn)(ptr(got), ptr(tw), ctypes.c_uint64(q)))
            assert np.all(np.abs(got) < q), (q, trial)
            assert np.array_equal(np.mod(got, q).astype(np.uint64), want), (q, trial)
    assert worst < 2 * q


@pytest.mark.parametrize("nd", [9, 10, 13])
@pytest.mark.parametrize("q", PRIMES + [3, 5, 131071, 131101])
def test_fold_of_digit_diagonals(lib, q, nd):
    """The matrix-core sum's last step: sum_s D_s 256^s mod q for 32-bit signed diagonals D_s, with 9, 10 or 13 of them
    (3-, 4- and 7-digit weights).  Boundaries: every diagonal at +-(2^31 - 1) and at -2^31 (the three partial sums at
    their largest), single diagonals at the extremes, zeros; then seeded random diagonals of full 32-bit range and of
    the benchmark's range (|D| < 2^26).  Moduli include 3, 5 and ones just below and above the multiplier 2^17."""
    rng = np.random.default_rng(1000 * nd + q % 997)
    c = np.array([pow(256, s, q) for s in range(nd)], dtype=np.uint64)
    lo, hi = -(1 << 31), (1 << 31) - 1
    rows = [np.full(nd, hi), np.full(nd, lo), np.zeros(nd), np.full(nd, 1), np.full(nd, -1),
            np.where(np.arange(nd) % 2 == 0, hi, lo), np.where(np.arange(nd) % 2 == 0, lo, hi)]
    for s in range(nd):
        for v in (hi, lo, 1, -1):
            row = np.zeros(nd)
            row[s] = v
            rows.append(row)
    edge = np.array(rows, dtype=np.int64).astype(np.int32)
    wide = rng.integers(lo, hi + 1, size=(150_000, nd), dtype=np.int64).astype(np.int32)
    bench = rng.integers(-(1 << 26), 1 << 26, size=(150_000, nd), dtype=np.int64).astype(np.int32)
    for D in (edge, wide, bench):
        D = np.ascontiguousarray(D)
        r = np.empty(D.shape[0], dtype=np.float64)
        assert lib.run_fold(ptr(D), ptr(c), nd, ctypes.c_uint64(q), ptr(r), ctypes.c_size_t(D.shape[0])) == 0
        assert lib.chk_fold(ptr(D), ptr(c), nd, ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(D.shape[0])) == 0
    # the judge itself: a planted off-by-one is caught
    r[0] += 1.0
    assert lib.chk_fold(ptr(D), ptr(c), nd, ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(D.shape[0])) == 1
