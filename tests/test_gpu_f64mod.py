"""The double-precision modular routines as the GPU evaluates them (ckks_f64mod_probe runs the device build of
csrc/f64mod.h), judged with the 128-bit integer checker of tests/f64mod_check.cpp on the grid of boundary and
near-tie cases of the CPU test plus seeded random ones: the device's fused multiply-add, rounding and conversions
behave as the host's do."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2604_16834_amd as hx  # noqa: E402
from test_f64mod import PRIMES, boundary_multiplicands, build_checker, near_tie_pairs, ptr  # noqa: E402


@pytest.fixture(scope="module")
def lib(tmp_path_factory):
    return build_checker(tmp_path_factory.mktemp("f64mod_gpu"))


def cases(q, limit, rng, n):
    edge_y = boundary_multiplicands(q, limit)
    edge_w = np.array(sorted({0, 1, 2, q // 2, (q + 1) // 2, q - 2, q - 1}), dtype=np.uint64)
    yy, ww = np.meshgrid(edge_y, edge_w)
    ty, tw = near_tie_pairs(q, rng, 5000, limit)
    y = np.concatenate([yy.ravel(), ty, rng.integers(-(limit - 1), limit, size=n, dtype=np.int64)])
    w = np.concatenate([ww.ravel(), tw, rng.integers(0, q, size=n, dtype=np.uint64)])
    return np.ascontiguousarray(y), np.ascontiguousarray(w)


def dev(a):
    return torch.from_numpy(a.view(np.int64) if a.dtype == np.uint64 else a).cuda()


@pytest.mark.parametrize("q", PRIMES)
def test_device_products_are_exact(lib, q):
    rng = np.random.default_rng(q % 1000003 + 11)
    for op, limit, num, den in ((hx.CKKS_F64_MULMOD, 1 << 51, 3, 4), (hx.CKKS_F64_MULMOD_ANY, q, 3, 4)):
        y, w = cases(q, limit, rng, 1_000_000)
        wq = w.astype(np.float64) / float(q)
        r = hx.ckks_f64mod_probe(op, dev(y), dev(w), dev(wq), q).cpu().numpy()
        worst = ctypes.c_double(0)
        bad = lib.chk_product(ptr(y), ptr(w), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(y)), num, den, ctypes.byref(worst))
        assert bad < 0, f"op {op}, q={q}: y={int(y[bad])} w={int(w[bad])} gave {r[bad]!r}"


@pytest.mark.parametrize("q", PRIMES)
def test_device_twiddle_products_up_to_2q(lib, q):
    """The lo passes' butterflies take the quotient from the rounded product for multiplicands up to 2q: exact, at most q."""
    rng = np.random.default_rng(q % 1000003 + 13)
    y, w = cases(q, 2 * q, rng, 500_000)
    r = hx.ckks_f64mod_probe(hx.CKKS_F64_MULMOD_ANY, dev(y), dev(w), None, q).cpu().numpy()
    worst = ctypes.c_double(0)
    bad = lib.chk_product(ptr(y), ptr(w), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(y)), 1, 1, ctypes.byref(worst))
    assert bad < 0, f"q={q}: y={int(y[bad])} w={int(w[bad])} gave {r[bad]!r}"


@pytest.mark.parametrize("nd,op", [(8, "CKKS_F64_DOT8"), (9, "CKKS_F64_DOT9")])
@pytest.mark.parametrize("q", PRIMES)
def test_device_conversion_sums(lib, q, nd, op):
    """The basis-conversion sum as a chain of fused multiply-adds on the device: operands at their extremes in one sign and
    alternating, products on the chain's rounding ties, random rows; against 128-bit integers."""
    rng = np.random.default_rng(q % 1000003 + 14 + nd)
    half_src = (1 << 49) - 1
    n = 200_000
    y = rng.integers(-half_src, half_src + 1, size=(n, nd), dtype=np.int64)
    y[0], y[1] = half_src, -half_src
    y[2, ::2], y[2, 1::2] = half_src, -half_src
    y[3, ::2], y[3, 1::2] = -half_src, half_src
    y[40:2000] = 4 * rng.integers(-(half_src // 4), half_src // 4, size=(1960, nd), dtype=np.int64) + 2
    tie = min(1 << 48, 1 << (q.bit_length() - 2))
    mixed = rng.integers(0, q, size=nd, dtype=np.uint64)
    mixed[::2] = (q + 1) // 2
    for cw in (rng.integers(0, q, size=nd, dtype=np.uint64), np.full(nd, q - 1, dtype=np.uint64), np.full(nd, (q + 1) // 2, dtype=np.uint64),
               np.full(nd, (q - 1) // 2, dtype=np.uint64), np.full(nd, tie, dtype=np.uint64), mixed):
        cw = np.ascontiguousarray(cw)
        yy = np.ascontiguousarray(y)
        r = hx.ckks_f64mod_probe(getattr(hx, op), dev(yy), dev(cw), None, q).cpu().numpy()
        bad = lib.chk_dot(ptr(yy), ptr(cw), nd, ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(n))
        assert bad < 0, f"q={q} nd={nd}: row {yy[bad].tolist()} gave {r[bad]!r}"


@pytest.mark.parametrize("q", PRIMES)
def test_device_reduce_canonical_and_centre(lib, q):
    rng = np.random.default_rng(q % 1000003 + 12)
    lim = 1 << 53
    edges = [0, 1, q // 2, q // 2 + 1, q - 1, q, q + 1, lim - 1, lim - 2]
    edges += [k * q + d for k in (1, 2, 3, 7, (lim - 1) // q) for d in (-1, 0, 1, q // 2, q // 2 + 1) if k * q + d < lim]
    v = np.concatenate([np.array(edges + [-e for e in edges], dtype=np.int64), rng.integers(-(lim - 1), lim, size=500_000, dtype=np.int64),
                        rng.integers(-4 * q, 4 * q, size=200_000, dtype=np.int64)])
    r = hx.ckks_f64mod_probe(hx.CKKS_F64_REDUCE, dev(v), None, None, q).cpu().numpy()
    bad = lib.chk_reduce(ptr(v), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(v)))
    assert bad < 0, f"q={q}: reduce({int(v[bad])}) = {r[bad]!r}"
    c = hx.ckks_f64mod_probe(hx.CKKS_F64_CANONICAL, dev(v), None, None, q).cpu().numpy()
    cu = np.ascontiguousarray(c.astype(np.uint64))
    assert np.array_equal(cu.astype(np.float64), c)
    bad = lib.chk_canonical(ptr(v), ptr(cu), ctypes.c_uint64(q), ctypes.c_size_t(len(v)))
    assert bad < 0, f"q={q}: canonical({int(v[bad])}) = {c[bad]!r}"
    k = int(rng.integers(2, q))
    y = np.concatenate([boundary_multiplicands(q, 2 * q), rng.integers(-(2 * q - 1), 2 * q, size=200_000, dtype=np.int64)])
    kinv = pow(k, -1, q)
    near = [(((q - 1) // 2 + t) * kinv) % q for t in range(-2, 4)]
    y = np.ascontiguousarray(np.concatenate([y, np.array(near + [x - q for x in near], dtype=np.int64)]))
    w = np.full(len(y), k, dtype=np.uint64)
    r = hx.ckks_f64mod_probe(hx.CKKS_F64_CENTRE, dev(y), dev(w), dev(w.astype(np.float64) / float(q)), q).cpu().numpy()
    bad = lib.chk_centre(ptr(y), ctypes.c_uint64(k), ptr(r), ctypes.c_uint64(q), ctypes.c_size_t(len(y)))
    assert bad < 0, f"q={q} k={k}: y={int(y[bad])} gave {r[bad]!r}"


def test_probe_rejects_bad_arguments():
    y = torch.zeros(4, dtype=torch.int64, device="cuda")
    with pytest.raises(hx.CkksError):
        hx.ckks_f64mod_probe(9, y, y, None, 12289)
    with pytest.raises(hx.CkksError):
        hx.ckks_f64mod_probe(hx.CKKS_F64_MULMOD, y, None, None, 12289)
    with pytest.raises(hx.CkksError):
        hx.ckks_f64mod_probe(hx.CKKS_F64_REDUCE, y, None, None, 1 << 50)
