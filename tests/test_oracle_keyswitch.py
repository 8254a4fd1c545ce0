"""Pins for the oracle's hybrid key switching, rescale and ciphertext products: exact
big-integer invariants on tiny parameters and decrypt-and-compare identities."""
from math import prod

import numpy as np
import pytest

from oracle import Oracle
from workloads.params import make_params
from helpers import crt, centred


def coeff_form(o, poly, mod_idx):
    return np.stack([o.ntt_inv(poly[a], t) for a, t in enumerate(mod_idx)])


@pytest.mark.parametrize("level", [2, 1, 0])
def test_modup_is_c_plus_small_multiple_of_digit_modulus(tiny_params, level):
    """Extended digit j == c + u*Q_j as integers with |d_j| <= |digit| * Q_j / 2 (centred,
    uncorrected extension), for the full digit {q0,q1} and the ragged digit {q2}, at every level."""
    p = tiny_params
    o = Oracle(p)
    rng = np.random.default_rng(10 + level)
    c = np.stack([rng.integers(0, p.moduli[i], size=o.N, dtype=np.uint64) for i in range(level + 1)])
    d = o.modup(c, level)
    ext = o.ext_moduli_idx(level)
    ext_mod = [p.moduli[t] for t in ext]
    c_coeff = coeff_form(o, c, list(range(level + 1)))
    assert d.shape[0] == o.live_digits(level)
    for j in range(d.shape[0]):
        lo, hi = j * o.alpha, min((j + 1) * o.alpha, level + 1)
        Qj = prod(p.moduli[lo:hi])
        dj = coeff_form(o, d[j], ext)
        E = prod(ext_mod)
        seen_u = set()
        for x in range(o.N):
            cx = centred(crt([c_coeff[i, x] for i in range(lo, hi)], p.moduli[lo:hi]), Qj)
            dx = centred(crt(dj[:, x], ext_mod), E)
            u, rem = divmod(dx - cx, Qj)
            assert rem == 0 and 2 * abs(dx) <= (hi - lo) * Qj
            seen_u.add(u)
        assert seen_u <= {-1, 0, 1} and (hi - lo == 1 and seen_u == {0} or hi - lo > 1)
        # the digit's own limbs are untouched
        assert np.array_equal(d[j, lo:hi], c[lo:hi])


@pytest.mark.parametrize("level", [2, 0])
def test_moddown_is_rounded_division_by_P_up_to_small_error(tiny_params, level):
    """u == round(V/P) - e (mod Q_level) with |e| <= k/2: |V - P*u| <= (k+1)*P/2, both signs seen."""
    p = tiny_params
    o = Oracle(p)
    ext = o.ext_moduli_idx(level)
    ext_mod = [p.moduli[t] for t in ext]
    rng = np.random.default_rng(20 + level)
    v = np.stack([rng.integers(0, q, size=o.N, dtype=np.uint64) for q in ext_mod])
    u = o.moddown(v, level)
    P = prod(p.moduli[p.num_q:])
    Q = prod(p.moduli[:level + 1])
    vc = coeff_form(o, v, ext)
    uc = coeff_form(o, u, list(range(level + 1)))
    signs = set()
    for x in range(o.N):
        V = crt(vc[:, x], ext_mod)
        U = crt(uc[:, x], p.moduli[:level + 1])
        U = min((U, U - Q, U + Q), key=lambda t: abs(V - P * t))   # representative nearest to V/P
        assert 2 * abs(V - P * U) <= (p.num_p + 1) * P
        signs.add(V - P * U > 0)
    assert signs == {True, False}


@pytest.mark.parametrize("level", [2, 1])
def test_rescale_is_rounded_division(tiny_params, level):
    p = tiny_params
    o = Oracle(p)
    rng = np.random.default_rng(30 + level)
    ct = np.stack([[rng.integers(0, p.moduli[i], size=o.N, dtype=np.uint64) for i in range(level + 1)] for _ in range(2)])
    out = o.rescale(ct, level)
    ql = p.moduli[level]
    Q = prod(p.moduli[:level + 1])
    for comp in range(2):
        cc = coeff_form(o, ct[comp], list(range(level + 1)))
        oc = coeff_form(o, out[comp], list(range(level)))
        for x in range(o.N):
            c = centred(crt(cc[:, x], p.moduli[:level + 1]), Q)
            want = (2 * c + ql) // (2 * ql)  # round to nearest, q odd: no ties
            for i in range(level):
                assert int(oc[i, x]) == want % p.moduli[i]


def test_switch_key_structure(tiny_params):
    """b_j + a_j s - F_j s' is the small error e_j: |e| <= 19 on every limb, same integer."""
    p = tiny_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(1)
    key = o.gen_relin_key(s_ntt, 2)
    s2 = o.mul(s_ntt, s_ntt, list(range(o.M)))
    P = prod(p.moduli[p.num_q:])
    for j in range(p.dnum):
        lo, hi = j * o.alpha, min((j + 1) * o.alpha, p.num_q)
        errs = []
        for t in range(o.M):
            q = p.moduli[t]
            F = P % q if lo <= t < hi else 0
            r = [(int(b) + int(a) * int(sv) - F * int(s2v)) % q for b, a, sv, s2v in zip(key[j, 0, t], key[j, 1, t], s_ntt[t], s2[t])]
            e = o.ntt_inv(np.array(r, dtype=np.uint64), t)
            errs.append([centred(int(v), q) for v in e])
        assert all(row == errs[0] for row in errs)
        assert max(abs(v) for v in errs[0]) <= 19 and any(errs[0])


def test_splitmix64_indexed_matches_the_sequential_generator():
    """The indexed form against the generator stepped one output at a time in Python integers, and against the first
    outputs for seed 1234567 that implementations of SplitMix64 are commonly checked with."""
    def sequential(seed, n):
        out, x, mask = [], seed, (1 << 64) - 1
        for _ in range(n):
            x = (x + 0x9E3779B97F4A7C15) & mask
            z = x
            z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
            z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
            out.append(z ^ (z >> 31))
        return out
    for seed in (0, 1234567, (1 << 64) - 5):
        got = Oracle.splitmix64_at(seed, np.arange(40)).tolist()
        assert got == sequential(seed, 40)
    assert Oracle.splitmix64_at(1234567, np.arange(5)).tolist() == [
        6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431, 16408922859458223821]


def test_expanded_key_halves_are_uniform_residues(tiny_params):
    """Every value is below its modulus, the first value of a limb is what the definition gives when followed by hand,
    limbs differ from each other, and the top three bits are flat (chi-square over 8 bins, 7 degrees of freedom)."""
    p = make_params(10, 4, 2, 2)
    o = Oracle(p)
    a = o.expand_key_a(99)
    assert a.shape == (o.dnum, o.M, o.N)
    for t in range(o.M):
        assert int(a[:, t].max()) < p.moduli[t]
    j, t, x = 1, 3, 17
    q = p.moduli[t]
    e = (j * o.M + t) * o.N + x
    want = None
    for attempt in range(64):
        v = int(Oracle.splitmix64_at(99, np.array([64 * e + attempt]))[0]) >> (64 - q.bit_length())
        if v < q:
            want = v
            break
    assert int(a[j, t, x]) == want
    assert not np.array_equal(a[0, 0], a[0, 1]) and not np.array_equal(a[0, 0], a[1, 0])
    assert not np.array_equal(a, o.expand_key_a(100))
    top = (a.reshape(-1) >> np.uint64(p.moduli[0].bit_length() - 3)).astype(np.int64)
    counts = np.bincount(top, minlength=8)[:8]
    expect = a.size / 8
    assert ((counts - expect) ** 2 / expect).sum() < 30.0
    # a small modulus makes rejections frequent: values stay exact residues and uniform
    small = Oracle(make_params(4, 2, 1, 1, bits=12))
    b = small.expand_key_a(5)
    assert all(int(b[:, t].max()) < small.moduli[t] for t in range(small.M))


def test_seeded_switch_key_has_the_key_structure_and_switches(tiny_params):
    """b_j + a_j s - F_j sigma_g(s) is a small error with a_j = the expansion of the seed, and a rotation with the seeded
    key decrypts to the rotated slots."""
    p = make_params(10, 4, 2, 2)
    o = Oracle(p)
    s, s_ntt = o.gen_secret(31)
    key = o.gen_rotation_key_seeded(s, s_ntt, 3, 32, a_seed=777)
    assert np.array_equal(key[:, 1], o.expand_key_a(777))
    g = o.galois(3)
    sp = np.zeros(o.N, dtype=np.int64)
    e = (np.arange(o.N, dtype=np.int64) * g) % (2 * o.N)
    sp[e % o.N] = np.where(e < o.N, s, -s)
    sp_ntt = o.lift_ntt(sp, list(range(o.M)))
    P = prod(p.moduli[p.num_q:])
    for j in range(p.dnum):
        lo, hi = j * o.alpha, min((j + 1) * o.alpha, p.num_q)
        for t in (0, o.M - 1, lo):
            q = p.moduli[t]
            F = P % q if lo <= t < hi else 0
            r = [(int(b) + int(a) * int(sv) - F * int(spv)) % q for b, a, sv, spv in zip(key[j, 0, t], key[j, 1, t], s_ntt[t], sp_ntt[t])]
            err = [centred(int(v), q) for v in o.ntt_inv(np.array(r, dtype=np.uint64), t)]
            assert max(abs(v) for v in err) <= 19 and any(err)
    plain = o.gen_rotation_key(s, s_ntt, 3, 32)
    assert not np.array_equal(key[:, 1], plain[:, 1])
    z = np.random.default_rng(33).uniform(-1, 1, o.n)
    level = p.num_q - 1
    ct = o.encrypt(z, 2.0 ** 40, level, s_ntt, 34)
    out = o.rotate(ct, level, 3, key, True)
    assert np.abs(o.decrypt(out, level, s_ntt, 2.0 ** 40) - np.roll(z, -3)).max() < 1e-6


def _noise_bound(o, level, sigma=3.2):
    N = o.N
    beta = o.live_digits(level)
    maxQ = max(prod(o.moduli[j * o.alpha:min((j + 1) * o.alpha, level + 1)]) for j in range(beta))
    P = prod(o.moduli[o.num_q:])
    # key-switch noise: sum_j d_j e_j / P with |d_j| < alpha*Q_j, plus the ModDown rounding by s
    return 8 * (beta * o.alpha * maxQ / P * sigma * N + o.num_p * N)


@pytest.mark.parametrize("level", [3, 2, 0])
def test_keyswitch_preserves_product_with_target_secret(cfg1_params, level):
    """out0 + out1*s == c*s' + small noise (coefficient form, centred)."""
    p = cfg1_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(3)
    key = o.gen_relin_key(s_ntt, 4)  # s' = s^2
    rng = np.random.default_rng(40)
    lim = list(range(level + 1))
    c = np.stack([rng.integers(0, p.moduli[i], size=o.N, dtype=np.uint64) for i in lim])
    out = o.keyswitch(c, key, level)
    sL = s_ntt[:level + 1]
    lhs = o.add(out[0], o.mul(out[1], sL, lim), level)
    rhs = o.mul(c, o.mul(sL, sL, lim), lim)
    diff = coeff_form(o, np.stack([(int(0) + (a.astype(object) - b.astype(object))) % p.moduli[i] for i, (a, b) in enumerate(zip(lhs, rhs))]).astype(np.uint64), lim)
    bound = _noise_bound(o, level)
    for i in lim:
        q = p.moduli[i]
        worst = max(abs(centred(int(v), q)) for v in diff[i])
        assert worst < bound < q / 2 ** 12
    # the noise is one integer polynomial: same centred value on every limb
    if level >= 1:
        assert [centred(int(v), p.moduli[0]) for v in diff[0]] == [centred(int(v), p.moduli[1]) for v in diff[1]]


@pytest.mark.parametrize("offset", [1, -1, 9, 2047, 300])
def test_rotation_is_left_slot_roll_both_orders(cfg1_params, offset):
    p = cfg1_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(5)
    z = np.random.default_rng(50).uniform(-1, 1, o.n)
    scale = 2.0 ** 40
    level = 3
    ct = o.encrypt(z, scale, level, s_ntt, 6)
    key = o.gen_rotation_key(s, s_ntt, offset, 7)
    un = o.rotate(ct, level, offset, key, hoisted=False)
    ho = o.rotate(ct, level, offset, key, hoisted=True)
    want = np.roll(z, -offset)
    du, dh = o.decrypt(un, level, s_ntt, scale), o.decrypt(ho, level, s_ntt, scale)
    assert np.abs(du - want).max() < 1e-5
    assert np.abs(dh - want).max() < 1e-5
    assert np.abs(du - dh).max() < 1e-5
    # centred digits commute with the automorphism's sign flips: the two orders agree exactly
    assert np.array_equal(un, ho)


def test_rotate_there_and_back(cfg1_params):
    p = cfg1_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(8)
    z = np.random.default_rng(51).uniform(-1, 1, o.n)
    ct = o.encrypt(z, 2.0 ** 40, 2, s_ntt, 9)
    k1 = o.gen_rotation_key(s, s_ntt, 17, 10)
    k2 = o.gen_rotation_key(s, s_ntt, -17, 11)
    back = o.rotate(o.rotate(ct, 2, 17, k1, True), 2, -17, k2, False)
    assert np.abs(o.decrypt(back, 2, s_ntt, 2.0 ** 40) - z).max() < 1e-5


def test_rotation_with_wrong_key_fails(cfg1_params):
    """Guards the test above against passing vacuously."""
    p = cfg1_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(8)
    z = np.random.default_rng(52).uniform(-1, 1, o.n)
    ct = o.encrypt(z, 2.0 ** 40, 3, s_ntt, 9)
    k = o.gen_rotation_key(s, s_ntt, 5, 10)
    bad = o.rotate(ct, 3, 4, k, True)
    assert np.abs(o.decrypt(bad, 3, s_ntt, 2.0 ** 40) - np.roll(z, -4)).max() > 1.0


def test_single_special_prime_is_too_noisy():
    """With alpha = 2 digits (~2^100) and one special prime (~2^50) the key-switch noise
    swamps a 2^40 scale: the reason the single-conv workload runs with two special primes."""
    from workloads.params import CONFIGS
    p = CONFIGS["cfg1_single_conv_k1"].params()
    o = Oracle(p)
    s, s_ntt = o.gen_secret(5)
    z = np.random.default_rng(53).uniform(-1, 1, o.n)
    ct = o.encrypt(z, 2.0 ** 40, 3, s_ntt, 6)
    key = o.gen_rotation_key(s, s_ntt, 1, 7)
    out = o.decrypt(o.rotate(ct, 3, 1, key, True), 3, s_ntt, 2.0 ** 40)
    assert np.abs(out - np.roll(z, -1)).max() > 1e3


@pytest.mark.parametrize("level", [3, 1])
def test_ctct_mul_relin_decrypts_to_slot_product(cfg1_params, level):
    p = cfg1_params
    o = Oracle(p)
    s, s_ntt = o.gen_secret(12)
    rlk = o.gen_relin_key(s_ntt, 13)
    rng = np.random.default_rng(60)
    za, zb = rng.uniform(-1, 1, o.n), rng.uniform(-1, 1, o.n)
    scale = 2.0 ** 40
    a = o.encrypt(za, scale, level, s_ntt, 14)
    b = o.encrypt(zb, scale, level, s_ntt, 15)
    prod_ct = o.ctct_mul_relin(a, b, rlk, level)
    assert np.abs(o.decrypt(prod_ct, level, s_ntt, scale * scale) - za * zb).max() < 1e-6
    res = o.rescale(prod_ct, level)
    # after the rescale the scale is only ~2^30, so its rounding (~sqrt(N) at the integer level) shows
    assert np.abs(o.decrypt(res, level - 1, s_ntt, scale * scale / p.moduli[level]) - za * zb).max() < 3e-5
    # x * 1 = x
    one = o.encrypt(np.ones(o.n), scale, level, s_ntt, 16)
    same = o.ctct_mul_relin(a, one, rlk, level)
    assert np.abs(o.decrypt(same, level, s_ntt, scale * scale) - za).max() < 1e-6


def test_ptct_mac_matches_python_integers(tiny_params):
    p = tiny_params
    o = Oracle(p)
    level = 2
    rng = np.random.default_rng(70)
    pts = [np.stack([rng.integers(0, p.moduli[i], size=o.N, dtype=np.uint64) for i in range(level + 1)]) for _ in range(5)]
    cts = [np.stack([[rng.integers(0, p.moduli[i], size=o.N, dtype=np.uint64) for i in range(level + 1)] for _ in range(2)]) for _ in range(5)]
    got = o.ptct_mac(pts, cts, level)
    for comp in range(2):
        for i in range(level + 1):
            q = p.moduli[i]
            want = [sum(int(pt[i, x]) * int(ct[comp, i, x]) for pt, ct in zip(pts, cts)) % q for x in range(o.N)]
            assert got[comp, i].tolist() == want
    # accumulate form: mac(first 2) then mac(last 3, acc) == mac(all)
    part = o.ptct_mac(pts[:2], cts[:2], level)
    assert np.array_equal(o.ptct_mac(pts[2:], cts[2:], level, acc=part), got)


def test_samplers():
    o = Oracle(make_params(12, 1, 0, 1))
    import ctypes as C
    t = np.empty(30000, dtype=np.int8)
    o.lib.orc_sample_ternary(C.c_uint64(1), len(t), t.ctypes.data_as(C.c_void_p))
    assert set(np.unique(t)) == {-1, 0, 1}
    assert all(abs((t == v).mean() - 1 / 3) < 0.01 for v in (-1, 0, 1))
    g = np.empty(200000, dtype=np.int8)
    o.lib.orc_sample_gauss(C.c_uint64(2), len(g), g.ctypes.data_as(C.c_void_p))
    assert abs(g.mean()) < 0.03 and abs(g.std() - np.sqrt(3.2 ** 2 + 1 / 12)) < 0.03 and np.abs(g).max() <= 19
    q = o.moduli[0]
    u = np.empty(100000, dtype=np.uint64)
    o.lib.orc_sample_uniform(C.c_uint64(3), C.c_uint64(q), len(u), u.ctypes.data_as(C.c_void_p))
    assert u.max() < q and abs(u.astype(np.float64).mean() / q - 0.5) < 0.01
    # different seeds give different streams, same seed the same stream
    u2 = np.empty_like(u)
    o.lib.orc_sample_uniform(C.c_uint64(3), C.c_uint64(q), len(u), u2.ctypes.data_as(C.c_void_p))
    assert np.array_equal(u, u2)


# ------------------------------------------------------------------ merged division (ModDown + rescale)
def test_divide_by_limbs_reduces_to_moddown_and_to_rescale(tiny_params):
    """Dropping the special primes is ModDown; dropping q_level is the rescale: same residues as the
    dedicated routines (which have their own big-integer pins)."""
    o = Oracle(tiny_params)
    rng = np.random.default_rng(80)
    level = 2
    ext = o.ext_moduli_idx(level)
    v = np.stack([rng.integers(0, o.moduli[t], o.N, dtype=np.uint64) for t in ext])
    assert np.array_equal(o.divide_by_limbs(v, list(range(level + 1)), list(range(o.num_q, o.M))), o.moddown(v, level))
    ct = np.stack([v[:level + 1], v[:level + 1][::-1].copy() % np.array([[o.moduli[i]] for i in range(level + 1)], dtype=np.uint64)])
    got = np.stack([o.divide_by_limbs(ct[c], list(range(level)), [level]) for c in range(2)])
    assert np.array_equal(got, o.rescale(ct, level))


def test_moddown_rescale_is_the_rounded_quotient(tiny_params):
    """Big-integer pin: the result times P*q_level differs from the input by less than (k+1)/2 * P*q_level
    on every coefficient (CRT over the kept limbs, centred)."""
    o = Oracle(tiny_params)
    rng = np.random.default_rng(81)
    level = 2
    ext = o.ext_moduli_idx(level)
    mods_ext = [o.moduli[t] for t in ext]
    v = np.stack([rng.integers(0, q, o.N, dtype=np.uint64) for q in mods_ext])
    out = o.moddown_rescale(v, level)
    assert out.shape == (level, o.N)
    v_coef = np.stack([o.ntt_inv(v[e], ext[e]) for e in range(len(ext))])
    out_coef = np.stack([o.ntt_inv(out[i], i) for i in range(level)])
    D = o.moduli[level]
    for t in range(o.num_q, o.M):
        D *= o.moduli[t]
    Qkeep = prod(o.moduli[:level])
    Qall = prod(mods_ext)
    for x in range(o.N):
        V = centred(crt([v_coef[e][x] for e in range(len(ext))], mods_ext), Qall)
        U = crt([out_coef[i][x] for i in range(level)], o.moduli[:level])
        # U = round(V / D) modulo Qkeep, up to the conversion error
        err = centred(U * D - V, Qkeep * D)
        assert abs(err) <= (o.num_p + 1) * D // 2 + D, (x, err)
