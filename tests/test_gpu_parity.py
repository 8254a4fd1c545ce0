"""GPU parity: every exported operation, called through the C boundary, against the CPU oracle on
the same seeded inputs -- bit-exact on every residue.  Sizes span several 2^11-point tiles, a
ragged last digit, the lowest level and single-tile / sub-tile rings."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2604_16834_amd as hx  # noqa: E402
from oracle import Oracle, conv2d_reference, activation_reference  # noqa: E402
from workloads import CONFIGS, make_params, image_batch, conv_weights, conv_tap_offsets  # noqa: E402
from gpu_common import rand_poly, rand_ct, w_residues  # noqa: E402


def both(params):
    return Oracle(params), hx.Context(params)


# ------------------------------------------------------------------------------------------ NTT
@pytest.mark.parametrize("log_n,bits", [(4, 20), (7, 30), (10, 50), (11, 50), (12, 50), (13, 50), (16, 50), (17, 50)])
def test_ntt_matches_oracle(log_n, bits):
    p = make_params(log_n, 3, 2, 1, bits=bits)
    orc, ctx = both(p)
    rng = np.random.default_rng(log_n)
    idx = [4, 0, 2, 1]                       # any order of moduli, special primes included
    batch = 3
    polys = np.stack([rand_poly(rng, [p.moduli[t] for t in idx], orc.N) for _ in range(batch)])
    polys[0, 0, :3] = (0, 1, p.moduli[idx[0]] - 1)
    d = hx.from_host(polys)
    hx.ckks_ntt_fwd(ctx, d, idx)
    fwd = hx.to_host(d)
    assert np.array_equal(fwd, orc.ntt_many(polys, idx))
    hx.ckks_ntt_inv(ctx, d, idx)
    assert np.array_equal(hx.to_host(d), polys)
    d = hx.from_host(polys)
    hx.ckks_ntt_inv(ctx, d, idx)
    assert np.array_equal(hx.to_host(d), orc.ntt_many(polys, idx, inverse=True))


@pytest.mark.parametrize("batch,bits", [(1, 50), (8, 50), (9, 50), (19, 50), (19, 57), (64, 50)])
def test_ntt_batches_span_the_item_loop(batch, bits):
    """The forward lo pass gives a workgroup up to eight polynomials of a batch, taken with the stride of the grid's extent
    over items: batches of one item, of exactly eight, of one more, and of 19 and 64 (three and eight workgroups per slice, the
    first with a ragged share) in both arithmetics; every residue against the oracle, forward and back."""
    p = make_params(12, 2, 1, 1, bits=bits)
    orc, ctx = both(p)
    rng = np.random.default_rng(1000 + batch)
    idx = [2, 0]
    polys = np.stack([rand_poly(rng, [p.moduli[t] for t in idx], orc.N) for _ in range(batch)])
    d = hx.from_host(polys)
    hx.ckks_ntt_fwd(ctx, d, idx)
    assert np.array_equal(hx.to_host(d), orc.ntt_many(polys, idx))
    hx.ckks_ntt_inv(ctx, d, idx)
    assert np.array_equal(hx.to_host(d), polys)


def test_ntt_single_limb_single_poly():
    p = make_params(12, 1, 0, 0)
    orc, ctx = both(p)
    a = rand_poly(np.random.default_rng(1), p.moduli, orc.N)
    d = hx.from_host(a)
    hx.ckks_ntt_fwd(ctx, d, [0], batch=1)
    assert np.array_equal(hx.to_host(d)[0], orc.ntt_fwd(a[0], 0))


# --------------------------------------------------------------------------------- key switching
@pytest.fixture(scope="module", params=[50, 57], ids=["q50", "q57"])
def ks_setup(request):
    wl = CONFIGS["small_rotations"]          # N = 2^13, 7 limbs in digits of 3,3,1, 3 special primes
    p = make_params(wl.log_n, wl.num_q, wl.num_p, wl.dnum, bits=request.param)   # 57-bit primes: general kernels
    orc, ctx = both(p)
    s, s_ntt = orc.gen_secret(11)
    rlk = orc.gen_relin_key(s_ntt, 12)
    return p, orc, ctx, s, s_ntt, rlk, hx.ckks_key_load(ctx, hx.from_host(rlk), 0)


@pytest.mark.parametrize("level", [6, 5, 3, 2, 0])
def test_keyswitch_matches_oracle(ks_setup, level):
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    c = rand_poly(np.random.default_rng(20 + level), p.moduli[:level + 1], orc.N)
    out = hx.ckks_keyswitch(ctx, hx.from_host(c), level, d_rlk)
    assert np.array_equal(hx.to_host(out), orc.keyswitch(c, rlk, level))


@pytest.mark.parametrize("level", [6, 4, 0])
@pytest.mark.parametrize("hoisted", [True, False])
def test_rotations_match_oracle(ks_setup, level, hoisted):
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    rng = np.random.default_rng(30 + level)
    z = rng.uniform(-1, 1, orc.n)
    ct = orc.encrypt(z, 2.0 ** 40, level, s_ntt, 31)
    offs = [1, -1, 64, 0, orc.n - 1, 1234, -orc.n]
    keys = [orc.gen_rotation_key(s, s_ntt, r, 40 + i) if r % orc.n else None for i, r in enumerate(offs)]
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(k), hx.ckks_galois_element(ctx, r)) if k is not None else None
             for k, r in zip(keys, offs)]
    outs = hx.ckks_rotate_hoisted(ctx, hx.from_host(ct), level, offs, dkeys, hoisted)
    want = orc.rotate_many(ct, level, offs, keys, hoisted)
    for r, got, w in zip(offs, outs, want):
        got = hx.to_host(got)
        assert np.array_equal(got, w), f"offset {r}"
        assert np.abs(orc.decrypt(got, level, s_ntt, 2.0 ** 40) - np.roll(z, -r)).max() < 1e-5


def test_unhoisted_rotations_batch_to_fit_the_workspace(ks_setup):
    """Unhoisted rotations go through the kernels in batches as large as the workspace holds: the workspace of a
    single rotation (one at a time), of three (batches of 3, 3, 1) and the full one give the oracle's residues."""
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    level = 5
    ct = orc.encrypt(np.random.default_rng(35).uniform(-1, 1, orc.n), 2.0 ** 40, level, s_ntt, 36)
    offs = [3, -2, 17, 0, 900, -77, 5, 2048]
    keys = [orc.gen_rotation_key(s, s_ntt, r, 60 + i) if r % orc.n else None for i, r in enumerate(offs)]
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(k), hx.ckks_galois_element(ctx, r)) if k is not None else None
             for k, r in zip(keys, offs)]
    want = orc.rotate_many(ct, level, offs, keys, False)
    d_ct = hx.from_host(ct)
    for count in (1, 3, len(offs)):
        nbytes = hx.ckks_workspace_bytes(ctx, hx.binding.CKKS_OP_ROTATE, level, count)
        ws = hx.empty((nbytes + 7) // 8)
        outs = hx.ckks_rotate_hoisted(ctx, d_ct, level, offs, dkeys, False, ws=ws)
        for r, got, w in zip(offs, outs, want):
            assert np.array_equal(hx.to_host(got), w), f"workspace for {count}, offset {r}"
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_rotate_hoisted(ctx, d_ct, level, offs, dkeys, False, ws=hx.empty(1024))
    assert e.value.code == hx.binding.CKKS_ERR_WORKSPACE_TOO_SMALL


def test_galois_element_matches_oracle(ks_setup):
    p, orc, ctx, *_ = ks_setup
    for r in (0, 1, -1, 5, orc.n - 1, orc.n, -orc.n - 3, 2 ** 20 + 7):
        assert hx.ckks_galois_element(ctx, r) == orc.galois(r)


# ------------------------------------------------------------------------------------ pointwise
@pytest.mark.parametrize("n_terms", [1, 9, 16, 17, 40])
def test_ptct_mac_matches_oracle(ks_setup, n_terms):
    p, orc, ctx, *_ = ks_setup
    level = 4
    rng = np.random.default_rng(50 + n_terms)
    pts = [rand_poly(rng, p.moduli[:level + 1], orc.N) for _ in range(n_terms)]
    cts = [rand_ct(rng, p.moduli, level, orc.N) for _ in range(n_terms)]
    dp, dc = [hx.from_host(x) for x in pts], [hx.from_host(x) for x in cts]
    acc = hx.ckks_ptct_mac(ctx, dp, dc, level)
    want = orc.ptct_mac(pts, cts, level)
    assert np.array_equal(hx.to_host(acc), want)
    # accumulate on top of an existing accumulator
    acc2 = hx.ckks_ptct_mac(ctx, dp[:1], dc[:1], level, acc=acc, accumulate=True)
    assert np.array_equal(hx.to_host(acc2), orc.ptct_mac(pts[:1], cts[:1], level, acc=want))


@pytest.mark.parametrize("level", [6, 3, 1])
def test_rescale_matches_oracle(ks_setup, level):
    p, orc, ctx, *_ = ks_setup
    ct = rand_ct(np.random.default_rng(60 + level), p.moduli, level, orc.N)
    ct[0, level, :4] = (0, 1, p.moduli[level] // 2, p.moduli[level] // 2 + 1)   # around the centring threshold
    out = hx.ckks_rescale(ctx, hx.from_host(ct), level)
    assert np.array_equal(hx.to_host(out), orc.rescale(ct, level))


@pytest.mark.parametrize("level", [6, 2, 0])
def test_ctct_mul_relin_matches_oracle(ks_setup, level):
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    rng = np.random.default_rng(70 + level)
    a, b = rand_ct(rng, p.moduli, level, orc.N), rand_ct(rng, p.moduli, level, orc.N)
    out = hx.ckks_ctct_mul_relin(ctx, hx.from_host(a), hx.from_host(b), level, d_rlk)
    assert np.array_equal(hx.to_host(out), orc.ctct_mul_relin(a, b, rlk, level))
    da = hx.from_host(a)
    sq = hx.ckks_ctct_mul_relin(ctx, da, da, level, d_rlk)         # squaring: both operands the same buffer
    assert np.array_equal(hx.to_host(sq), orc.ctct_mul_relin(a, a, rlk, level))


@pytest.mark.parametrize("log_n,num_q,num_p,dnum,bits", [(12, 8, 2, 4, 50), (12, 6, 3, 2, 50), (12, 5, 5, 1, 50), (13, 9, 3, 3, 50),
                                                       (12, 8, 2, 4, 56), (11, 6, 3, 2, 50), (12, 6, 2, 6, 50),
                                                       (14, 4, 2, 2, 50), (15, 3, 2, 2, 50), (15, 16, 4, 4, 50)])
def test_key_switch_paths_with_other_digit_shapes(log_n, num_q, num_p, dnum, bits):
    """Four digits of two limbs, two of three, a single digit, three full digits of three, six digits of one limb (more digits
    than the shared multi-rotation launch takes), four digits of four limbs at N = 2^15 (16 target limbs: the converting first
    pass' groups of six with a ragged last group); rings with one to four first-pass stages and the single-pass ring; both
    arithmetic paths: key switch, relinearised product and both rotation modes at the
    top level, at a level with a ragged last digit and at level 0."""
    p = make_params(log_n, num_q, num_p, dnum, bits=bits)
    orc, ctx = both(p)
    s, s_ntt = orc.gen_secret(81)
    rlk = orc.gen_relin_key(s_ntt, 82)
    d_rlk = hx.ckks_key_load(ctx, hx.from_host(rlk), 0)
    offs = [1, -3, 0, 37]
    keys = [orc.gen_rotation_key(s, s_ntt, r, 83 + i) if r else None for i, r in enumerate(offs)]
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(k), hx.ckks_galois_element(ctx, r)) if k is not None else None
             for k, r in zip(keys, offs)]
    alpha = -(-num_q // dnum)
    for level in sorted({num_q - 1, max(0, num_q - 1 - alpha // 2 - 1), 0}, reverse=True):
        rng = np.random.default_rng(90 + level)
        c = rand_poly(rng, p.moduli[:level + 1], orc.N)
        assert np.array_equal(hx.to_host(hx.ckks_keyswitch(ctx, hx.from_host(c), level, d_rlk)), orc.keyswitch(c, rlk, level)), level
        a, b = rand_ct(rng, p.moduli, level, orc.N), rand_ct(rng, p.moduli, level, orc.N)
        got = hx.ckks_ctct_mul_relin(ctx, hx.from_host(a), hx.from_host(b), level, d_rlk)
        assert np.array_equal(hx.to_host(got), orc.ctct_mul_relin(a, b, rlk, level)), level
        for hoisted in (True, False):
            outs = hx.ckks_rotate_hoisted(ctx, hx.from_host(a), level, offs, dkeys, hoisted)
            want = orc.rotate_many(a, level, offs, keys, hoisted)
            for r, o, w in zip(offs, outs, want):
                assert np.array_equal(hx.to_host(o), w), (level, hoisted, r)


# ----------------------------------------------------------------------------------- convolution
def conv_case(name, level=None, bits=50, four_keys=False, deferred=False, merged=False, narrow=False):
    wl = CONFIGS[name]
    p = make_params(wl.log_n, wl.num_q, wl.num_p, wl.dnum, bits=bits)
    orc, ctx = both(p)
    level = p.num_q - 1 if level is None else level
    s, s_ntt = orc.gen_secret(101)
    img = image_batch(wl.batch, wl.c_in, wl.height, wl.width)
    w = conv_weights(wl.c_out, wl.c_in, dist="uniform" if wl.c_in == 1 else "he_normal")
    scale = 2.0 ** 40
    cts = [orc.encrypt(orc.pack_channel(img, c), scale, level, s_ntt, 110 + c) for c in range(wl.c_in)]
    offs = conv_tap_offsets(wl.width)
    keys = {off: orc.gen_rotation_key(s, s_ntt, off, 200 + i) for i, off in enumerate(offs) if off}
    operands = orc.conv_operands_ext if deferred else orc.conv_operands
    masks, w_int = operands(w, wl.height, wl.width, wl.batch, level, 2.0 ** 28, p.moduli[level] / 2.0 ** 28)
    w_moduli = [p.moduli[t] for t in orc.ext_moduli_idx(level)] if deferred else p.moduli
    mode = hx.HE_CONV_DEFERRED_MODDOWN if deferred else (hx.HE_CONV_ALIGN_FOUR_KEYS if four_keys else hx.HE_CONV_ALIGN_DIRECT)
    if merged:
        mode = hx.HE_CONV_DEFERRED_MERGED
    if four_keys:                                 # only the keys of -1, +1, -W, +W exist
        keys = {off: k for off, k in keys.items() if off in (-1, 1, -wl.width, wl.width)}
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(keys[off]), hx.ckks_galois_element(ctx, off)) if off in keys else None for off in offs]
    wb = hx.conv_weight_bits(w_int) if narrow else 0         # the bound on the integer weights, stated or not
    assert not narrow or wb <= 24
    outs = hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, [hx.from_host(c) for c in cts], dkeys,
                              hx.from_host(masks), hx.from_host(w_residues(w_int, w_moduli, len(w_moduli) - 1 if deferred else level)),
                              wl.c_out, alignment=mode, weight_bits=wb)
    return wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, [hx.to_host(o) for o in outs]


@pytest.mark.parametrize("name,level,bits", [("cfg1_single_conv", None, 50), ("cfg1_single_conv_k1", None, 50), ("small_conv", None, 50),
                                             ("small_conv", 2, 50), ("small_conv", None, 56), ("small_conv", None, 36),
                                             ("small_conv_d6", None, 50), ("tiny_ring_conv", None, 50)])
def test_he_conv_matches_oracle_and_float_conv(name, level, bits):
    # 56-bit primes take the general 128-bit accumulation kernels, <= 50-bit ones the carry-free split ones
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case(name, level, bits)
    want = orc.he_conv(cts, level, wl.width, keys, masks, w_int)
    ref = conv2d_reference(img, w)
    for o in range(wl.c_out):
        assert np.array_equal(outs[o], want[o]), f"output channel {o}"
        if name.endswith("_k1") or bits < 50:
            continue    # one special prime for 2-limb digits / 36-bit primes under a 2^40 scale: limb parity only
        dec = orc.unpack_channel(orc.decrypt(outs[o], level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(dec - ref[:, o]).max() < 1e-4


@pytest.mark.parametrize("name,deferred,merged", [("cfg1_single_conv", False, False), ("small_conv", False, False),
                                                  ("small_conv", True, False), ("small_conv", True, True)])
def test_he_conv_with_stated_weight_bound_matches_oracle(name, deferred, merged):
    """The weights are integers of at most 23 bits: with that bound stated the multiply-accumulate writes them in
    three signed digits instead of seven (negative ones through their centred representative): same residues."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case(name, deferred=deferred, merged=merged, narrow=True)
    assert (w_int < 0).any() and (w_int > 0).any()
    want = orc.he_conv_deferred(cts, level, wl.width, keys, masks, w_int, merged=merged) if deferred \
        else orc.he_conv(cts, level, wl.width, keys, masks, w_int)
    for o in range(wl.c_out):
        assert np.array_equal(outs[o], want[o]), f"output channel {o}"


@pytest.mark.parametrize("name,level,bits", [("cfg1_single_conv", None, 50), ("small_conv", None, 50), ("small_conv", 3, 56)])
def test_he_conv_four_key_alignment_matches_oracle(name, level, bits):
    """The paper's two-stage input alignment with four rotation keys (Eqs. 8-10): same residues as the
    oracle's four-key schedule, same slots as the float64 convolution."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case(name, level, bits, four_keys=True)
    assert len(keys) == 4
    want = orc.he_conv(cts, level, wl.width, keys, masks, w_int, four_keys=True)
    ref = conv2d_reference(img, w)
    for o in range(wl.c_out):
        assert np.array_equal(outs[o], want[o]), f"output channel {o}"
        dec = orc.unpack_channel(orc.decrypt(outs[o], level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(dec - ref[:, o]).max() < 1e-4


@pytest.mark.parametrize("name,level,bits", [("cfg1_single_conv", None, 50), ("small_conv", None, 50), ("small_conv", 2, 50),
                                             ("small_conv", 3, 56)])
def test_he_conv_deferred_moddown_matches_oracle(name, level, bits):
    """One division by P per output channel, after the sum on the extended basis: same residues as the
    oracle's deferred schedule, same slots as the float64 convolution."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case(name, level, bits, deferred=True)
    want = orc.he_conv_deferred(cts, level, wl.width, keys, masks, w_int)
    ref = conv2d_reference(img, w)
    for o in range(wl.c_out):
        assert np.array_equal(outs[o], want[o]), f"output channel {o}"
        dec = orc.unpack_channel(orc.decrypt(outs[o], level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(dec - ref[:, o]).max() < 1e-4


@pytest.mark.parametrize("name,level,bits", [("cfg1_single_conv", None, 50), ("small_conv", None, 50), ("small_conv", 1, 50),
                                             ("small_conv", 3, 56), ("small_conv_d6", None, 50), ("small_conv_d6", 3, 50),
                                             ("tiny_ring_conv", None, 50)])
def test_he_conv_deferred_merged_division_matches_oracle(name, level, bits):
    """The deferred schedule with ModDown and rescale of every sum as one division by P*q_level."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case(name, level, bits, deferred=True, merged=True)
    want = orc.he_conv_deferred(cts, level, wl.width, keys, masks, w_int, merged=True)
    ref = conv2d_reference(img, w)
    for o in range(wl.c_out):
        assert np.array_equal(outs[o], want[o]), f"output channel {o}"
        dec = orc.unpack_channel(orc.decrypt(outs[o], level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(dec - ref[:, o]).max() < 1e-4


@pytest.mark.parametrize("mask_bits", [28, 20], ids=["w24", "w32"])
def test_he_conv_64_input_channels_in_the_timed_schedule(mask_bits):
    """64 -> 40 channels: 576 terms, the multiply-accumulate's regular instantiation (whole 64-term blocks, term-innermost
    operand layout, both output tiles, nine blocks through the double-buffered pipeline) in the deferred schedule with the
    merged division, as the block-slice benchmark runs it: every residue of every output against the oracle, with the
    weight bound stated (three signed digits for the 2^28 mask scale, four for 2^20) and without it (seven)."""
    wl = CONFIGS["small_conv_c64"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(901)
    img = image_batch(wl.batch, wl.c_in, wl.height, wl.width)
    w = conv_weights(wl.c_out, wl.c_in)
    scale = 2.0 ** 40
    cts = [orc.encrypt(orc.pack_channel(img, c), scale, level, s_ntt, 910 + c) for c in range(wl.c_in)]
    offs = conv_tap_offsets(wl.width)
    keys = {off: orc.gen_rotation_key(s, s_ntt, off, 990 + i) for i, off in enumerate(offs) if off}
    masks, w_int = orc.conv_operands_ext(w, wl.height, wl.width, wl.batch, level, 2.0 ** mask_bits, p.moduli[level] / 2.0 ** mask_bits)
    wb = hx.conv_weight_bits(w_int)
    assert (16 < wb <= 24) if mask_bits == 28 else (24 < wb <= 32), wb
    ext_moduli = [p.moduli[t] for t in orc.ext_moduli_idx(level)]
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(keys[off]), hx.ckks_galois_element(ctx, off)) if off else None for off in offs]
    d_cts = [hx.from_host(c) for c in cts]
    d_masks, d_w = hx.from_host(masks), hx.from_host(w_residues(w_int, ext_moduli, len(ext_moduli) - 1))
    want = orc.he_conv_deferred(cts, level, wl.width, keys, masks, w_int, merged=True)
    ref = conv2d_reference(img, w)
    for bits in (wb, 0):
        outs = hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, d_cts, dkeys, d_masks, d_w, wl.c_out,
                                  alignment=hx.HE_CONV_DEFERRED_MERGED, weight_bits=bits, w_int_host=w_int, check_weights=True)
        for o in range(wl.c_out):
            got = hx.to_host(outs[o])
            assert np.array_equal(got, want[o]), f"output channel {o}, weight_bits {bits}"
            dec = orc.unpack_channel(orc.decrypt(got, level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
            assert np.abs(dec - ref[:, o]).max() < 1e-4


def test_weight_bound_is_checked_when_asked():
    """A weight beyond the stated bound is rejected by the host check (integer weights given) and by the device check
    (residues only), instead of silently giving wrong residues; weights inside the bound, negative ones included, pass."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case("small_conv", deferred=True, merged=True, narrow=True)
    ctx = hx.Context(p)
    ext_moduli = [p.moduli[t] for t in orc.ext_moduli_idx(level)]
    wb = hx.conv_weight_bits(w_int)
    d_w = hx.from_host(w_residues(w_int, ext_moduli, len(ext_moduli) - 1))
    hx.he_conv_check_weights(ctx, wl.c_in, wl.c_out, level, d_w, wb, hx.HE_CONV_DEFERRED_MERGED)
    hx.he_conv_check_weights(ctx, wl.c_in, wl.c_out, level, d_w, 0, hx.HE_CONV_DEFERRED_MERGED)      # no promise: nothing to test
    with pytest.raises(hx.CkksError) as e:
        hx.he_conv_check_weights(ctx, wl.c_in, wl.c_out, level, d_w, wb - 1, hx.HE_CONV_DEFERRED_MERGED)
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG
    for bad_value in (1 << (wb - 1), -(1 << (wb - 1))):      # the first magnitudes outside |w| < 2^(wb-1), either sign
        w_bad = w_int.copy()
        w_bad[1, 2, 5] = bad_value
        d_bad = hx.from_host(w_residues(w_bad, ext_moduli, len(ext_moduli) - 1))
        with pytest.raises(hx.CkksError) as e:
            hx.he_conv_check_weights(ctx, wl.c_in, wl.c_out, level, d_bad, wb, hx.HE_CONV_DEFERRED_MERGED)
        assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG and "weight residues" in str(e.value)
        offs = conv_tap_offsets(wl.width)
        dkeys = [hx.ckks_key_load(ctx, hx.from_host(keys[off]), hx.ckks_galois_element(ctx, off)) if off else None for off in offs]
        args = (ctx, wl.height, wl.width, wl.batch, level, [hx.from_host(c) for c in cts], dkeys, hx.from_host(masks), d_bad, wl.c_out)
        with pytest.raises(ValueError):
            hx.he_conv_batched(*args, alignment=hx.HE_CONV_DEFERRED_MERGED, weight_bits=wb, w_int_host=w_bad)
        with pytest.raises(hx.CkksError):
            hx.he_conv_batched(*args, alignment=hx.HE_CONV_DEFERRED_MERGED, weight_bits=wb, check_weights=True)
    w_edge = w_int.copy()
    w_edge[0, 0, 0], w_edge[0, 0, 1] = (1 << (wb - 1)) - 1, -((1 << (wb - 1)) - 1)                   # the largest admitted magnitudes
    hx.he_conv_check_weights(ctx, wl.c_in, wl.c_out, level, hx.from_host(w_residues(w_edge, ext_moduli, len(ext_moduli) - 1)), wb,
                             hx.HE_CONV_DEFERRED_MERGED)


def test_he_conv_deferred_needs_extended_operands():
    wl = CONFIGS["cfg1_single_conv"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    ct = hx.from_host(rand_ct(np.random.default_rng(2), p.moduli, level, orc.N))
    with pytest.raises(ValueError):          # masks on the q-limbs only
        hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, [ct], [None] * 9, hx.empty(9, level + 1, orc.N),
                           hx.empty(1, 1, 9, level + 1), 1, alignment=hx.HE_CONV_DEFERRED_MODDOWN)
    with pytest.raises(hx.CkksError) as e:
        hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, [ct], [None] * 9, hx.empty(9, level + 1, orc.N),
                           hx.empty(1, 1, 9, level + 1), 1, alignment=7)
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG


def test_he_conv_four_keys_rejects_a_missing_key():
    wl = CONFIGS["cfg1_single_conv"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    ct = hx.from_host(rand_ct(np.random.default_rng(2), p.moduli, level, orc.N))
    with pytest.raises(hx.CkksError) as e:
        hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, [ct], [None] * 9, hx.empty(9, level + 1, orc.N),
                           hx.empty(1, 1, 9, level + 1), 1, alignment=hx.HE_CONV_ALIGN_FOUR_KEYS)
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY


def test_he_conv_equals_composition_of_exported_ops():
    """he_conv_batched == rotate_hoisted + ptct_mac (with materialised weight plaintexts) + rescale,
    all on the GPU: the factored weights are an exact identity."""
    wl, p, orc, level, s_ntt, img, w, scale, cts, keys, masks, w_int, outs = conv_case("small_conv")
    ctx = hx.Context(p)
    offs = conv_tap_offsets(wl.width)
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(keys[off]), hx.ckks_galois_element(ctx, off)) if off else None for off in offs]
    aligned = [hx.ckks_rotate_hoisted(ctx, hx.from_host(c), level, offs, dkeys, True) for c in cts]
    for o in range(wl.c_out):
        pts, terms = [], []
        for c in range(wl.c_in):
            for t in range(9):
                pts.append(hx.from_host(orc.scalar_mul(masks[t], orc.scalar_residues(int(w_int[o, c, t]), level), level)))
                terms.append(aligned[c][t])
        acc = hx.ckks_ptct_mac(ctx, pts, terms, level)
        assert np.array_equal(hx.to_host(hx.ckks_rescale(ctx, acc, level)), outs[o])


# ----------------------------------------------------------------------------------- accumulator
@pytest.mark.parametrize("g,level", [(4, 4), (2, 2), (1, 3), (10, 4)])
def test_accumulator_merge_matches_oracle(g, level):
    """Cleaned blocks side by side: residues against the oracle, slots against the concatenation.
    g = 10 takes two batches of rotations; g = 1 is mask-and-rescale."""
    p = CONFIGS["small_conv"].params()
    orc, ctx = both(p)
    s, s_ntt = orc.gen_secret(401)
    sts = orc.n // 16 if g > 4 else orc.n // 4
    rng = np.random.default_rng(402 + g)
    zs = [rng.uniform(-1, 1, orc.n) for _ in range(g)]
    scale = 2.0 ** 40
    cts = [orc.encrypt(z, scale, level, s_ntt, 410 + i) for i, z in enumerate(zs)]
    M = orc.encode_ntt(orc.cleaning_mask(sts), float(p.moduli[level]), level)
    keys = {-i * sts: orc.gen_rotation_key(s, s_ntt, -i * sts, 430 + i) for i in range(1, g)}
    dkeys = [None] + [hx.ckks_key_load(ctx, hx.from_host(keys[-i * sts]), hx.ckks_galois_element(ctx, -i * sts)) for i in range(1, g)]
    out = hx.to_host(hx.he_accumulator_merge(ctx, [hx.from_host(c) for c in cts], level, sts, hx.from_host(M), dkeys))
    assert np.array_equal(out, orc.accumulator_merge(cts, level, sts, M, keys))
    want = np.zeros(orc.n)
    want[:g * sts] = np.concatenate([z[:sts] for z in zs])
    assert np.abs(orc.decrypt(out, level - 1, s_ntt, scale) - want).max() < 1e-5


def test_accumulator_merge_rejects_overfull_and_wrong_keys():
    p = CONFIGS["small_conv"].params()
    orc, ctx = both(p)
    level = 2
    ct = hx.from_host(rand_ct(np.random.default_rng(3), p.moduli, level, orc.N))
    mask = hx.empty(level + 1, orc.N)
    with pytest.raises(hx.CkksError) as e:                 # 3 blocks of n/2 slots do not fit
        hx.he_accumulator_merge(ctx, [ct] * 3, level, orc.n // 2, mask, [None] * 3)
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG
    with pytest.raises(hx.CkksError) as e:
        hx.he_accumulator_merge(ctx, [ct] * 2, level, orc.n // 2, mask, [None, None])
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY


# ------------------------------------------------------------------------------ fully connected
def fc_case(d_in, d_out, batch, base, log_n=10, seed=500):
    p = make_params(log_n, 6, 2, 3)
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(seed)
    rng = np.random.default_rng(seed + 1)
    W = rng.normal(0, 0.3, (d_out, d_in))
    bias = rng.uniform(-0.5, 0.5, d_out)
    X = rng.uniform(-1, 1, (batch, d_in))
    z = np.zeros(orc.n)
    z[:batch * d_in] = X.reshape(-1)
    scale = 2.0 ** 40
    ct = orc.encrypt(z, scale, level, s_ntt, seed + 2)
    delta, lo, hi = orc.fc_shifts(d_in, d_out, batch, base)
    sums = [2 ** t for t in range(d_in.bit_length() - 1)]
    merges = [-i for i in range(d_out)]
    offsets = sorted({r for r in sums + merges + lo + hi if r % orc.n})
    keys = {r: orc.gen_rotation_key(s, s_ntt, r, seed + 10 + k) for k, r in enumerate(offsets)}
    dkeys = {r: hx.ckks_key_load(ctx, hx.from_host(k), hx.ckks_galois_element(ctx, r)) for r, k in keys.items()}
    ops = orc.fc_operands(W, bias, batch, level, base, scale)
    want = orc.fc_batched(ct, level, d_in, d_out, batch, base, *ops, keys)
    w_enc, merge_mask, place, bias_pt = [hx.from_host(a) for a in ops]
    pick = lambda offs: [dkeys.get(r) for r in offs]
    run = lambda **kw: hx.he_fc_batched(ctx, hx.from_host(ct), level, d_in, d_out, batch, base, w_enc, merge_mask, place, bias_pt,
                                        pick(sums), pick(merges), pick(lo), pick(hi), **kw)
    return dict(orc=orc, ctx=ctx, level=level, s_ntt=s_ntt, scale=scale, X=X, W=W, bias=bias, want=want, run=run, dkeys=dkeys,
                args=(sums, merges, lo, hi))


@pytest.mark.parametrize("d_in,d_out,batch,base", [(16, 4, 8, 3), (8, 8, 4, 2), (32, 10, 16, 4), (64, 10, 8, 1), (16, 1, 5, 8),
                                                   (8, 2, 40, 2), (8, 2, 40, 20)])
def test_fc_batched_matches_oracle(d_in, d_out, batch, base):
    """Residues against the oracle and slots against W x + b: ragged base blocks (8 = 3+3+2), d_out = d_in (no layout
    rotation), ten outputs (two batches of merge rotations), base 1 (only second rotations), base > batch (only first
    rotations), one output (no merge rotation), 20 second rotations (three batches, a final sum in two launches),
    20 first rotations (three batches)."""
    k = fc_case(d_in, d_out, batch, base)
    orc, level = k["orc"], k["level"]
    got = hx.to_host(k["run"]())
    assert got.shape == (2, level - 2, orc.N)
    assert np.array_equal(got, k["want"])
    dec = orc.decrypt(got, level - 3, k["s_ntt"], k["scale"])
    want = (k["X"] @ k["W"].T + k["bias"]).reshape(-1)
    assert np.abs(dec[:batch * d_out] - want).max() < 1e-4
    assert np.abs(dec[batch * d_out:]).max() < 1e-4


def test_fc_batched_spans_tiles_and_reuses_its_workspace():
    """N = 2^12 (several tiles of every kernel), the classifier's 64 -> 10 shape, twice in the same workspace."""
    d_in, d_out, batch, base = 64, 10, 32, 6
    k = fc_case(d_in, d_out, batch, base, log_n=12, seed=540)
    ctx, level = k["ctx"], k["level"]
    ws = hx.empty(hx.he_fc_workspace_bytes(ctx, d_in, d_out, batch, level, base) // 8)
    ws.fill_(-1)
    a = hx.to_host(k["run"](ws=ws))
    b = hx.to_host(k["run"](ws=ws))
    assert np.array_equal(a, k["want"]) and np.array_equal(b, k["want"])


def test_fc_batched_rejects_bad_shapes_and_keys():
    k = fc_case(16, 4, 8, 3)
    ctx, level, orc = k["ctx"], k["level"], k["orc"]
    sums, merges, lo, hi = k["args"]
    ct = hx.empty(2, level + 1, orc.N)
    w = hx.empty(4, level + 1, orc.N)
    mm, pm, b = hx.empty(level, orc.N), hx.empty(8, level - 1, orc.N), hx.empty(level - 2, orc.N)
    pick = lambda offs: [k["dkeys"].get(r) for r in offs]
    good = [pick(sums), pick(merges), pick(lo), pick(hi)]
    for i in range(4):                                        # a missing or mismatched key in each list
        lists = [list(x) for x in good]
        lists[i][-1] = None if i else lists[i][0]
        with pytest.raises(hx.CkksError) as e:
            hx.he_fc_batched(ctx, ct, level, 16, 4, 8, 3, w, mm, pm, b, *lists)
        assert e.value.code == hx.binding.CKKS_ERR_NO_KEY
    with pytest.raises(hx.CkksError) as e:                    # d_in not a power of two
        hx.he_fc_batched(ctx, ct, level, 12, 4, 8, 3, w, mm, pm, b, pick(sums)[:3], pick(merges), pick(lo), pick(hi))
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG
    with pytest.raises(hx.CkksError) as e:                    # too small a workspace
        hx.he_fc_batched(ctx, ct, level, 16, 4, 8, 3, w, mm, pm, b, *good, ws=hx.empty(1024))
    assert e.value.code == hx.binding.CKKS_ERR_WORKSPACE_TOO_SMALL


def test_overlap_switch_gives_identical_results():
    """Twenty channels (three batches, two of them in flight at a time on the context's two streams) through the
    activation with the overlap on and off, repeatedly into the same outputs: every result equals the oracle's."""
    wl = CONFIGS["small_block"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(901)
    rlk = orc.gen_relin_key(s_ntt, 902)
    d_rlk = hx.ckks_key_load(ctx, hx.from_host(rlk), 0)
    rng = np.random.default_rng(903)
    plan = orc.act_schedule(level, 2.0 ** 50)
    cts = [orc.encrypt(rng.uniform(-1, 1, orc.n), 2.0 ** 50, level, s_ntt, 904 + i) for i in range(20)]
    want = [orc.poly_activation_merged(ct, level, plan["k"], rlk) for ct in cts[:3]] + [None] * 17
    want[8], want[19] = (orc.poly_activation_merged(cts[i], level, plan["k"], rlk) for i in (8, 19))
    dx = [hx.from_host(ct) for ct in cts]
    outs = None
    for on in (True, False, True, True):
        hx.ckks_ctx_set_overlap(ctx, on)
        outs = hx.he_poly_act_deg7(ctx, dx, level, plan["k"], d_rlk, outs=outs, merged=True)
        got = [hx.to_host(o) for o in outs]
        for i, w in enumerate(want):
            if w is not None:
                assert np.array_equal(got[i], w), f"overlap {on}, channel {i}"
        if on is False:
            ref = got
    for a, b in zip(got, ref):
        assert np.array_equal(a, b)


def test_two_stream_activation_replays_from_a_graph():
    """The activation of 20 channels (both of the context's streams in use) captured into a HIP graph: every replay,
    with eager work and a synchronisation in between, gives the eager (oracle-checked) result."""
    import torch
    wl = CONFIGS["small_block"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(911)
    rlk = orc.gen_relin_key(s_ntt, 912)
    d_rlk = hx.ckks_key_load(ctx, hx.from_host(rlk), 0)
    rng = np.random.default_rng(913)
    plan = orc.act_schedule(level, 2.0 ** 50)
    cts = [orc.encrypt(rng.uniform(-1, 1, orc.n), 2.0 ** 50, level, s_ntt, 914 + i) for i in range(20)]
    dx = [hx.from_host(ct) for ct in cts]
    outs = [hx.empty(2, level - 3, orc.N) for _ in cts]
    ws = hx.empty(hx.ckks_workspace_bytes(ctx, hx.binding.CKKS_OP_POLY_ACT, level, len(cts)) // 8 + 1)
    st = torch.cuda.Stream()
    run = lambda: hx.he_poly_act_deg7(ctx, dx, level, plan["k"], d_rlk, outs=outs, ws=ws, merged=True, stream=st.cuda_stream)
    with torch.cuda.stream(st):
        run()
        st.synchronize()
        ref = [o.clone() for o in outs]
        for i in (0, 9, 19):
            assert np.array_equal(hx.to_host(ref[i]), orc.poly_activation_merged(cts[i], level, plan["k"], rlk))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            run()
        for _ in range(3):
            for o in outs:
                o.zero_()
            torch.randn(1 << 16, device="cuda").sum().item()      # eager work and a synchronisation between replays
            graph.replay()
            torch.cuda.synchronize()
            assert all(torch.equal(a, b) for a, b in zip(outs, ref))


def test_deferred_convolution_replays_from_a_graph():
    """The convolution (deferred, merged division: fused taps, matrix-core sum, conversions and division inside the
    transforms) captured into a HIP graph: every replay gives the eager, oracle-checked result."""
    import torch
    wl = CONFIGS["small_conv"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(921)
    img = image_batch(wl.batch, wl.c_in, wl.height, wl.width)
    w = conv_weights(wl.c_out, wl.c_in, dist="he_normal")
    cts = [orc.encrypt(orc.pack_channel(img, c), 2.0 ** 40, level, s_ntt, 922 + c) for c in range(wl.c_in)]
    offs = conv_tap_offsets(wl.width)
    keys = {off: orc.gen_rotation_key(s, s_ntt, off, 930 + i) for i, off in enumerate(offs) if off}
    masks, w_int = orc.conv_operands_ext(w, wl.height, wl.width, wl.batch, level, 2.0 ** 28, p.moduli[level] / 2.0 ** 28)
    w_moduli = [p.moduli[t] for t in orc.ext_moduli_idx(level)]
    dkeys = [hx.ckks_key_load(ctx, hx.from_host(keys[off]), hx.ckks_galois_element(ctx, off)) if off in keys else None for off in offs]
    d_in = [hx.from_host(c) for c in cts]
    d_masks, d_w = hx.from_host(masks), hx.from_host(w_residues(w_int, w_moduli, len(w_moduli) - 1))
    outs = [hx.empty(2, level, orc.N) for _ in range(wl.c_out)]
    mode = hx.HE_CONV_DEFERRED_MERGED
    ws = hx.empty(hx.he_conv_workspace_bytes(ctx, wl.c_in, wl.c_out, wl.height, wl.width, wl.batch, level, mode) // 8 + 1)
    st = torch.cuda.Stream()
    run = lambda: hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, d_in, dkeys, d_masks, d_w, wl.c_out, outs=outs, ws=ws,
                                     alignment=mode, stream=st.cuda_stream)
    with torch.cuda.stream(st):
        run()
        st.synchronize()
        ref = [o.clone() for o in outs]
        want = orc.he_conv_deferred(cts, level, wl.width, keys, masks, w_int, merged=True)
        for o in range(wl.c_out):
            assert np.array_equal(hx.to_host(ref[o]), want[o])
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            run()
        for _ in range(3):
            for o in outs:
                o.zero_()
            ws.zero_()
            torch.randn(1 << 16, device="cuda").sum().item()      # eager work and a synchronisation between replays
            graph.replay()
            torch.cuda.synchronize()
            assert all(torch.equal(a, b) for a, b in zip(outs, ref))


# --------------------------------------------------------------------------------- staged keys
@pytest.mark.parametrize("log_n,num_q,num_p,dnum,bits", [(12, 4, 2, 2, 50), (10, 3, 1, 3, 57), (5, 3, 1, 2, 12)])
def test_key_expansion_matches_oracle(log_n, num_q, num_p, dnum, bits):
    """The public halves written on the device from a seed equal the oracle's expansion; the b halves are not touched.
    50- and 57-bit moduli, and 12-bit ones where rejections are frequent."""
    p = make_params(log_n, num_q, num_p, dnum, bits=bits)
    orc, ctx = both(p)
    rng = np.random.default_rng(800)
    key = rng.integers(0, 1 << 40, (dnum, 2, orc.M, orc.N), dtype=np.uint64)
    for seed in (0, 777, (1 << 64) - 3):
        d = hx.ckks_key_expand_a(ctx, seed, hx.from_host(key))
        got = hx.to_host(d).reshape(key.shape)
        assert np.array_equal(got[:, 1], orc.expand_key_a(seed))
        assert np.array_equal(got[:, 0], key[:, 0])


def test_staged_keys_equal_the_oracle_keys_and_rotate():
    """Two seeded rotation keys staged from pinned host memory on a side stream (b halves copied, a halves expanded):
    the device keys equal the oracle's keys word for word and a hoisted rotation with them matches the oracle."""
    import torch
    p = CONFIGS["small_rotations"].params()
    orc, ctx = both(p)
    s, s_ntt = orc.gen_secret(810)
    offs, seeds = [5, -3], [9001, 9002]
    keys = [orc.gen_rotation_key_seeded(s, s_ntt, r, 811 + i, a_seed=seeds[i]) for i, r in enumerate(offs)]
    host_b = [torch.from_numpy(np.ascontiguousarray(k[:, 0]).view(np.int64)).pin_memory() for k in keys]
    dev = [hx.empty(p.dnum, 2, orc.M, orc.N).fill_(-1) for _ in keys]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())           # the fill above runs on the current stream
    hx.ckks_keyset_stage(ctx, host_b, seeds, dev, stream=side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for k, d in zip(keys, dev):
        assert np.array_equal(hx.to_host(d).reshape(k.shape), k)
    level = p.num_q - 1
    ct = rand_ct(np.random.default_rng(812), p.moduli, level, orc.N)
    dk = [hx.ckks_key_load(ctx, d, hx.ckks_galois_element(ctx, r)) for d, r in zip(dev, offs)]
    outs = hx.ckks_rotate_hoisted(ctx, hx.from_host(ct), level, offs, dk, hoisted=True)
    for o, w in zip(outs, orc.rotate_many(ct, level, offs, keys, True)):
        assert np.array_equal(hx.to_host(o), w)
    with pytest.raises(ValueError):
        hx.ckks_keyset_stage(ctx, host_b[:1], seeds, dev)


# ------------------------------------------------------------------- down-sampling compaction
def run_downsample(orc, ctx, s, s_ntt, cts, level, plan, seed, deferred=False):
    """Both stages of the plan on the GPU (channel vector at once) and in the oracle (one by one); returns (got, want)."""
    offs = sorted({r for lo, hi, _ in plan for r in list(lo) + list(hi) if r % orc.n})
    keys = {r: orc.gen_rotation_key(s, s_ntt, r, seed + k) for k, r in enumerate(offs)}
    dkeys = {r: hx.ckks_key_load(ctx, hx.from_host(k), hx.ckks_galois_element(ctx, r)) for r, k in keys.items()}
    cur = [hx.from_host(ct) for ct in cts]
    want = [ct for ct in cts]
    for stage, (lo, hi, slot_masks) in enumerate(plan):
        lv = level - stage
        if deferred:
            ext = orc.ext_moduli_idx(lv)
            enc = [[None if m is None else orc.lift_ntt(orc.encode(m, float(orc.moduli[lv])), ext) for m in row] for row in slot_masks]
        else:
            enc = [[None if m is None else orc.encode_ntt(m, float(orc.moduli[lv]), lv) for m in row] for row in slot_masks]
        cur = hx.he_relayout_two_rotations(ctx, cur, lv, lo, [dkeys.get(r) for r in lo], hi, [dkeys.get(r) for r in hi],
                                           [[None if m is None else hx.from_host(m) for m in row] for row in enc],
                                           schedule=hx.HE_RELAYOUT_DEFERRED if deferred else hx.HE_RELAYOUT_DIRECT)
        ref = orc.relayout_two_rotations_deferred if deferred else orc.relayout_two_rotations
        want = [ref(ct, lv, lo, hi, enc, keys) for ct in want]
        for b in range(len(cts)):
            assert np.array_equal(hx.to_host(cur[b]), want[b]), f"stage {stage}, ciphertext {b}"
    return [hx.to_host(t) for t in cur], want


@pytest.mark.parametrize("height,width,batch,r,base,n_ct", [(4, 4, 8, 2, 3, 1), (4, 8, 5, 2, 0, 3), (8, 8, 2, 4, 1, 2), (2, 2, 20, 2, 20, 10)])
def test_downsample_compaction_matches_oracle(height, width, batch, r, base, n_ct):
    """Stride-r slot compaction of a channel vector: residues of both stages against the oracle, slots against numpy
    slicing.  One ciphertext (first rotations batched over offsets), three (two offsets per batch), ten (two channel
    batches; 20 first rotations and a single second one), stride 4, base 1 (only second rotations in stage B)."""
    p = make_params(10, 5, 2, 3)
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(600)
    rng = np.random.default_rng(601)
    scale = 2.0 ** 40
    X = rng.uniform(-1, 1, (n_ct, batch, height, width))
    cts = []
    for c in range(n_ct):
        z = rng.uniform(-1, 1, orc.n)                       # junk behind the images
        z[:batch * height * width] = X[c].reshape(-1)
        cts.append(orc.encrypt(z, scale, level, s_ntt, 610 + c))
    plan = orc.downsample_plan(height, width, batch, r, base)
    got, _ = run_downsample(orc, ctx, s, s_ntt, cts, level, plan, 650)
    for c in range(n_ct):
        dec = orc.decrypt(got[c], level - 2, s_ntt, scale)
        want = X[c][:, ::r, ::r].reshape(-1)
        assert np.abs(dec[:want.size] - want).max() < 1e-5 and np.abs(dec[want.size:]).max() < 1e-5


@pytest.mark.parametrize("height,width,batch,r,base,group,n_ct", [(4, 4, 8, 2, 3, 1, 1), (4, 8, 5, 2, 5, 2, 3), (8, 8, 2, 2, 1, 4, 10),
                                                                  (2, 2, 40, 2, 2, 1, 2)])
def test_downsample_compaction_deferred_matches_oracle(height, width, batch, r, base, group, n_ct):
    """The schedule with the divisions by P after the sums: residues of both stages against the oracle's deferred
    re-layout, slots against numpy slicing.  Several rows per group (16 first rotations, no second one inside the
    images), base = batch (only first rotations over the images), 20 second rotations (summed in two launches),
    ten ciphertexts (two channel batches)."""
    p = make_params(10, 5, 2, 3)
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(620)
    rng = np.random.default_rng(621)
    scale = 2.0 ** 40
    X = rng.uniform(-1, 1, (n_ct, batch, height, width))
    cts = []
    for c in range(n_ct):
        z = rng.uniform(-1, 1, orc.n)
        z[:batch * height * width] = X[c].reshape(-1)
        cts.append(orc.encrypt(z, scale, level, s_ntt, 630 + c))
    plan = orc.downsample_plan(height, width, batch, r, base, rows_per_group=group)
    got, _ = run_downsample(orc, ctx, s, s_ntt, cts, level, plan, 670, deferred=True)
    for c in range(n_ct):
        dec = orc.decrypt(got[c], level - 2, s_ntt, scale)
        want = X[c][:, ::r, ::r].reshape(-1)
        assert np.abs(dec[:want.size] - want).max() < 1e-5 and np.abs(dec[want.size:]).max() < 1e-5


def test_relayout_rejects_bad_arguments():
    p = make_params(10, 5, 2, 3)
    orc, ctx = both(p)
    level = 3
    s, s_ntt = orc.gen_secret(700)
    key = hx.ckks_key_load(ctx, hx.from_host(orc.gen_rotation_key(s, s_ntt, 4, 701)), hx.ckks_galois_element(ctx, 4))
    ct, m = hx.empty(2, level + 1, orc.N), hx.empty(level + 1, orc.N)
    with pytest.raises(hx.CkksError) as e:                  # the key was made for another offset
        hx.he_relayout_two_rotations(ctx, [ct], level, [0, 5], [None, key], [0], [None], [[m, m]])
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY
    with pytest.raises(hx.CkksError) as e:                  # a second rotation without any mask
        hx.he_relayout_two_rotations(ctx, [ct], level, [0, 4], [None, key], [0, 4], [None, key], [[m, m], [None, None]])
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG
    with pytest.raises(hx.CkksError) as e:                  # level 0 has no limb to drop
        hx.he_relayout_two_rotations(ctx, [hx.empty(2, 1, orc.N)], 0, [0], [None], [0], [None], [[hx.empty(1, orc.N)]],
                                     outs=[hx.empty(0)])
    assert e.value.code == hx.binding.CKKS_ERR_LEVEL_MISMATCH
    for schedule, mm in ((hx.HE_RELAYOUT_DIRECT, m), (hx.HE_RELAYOUT_DEFERRED, hx.empty(level + 1 + p.num_p, orc.N))):
        with pytest.raises(hx.CkksError) as e:
            hx.he_relayout_two_rotations(ctx, [ct], level, [0, 4], [None, key], [0], [None], [[mm, mm]], schedule=schedule, ws=hx.empty(512))
        assert e.value.code == hx.binding.CKKS_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(ValueError):                         # masks of the other schedule's shape
        hx.he_relayout_two_rotations(ctx, [ct], level, [0, 4], [None, key], [0], [None], [[m, m]], schedule=hx.HE_RELAYOUT_DEFERRED)


# ------------------------------------------------------------------------------------ activation
@pytest.mark.parametrize("n_ct", [1, 3, 10])
def test_poly_activation_matches_oracle(n_ct):
    """1 ciphertext, a partial batch, and more than one batch of 8."""
    wl = CONFIGS["small_block"]
    p = wl.params()
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(301)
    rlk = orc.gen_relin_key(s_ntt, 302)
    rng = np.random.default_rng(303)
    scale = 2.0 ** 50
    plan = orc.act_schedule(level, scale)
    xs = [rng.uniform(-1, 1, orc.n) for _ in range(n_ct)]
    cts = [orc.encrypt(x, scale, level, s_ntt, 304 + i) for i, x in enumerate(xs)]
    outs = hx.he_poly_act_deg7(ctx, [hx.from_host(ct) for ct in cts], level, plan["k"], hx.ckks_key_load(ctx, hx.from_host(rlk), 0))
    for i in range(n_ct):
        got = hx.to_host(outs[i])
        assert np.array_equal(got, orc.poly_activation(cts[i], level, plan["k"], rlk)), f"channel {i}"
        dec = orc.decrypt(got, plan["out_level"], s_ntt, plan["out_scale"])
        assert np.abs(dec - activation_reference(xs[i])).max() < 1e-3


@pytest.mark.parametrize("n_ct,bits,log_n", [(1, 50, None), (10, 50, None), (2, 56, None), (2, 50, 14), (1, 50, 15)])
def test_poly_activation_merged_division_matches_oracle(n_ct, bits, log_n):
    wl = CONFIGS["small_block"]
    p = make_params(log_n or wl.log_n, wl.num_q, wl.num_p, wl.dnum, bits=bits)
    orc, ctx = both(p)
    level = p.num_q - 1
    s, s_ntt = orc.gen_secret(351)
    rlk = orc.gen_relin_key(s_ntt, 352)
    rng = np.random.default_rng(353)
    scale = float(2 ** (bits - 1)) if bits > 50 else 2.0 ** 50
    plan = orc.act_schedule(level, scale)
    xs = [rng.uniform(-1, 1, orc.n) for _ in range(n_ct)]
    cts = [orc.encrypt(x, scale, level, s_ntt, 354 + i) for i, x in enumerate(xs)]
    outs = hx.he_poly_act_deg7(ctx, [hx.from_host(ct) for ct in cts], level, plan["k"], hx.ckks_key_load(ctx, hx.from_host(rlk), 0),
                               merged=True)
    for i in range(n_ct):
        got = hx.to_host(outs[i])
        assert np.array_equal(got, orc.poly_activation_merged(cts[i], level, plan["k"], rlk)), f"channel {i}"
        dec = orc.decrypt(got, plan["out_level"], s_ntt, plan["out_scale"])
        assert np.abs(dec - activation_reference(xs[i])).max() < 1e-3


# ----------------------------------------------------------------------------------- error paths
def test_error_codes(ks_setup):
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    level = 3
    ct = hx.from_host(rand_ct(np.random.default_rng(1), p.moduli, level, orc.N))
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_keyswitch(ctx, ct[0], level, d_rlk, ws=hx.empty(16))
    assert e.value.code == hx.binding.CKKS_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_keyswitch(ctx, ct[0], level, None)
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_rescale(ctx, hx.empty(2, 1, orc.N), 0)
    assert e.value.code == hx.binding.CKKS_ERR_LEVEL_MISMATCH
    k1 = hx.ckks_key_load(ctx, hx.from_host(rlk), hx.ckks_galois_element(ctx, 1))
    with pytest.raises(hx.CkksError) as e:                 # key of offset 1 offered for offset 2
        hx.ckks_rotate_hoisted(ctx, ct, level, [2], [k1])
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY
    with pytest.raises(hx.CkksError) as e:                 # a rotation key is not a relinearisation key
        hx.ckks_ctct_mul_relin(ctx, ct, ct, level, k1)
    assert e.value.code == hx.binding.CKKS_ERR_NO_KEY
    with pytest.raises(hx.CkksError) as e:                 # slot constraint m*b <= n
        hx.he_conv_batched(ctx, 64, 64, 2, level, [ct], [None] * 9, hx.empty(9, level + 1, orc.N), hx.empty(1, 1, 9, level + 1), 1)
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_ntt_fwd(ctx, hx.empty(1, 1, orc.N), [99])
    assert e.value.code == hx.binding.CKKS_ERR_INVALID_ARG


def test_empty_inputs_are_rejected(ks_setup):
    """A zero count is an argument error at every entry point (nothing is enqueued)."""
    p, orc, ctx, s, s_ntt, rlk, d_rlk = ks_setup
    level = 2
    ct = hx.from_host(rand_ct(np.random.default_rng(2), p.moduli, level, orc.N))
    pt = hx.from_host(rand_poly(np.random.default_rng(3), p.moduli[:level + 1], orc.N))
    bad = hx.binding.CKKS_ERR_INVALID_ARG
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_rotate_hoisted(ctx, ct, level, [], [])
    assert e.value.code == bad
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_ptct_mac(ctx, [], [], level)
    assert e.value.code == bad
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_ntt_fwd(ctx, hx.empty(1, 1, orc.N)[:0], [], batch=0)
    assert e.value.code == bad
    with pytest.raises(hx.CkksError) as e:
        hx.ckks_ntt_inv(ctx, hx.empty(1, 1, orc.N)[:0], [0], batch=0)
    assert e.value.code == bad
    with pytest.raises(hx.CkksError) as e:
        hx.he_conv_batched(ctx, 8, 8, 0, level, [ct], [None] * 9, hx.empty(9, level + 1, orc.N), hx.empty(1, 1, 9, level + 1), 1)
    assert e.value.code == bad
    # the operands above are still usable afterwards: one term, accumulate off
    acc = hx.ckks_ptct_mac(ctx, [pt], [ct], level)
    assert np.array_equal(hx.to_host(acc), orc.ptct_mac([hx.to_host(pt)], [hx.to_host(ct)], level))

