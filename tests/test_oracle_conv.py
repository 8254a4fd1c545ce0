"""Pins for the oracle's client side and the batched convolution: the canonical embedding by
its O(N^2) definition, the float64 convolution against scipy, decrypted HE convolutions against
the float64 convolution, and special cases that collapse to simpler operations."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import Oracle, conv2d_reference, activation_reference, ACT_COEFFS
from workloads import CONFIGS, make_params, image_batch, conv_weights, conv_tap_offsets


def test_encode_decode_against_embedding_definition():
    o = Oracle(make_params(8, 1, 0, 1))
    rng = np.random.default_rng(0)
    z = rng.uniform(-1, 1, o.n)
    m = o.encode(z, 2.0 ** 30)
    slots = o.embed_definition(m) / 2.0 ** 30
    assert np.abs(slots.real - z).max() < 1e-6 and np.abs(slots.imag).max() < 1e-6
    assert np.abs(o.decode(m, 2.0 ** 30) - slots.real).max() < 1e-9
    # a constant vector encodes to a constant polynomial, the slot index e_0 alone to a known one
    assert o.encode(np.full(o.n, 0.75), 2.0 ** 20).tolist() == [int(0.75 * 2 ** 20)] + [0] * (o.N - 1)


@pytest.mark.parametrize("log_n", [5, 12, 16])
def test_encode_decode_round_trip(log_n):
    o = Oracle(make_params(log_n, 1, 0, 1))
    z = np.random.default_rng(1).uniform(-1, 1, o.n)
    assert np.abs(o.decode(o.encode(z, 2.0 ** 40), 2.0 ** 40) - z).max() < 2.0 ** -30


def test_product_of_encodings_is_slotwise_product():
    p = make_params(6, 2, 0, 1)
    o = Oracle(p)
    rng = np.random.default_rng(2)
    za, zb = rng.uniform(-1, 1, o.n), rng.uniform(-1, 1, o.n)
    sc = 2.0 ** 20
    q = p.moduli[0]
    a = np.array([int(v) % q for v in o.encode(za, sc)], dtype=np.uint64)
    b = np.array([int(v) % q for v in o.encode(zb, sc)], dtype=np.uint64)
    c = o.schoolbook(q, a, b)
    cc = np.array([int(v) - q if int(v) > q // 2 else int(v) for v in c], dtype=np.float64)
    assert np.abs(o.decode(cc, sc * sc) - za * zb).max() < 1e-4


def test_rounding_is_half_away_from_zero():
    from oracle.core import round_half_away
    assert round_half_away(np.array([0.5, -0.5, 1.5, -1.5, 2.4, -2.6])).tolist() == [1, -1, 2, -2, 2, -3]


def test_encrypt_decrypt(cfg1_params):
    o = Oracle(cfg1_params)
    s, s_ntt = o.gen_secret(1)
    z = np.random.default_rng(3).uniform(-1, 1, o.n)
    for level in (3, 1, 0):
        ct = o.encrypt(z, 2.0 ** 40, level, s_ntt, 2 + level)
        assert np.abs(o.decrypt(ct, level, s_ntt, 2.0 ** 40) - z).max() < 1e-8
    _, other = o.gen_secret(99)
    assert np.abs(o.decrypt(ct, 0, other, 2.0 ** 40) - z).max() > 1.0


def test_float_conv_matches_scipy():
    rng = np.random.default_rng(4)
    img = rng.uniform(-1, 1, (3, 4, 6, 5))
    w = rng.normal(0, 0.3, (2, 4, 3, 3))
    got = conv2d_reference(img, w)
    for b in range(3):
        for o_ in range(2):
            want = sum(correlate2d(img[b, c], w[o_, c], mode="same", boundary="fill", fillvalue=0) for c in range(4))
            assert np.abs(got[b, o_] - want).max() < 1e-12


def test_pack_and_masks():
    o = Oracle(make_params(8, 1, 0, 1))
    img = np.arange(2 * 1 * 4 * 4, dtype=np.float64).reshape(2, 1, 4, 4)
    z = o.pack_channel(img, 0)
    assert z[:32].tolist() == list(range(32)) and not z[32:].any()
    with pytest.raises(ValueError):
        o.pack_channel(np.zeros((9, 1, 4, 4)), 0)  # 9*16 > 128 slots
    masks = o.tap_masks(4, 4, 2)
    assert masks[4, :32].all() and not masks[:, 32:].any()          # centre tap: all ones
    top_left = masks[0, :16].reshape(4, 4)                          # tap (-1,-1)
    assert not top_left[0].any() and not top_left[:, 0].any() and top_left[1:, 1:].all()
    assert np.array_equal(masks[0, :16], masks[0, 16:32])            # replicated over the batch
    # masked roll == zero-padded shift, including across image boundaries
    offs = conv_tap_offsets(4)
    for t, (dy, dx) in enumerate([(a, b) for a in (-1, 0, 1) for b in (-1, 0, 1)]):
        shifted = np.zeros_like(img)
        for y in range(4):
            for x in range(4):
                if 0 <= y + dy < 4 and 0 <= x + dx < 4:
                    shifted[:, :, y, x] = img[:, :, y + dy, x + dx]
        assert np.array_equal((np.roll(z, -offs[t]) * masks[t])[:32], shifted.reshape(-1))


def _conv_setup(name, seed_base, level=None):
    wl = CONFIGS[name]
    p = wl.params()
    o = Oracle(p)
    level = p.num_q - 1 if level is None else level
    s, s_ntt = o.gen_secret(seed_base)
    img = image_batch(wl.batch, wl.c_in, wl.height, wl.width)
    w = conv_weights(wl.c_out, wl.c_in, dist="uniform" if wl.c_in == 1 else "he_normal")
    scale = 2.0 ** 40
    cts = [o.encrypt(o.pack_channel(img, c), scale, level, s_ntt, seed_base + 10 + c) for c in range(wl.c_in)]
    keys = {off: o.gen_rotation_key(s, s_ntt, off, seed_base + 100 + i)
            for i, off in enumerate(conv_tap_offsets(wl.width)) if off != 0}
    return wl, p, o, level, s, s_ntt, img, w, scale, cts, keys


@pytest.mark.parametrize("name", ["cfg1_single_conv", "small_conv"])
def test_he_conv_decrypts_to_float_conv(name):
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup(name, 1000)
    delta_m = 2.0 ** 28
    delta_w = p.moduli[level] / delta_m           # so that the rescale restores the input scale
    M, w_int = o.conv_operands(w, wl.height, wl.width, wl.batch, level, delta_m, delta_w)
    outs = o.he_conv(cts, level, wl.width, keys, M, w_int)
    want = conv2d_reference(img, w)
    for oc, ct in outs.items():
        got = o.unpack_channel(o.decrypt(ct, level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(got - want[:, oc]).max() < 1e-4
    # unused slots stay (almost) zero
    z = o.decrypt(outs[0], level - 1, s_ntt, scale)
    assert np.abs(z[wl.batch * wl.height * wl.width:]).max() < 1e-4 if wl.batch * wl.height * wl.width < o.n else True


def test_he_conv_centre_only_kernel_is_scalar_multiple():
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("cfg1_single_conv", 2000)
    w = np.zeros_like(w)
    w[0, 0, 1, 1] = 0.375
    delta_m = 2.0 ** 28
    M, w_int = o.conv_operands(w, wl.height, wl.width, wl.batch, level, delta_m, p.moduli[level] / delta_m)
    out = o.he_conv(cts, level, wl.width, keys, M, w_int)[0]
    got = o.decrypt(out, level - 1, s_ntt, scale)
    assert np.abs(got - 0.375 * o.pack_channel(img, 0)).max() < 1e-5


def test_he_conv_unhoisted_schedule_agrees():
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("cfg1_single_conv", 3000)
    delta_m = 2.0 ** 28
    M, w_int = o.conv_operands(w, wl.height, wl.width, wl.batch, level, delta_m, p.moduli[level] / delta_m)
    a = o.he_conv(cts, level, wl.width, keys, M, w_int, hoisted=True)[0]
    b = o.he_conv(cts, level, wl.width, keys, M, w_int, hoisted=False)[0]
    assert np.array_equal(a, b)


def test_four_key_alignment_gives_the_same_aligned_slots():
    """The two-stage alignment with the keys {-1, +1, -W, +W} (Eqs. 8-10) and the eight direct
    rotations decrypt to the same nine vectors: the input rolled by dy*W+dx."""
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("small_conv", 5000)
    W = wl.width
    four = {off: keys[off] for off in (-1, 1, -W, W)}            # only these four keys exist
    z = o.pack_channel(img, 0)
    a = o.align_four_keys(cts[0], level, W, four)
    b = o.align_direct(cts[0], level, W, keys)
    assert len(a) == len(b) == 9
    for t, off in enumerate(conv_tap_offsets(W)):
        za, zb = o.decrypt(a[t], level, s_ntt, scale), o.decrypt(b[t], level, s_ntt, scale)
        assert np.abs(za - np.roll(z, -off)).max() < 1e-5, t
        assert np.abs(za - zb).max() < 1e-5, t
    assert np.array_equal(a[4], b[4])                               # the centre is the input itself
    for t in (1, 3, 5, 7):                                          # one-step taps: the very same key switch
        assert np.array_equal(a[t], b[t]), t
    for t in (0, 2, 6, 8):                                          # corners: two key switches, other residues
        assert not np.array_equal(a[t], b[t]), t


@pytest.mark.parametrize("name", ["cfg1_single_conv", "small_conv"])
def test_he_conv_four_keys_decrypts_to_float_conv(name):
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup(name, 6000)
    W = wl.width
    four = {off: keys[off] for off in (-1, 1, -W, W)}
    delta_m = 2.0 ** 28
    M, w_int = o.conv_operands(w, wl.height, wl.width, wl.batch, level, delta_m, p.moduli[level] / delta_m)
    outs = o.he_conv(cts, level, W, four, M, w_int, four_keys=True)
    want = conv2d_reference(img, w)
    for oc, ct in outs.items():
        got = o.unpack_channel(o.decrypt(ct, level - 1, s_ntt, scale), wl.batch, wl.height, wl.width)
        assert np.abs(got - want[:, oc]).max() < 1e-4


def test_mac_on_extended_basis_matches_python_integers(tiny_params):
    o = Oracle(tiny_params)
    level = 1                                                    # extended basis: q_0, q_1, p_0, p_1
    ext = o.ext_moduli_idx(level)
    assert ext == [0, 1, 3, 4]
    rng = np.random.default_rng(6)
    pts = [np.stack([rng.integers(0, o.moduli[t], o.N, dtype=np.uint64) for t in ext]) for _ in range(5)]
    xs = [np.stack([np.stack([rng.integers(0, o.moduli[t], o.N, dtype=np.uint64) for t in ext]) for _ in range(2)]) for _ in range(5)]
    got = o.mac_ext(pts, xs, level)
    for comp in range(2):
        for e, t in enumerate(ext):
            q = o.moduli[t]
            want = [sum(int(pts[k][e][x]) * int(xs[k][comp][e][x]) for k in range(5)) % q for x in range(o.N)]
            assert got[comp, e].tolist() == want
    P = o.moduli[3] * o.moduli[4]
    assert o.special_product_residues(level).tolist() == [P % o.moduli[0], P % o.moduli[1], 0, 0]
    assert o.scalar_residues_ext(-3, level).tolist() == [o.moduli[t] - 3 for t in ext]
    sm = o.scalar_mul_ext(xs[0], o.scalar_residues_ext(-3, level), level)
    assert sm[1, 2].tolist() == [(-3 * int(v)) % o.moduli[3] for v in xs[0][1][2]]


def test_deferred_moddown_alignment_is_the_rotation_times_P():
    """ModDown of each pre-division aligned copy is the hoisted rotation itself (same residues), and
    on tiny parameters the copy is congruent to P * Rot modulo every q_i up to the rounding part."""
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("small_conv", 7000)
    a = o.align_deferred(cts[0], level, wl.width, keys)
    b = o.align_direct(cts[0], level, wl.width, keys)
    E = level + 1 + o.num_p
    for t in range(9):
        assert a[t].shape == (2, E, o.N)
        got = np.stack([o.moddown(a[t][0], level), o.moddown(a[t][1], level)])
        assert np.array_equal(got, b[t]), t
    assert not a[4][:, level + 1:].any()                        # centre: P * ct vanishes on the special primes


@pytest.mark.parametrize("name", ["cfg1_single_conv", "small_conv"])
def test_he_conv_deferred_moddown_decrypts_to_float_conv(name):
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup(name, 8000)
    delta_m = 2.0 ** 28
    delta_w = p.moduli[level] / delta_m
    M_ext, w_int = o.conv_operands_ext(w, wl.height, wl.width, wl.batch, level, delta_m, delta_w)
    M, w_int2 = o.conv_operands(w, wl.height, wl.width, wl.batch, level, delta_m, delta_w)
    assert np.array_equal(M_ext[:, :level + 1], M) and np.array_equal(w_int, w_int2)
    outs = o.he_conv_deferred(cts, level, wl.width, keys, M_ext, w_int)
    direct = o.he_conv(cts, level, wl.width, keys, M, w_int)
    want = conv2d_reference(img, w)
    for oc, ct in outs.items():
        z = o.decrypt(ct, level - 1, s_ntt, scale)
        assert np.abs(o.unpack_channel(z, wl.batch, wl.height, wl.width) - want[:, oc]).max() < 1e-4
        assert np.abs(z - o.decrypt(direct[oc], level - 1, s_ntt, scale)).max() < 1e-5
        assert not np.array_equal(ct, direct[oc])                # one rounding instead of many: other residues


def test_he_conv_deferred_centre_only_kernel_equals_direct():
    """With only the centre weight nothing is rotated: ModDown(P * y) = y exactly, so both schedules
    must give the very same residues."""
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("cfg1_single_conv", 9000)
    w = np.zeros_like(w)
    w[0, 0, 1, 1] = -0.4375
    delta_m = 2.0 ** 28
    M_ext, w_int = o.conv_operands_ext(w, wl.height, wl.width, wl.batch, level, delta_m, p.moduli[level] / delta_m)
    a = o.he_conv_deferred(cts, level, wl.width, keys, M_ext, w_int)[0]
    b = o.he_conv(cts, level, wl.width, keys, M_ext[:, :level + 1], w_int)[0]
    assert np.array_equal(a, b)


def test_accumulator_merge_concatenates_cleaned_blocks():
    """g = 4 intermediate ciphertexts with data in the first quarter of the slots and junk behind it:
    the merged ciphertext decrypts to the four cleaned blocks side by side; g = 1 is mask-and-rescale."""
    p = CONFIGS["small_conv"].params()
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(10000)
    g, sts = 4, o.n // 4
    rng = np.random.default_rng(7)
    zs = [rng.uniform(-1, 1, o.n) for _ in range(g)]               # slots beyond sts are junk to be cleaned
    scale = 2.0 ** 40
    cts = [o.encrypt(z, scale, level, s_ntt, 10001 + i) for i, z in enumerate(zs)]
    M = o.encode_ntt(o.cleaning_mask(sts), float(p.moduli[level]), level)   # mask at scale q_level: the rescale restores 2^40
    keys = {-i * sts: o.gen_rotation_key(s, s_ntt, -i * sts, 10100 + i) for i in range(1, g)}
    out = o.accumulator_merge(cts, level, sts, M, keys)
    assert out.shape == (2, level, o.N)
    want = np.concatenate([z[:sts] for z in zs])
    assert np.abs(o.decrypt(out, level - 1, s_ntt, scale) - want).max() < 1e-5
    one = o.accumulator_merge(cts[:1], level, sts, M, {})
    assert np.array_equal(one, o.rescale(o.ptct_mac([M], [cts[0]], level), level))
    z1 = o.decrypt(one, level - 1, s_ntt, scale)
    assert np.abs(z1[:sts] - zs[0][:sts]).max() < 1e-5 and np.abs(z1[sts:]).max() < 1e-5
    with pytest.raises(ValueError):
        o.accumulator_merge(cts * 2, level, sts, M, keys)


def downsample_keys(o, s, s_ntt, plan, seed):
    offs = sorted({r for lo, hi, _ in plan for r in list(lo) + list(hi) if r % o.n})
    return {r: o.gen_rotation_key(s, s_ntt, r, seed + k) for k, r in enumerate(offs)}


@pytest.mark.parametrize("height,width,batch,r,base", [(4, 4, 8, 2, 3), (4, 8, 5, 2, 0), (8, 8, 2, 4, 1), (2, 2, 16, 2, 16)])
def test_downsample_compaction_is_the_strided_selection(height, width, batch, r, base):
    """Every image keeps its elements (r y', r x') and the kept elements of image j end up row-major in slots
    [j H'W', (j+1) H'W'); the dropped elements and the unused slots decrypt to zero (float64 reference: numpy slicing)."""
    p = make_params(10, 5, 2, 3)
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(14000)
    X = np.random.default_rng(11).uniform(-1, 1, (batch, height, width))
    z = np.random.default_rng(12).uniform(-1, 1, o.n)          # junk behind the images: it has to vanish
    z[:X.size] = X.reshape(-1)
    scale = 2.0 ** 40
    ct = o.encrypt(z, scale, level, s_ntt, 14001)
    plan = o.downsample_plan(height, width, batch, r, base)
    out = o.downsample_compact(ct, level, plan, downsample_keys(o, s, s_ntt, plan, 14100))
    assert out.shape == (2, level - 1, o.N)
    got = o.decrypt(out, level - 2, s_ntt, scale)
    want = X[:, ::r, ::r].reshape(-1)
    assert np.abs(got[:want.size] - want).max() < 1e-5
    assert np.abs(got[want.size:]).max() < 1e-5


@pytest.mark.parametrize("height,width,batch,r,base,group", [(4, 4, 8, 2, 3, 1), (4, 8, 5, 2, 5, 2), (8, 8, 2, 2, 1, 4)])
def test_downsample_compaction_with_deferred_divisions(height, width, batch, r, base, group):
    """The deferred schedule (sums on the extended basis, one merged division per second rotation, one ModDown) gives the
    strided selection too, agrees with the plain schedule in the slots to rounding noise, and differs in the residues;
    several rows per group (many first, few second rotations; group = H': no second rotation inside the images)."""
    p = make_params(10, 5, 2, 3)
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(14500)
    X = np.random.default_rng(21).uniform(-1, 1, (batch, height, width))
    z = np.random.default_rng(22).uniform(-1, 1, o.n)
    z[:X.size] = X.reshape(-1)
    scale = 2.0 ** 40
    ct = o.encrypt(z, scale, level, s_ntt, 14501)
    plan = o.downsample_plan(height, width, batch, r, base, rows_per_group=group)
    keys = downsample_keys(o, s, s_ntt, plan, 14600)
    out = o.downsample_compact(ct, level, plan, keys, deferred=True)
    ref = o.downsample_compact(ct, level, plan, keys, deferred=False)
    assert out.shape == ref.shape == (2, level - 1, o.N) and not np.array_equal(out, ref)
    got = o.decrypt(out, level - 2, s_ntt, scale)
    want = X[:, ::r, ::r].reshape(-1)
    assert np.abs(got[:want.size] - want).max() < 1e-5 and np.abs(got[want.size:]).max() < 1e-5
    assert np.abs(got - o.decrypt(ref, level - 2, s_ntt, scale)).max() < 1e-6


def test_aligned_copy_divides_to_the_rotation():
    """ModDown of the pre-division copy is the hoisted rotation, residue for residue (offset 0: the ciphertext itself)."""
    p = make_params(10, 4, 2, 2)
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(14700)
    ct = o.encrypt(np.random.default_rng(23).uniform(-1, 1, o.n), 2.0 ** 40, level, s_ntt, 14701)
    digits = o.modup(ct[1], level)
    for off in (0, 7, -3):
        key = o.gen_rotation_key(s, s_ntt, off, 14710 + off) if off else None
        x = o.aligned_ext(ct, level, off, key, digits)
        down = np.stack([o.moddown(x[0], level), o.moddown(x[1], level)])
        assert np.array_equal(down, o.rotate(ct, level, off, key, True, digits))


@pytest.mark.parametrize("group", [1, 2])
def test_downsample_plan_moves_every_kept_slot_exactly_once(group):
    """The plan alone, on slot indices: following mask -> first rotation -> second rotation sends the slot of every kept
    element to its compact position, no two masks of a stage overlap after their rotations, and the slot accounting of the
    pipeline holds (sts' = sts / r^2)."""
    o = Oracle(make_params(10, 1, 0, 1))
    height, width, batch, r = 4, 8, 7, 2
    (lo_a, hi_a, m_a), (lo_b, hi_b, m_b) = o.downsample_plan(height, width, batch, r, 3, rows_per_group=group)
    assert len(lo_a) == group * (width // r) and len(hi_a) == height // r // group
    pos = {}                                                       # slot -> (j, y', x') through the stages
    for j in range(batch):
        for y in range(height // r):
            for x in range(width // r):
                pos[j * height * width + r * y * width + r * x] = (j, y, x)
    for lo, hi, masks in ((lo_a, hi_a, m_a), (lo_b, hi_b, m_b)):
        nxt = {}
        for h, row in enumerate(masks):
            for l, m in enumerate(row):
                if m is None:
                    continue
                for slot in np.flatnonzero(m):
                    src = int(slot) + lo[l]                        # where the selected slot was before the first rotation
                    assert src in pos, "a mask selects a slot that holds no kept element"
                    dst = int(slot) - hi[h]
                    assert dst not in nxt
                    nxt[dst] = pos.pop(src)
        assert not pos, "a kept element is selected by no mask"
        pos = nxt
    h2, w2 = height // r, width // r
    assert pos == {j * h2 * w2 + y * w2 + x: (j, y, x) for j in range(batch) for y in range(h2) for x in range(w2)}
    assert len(pos) * r * r == batch * height * width


def test_strided_conv_then_accumulator_fills_the_ciphertext():
    """The block-group transition end to end: g = 4 tiles of images go through a 3x3 convolution, are down-sampled with
    stride 2 and merged by the accumulator into one ciphertext holding 4x the images at the smaller size; the slots
    equal the stride-2 convolution (float64 reference, sliced) of all tiles side by side."""
    p = make_params(10, 6, 2, 3)
    o = Oracle(p)
    level = p.num_q - 1
    height = width = 4
    batch, g, c_in = 8, 4, 2
    s, s_ntt = o.gen_secret(15000)
    scale = 2.0 ** 40
    w = conv_weights(1, c_in, dist="he_normal")
    offs = conv_tap_offsets(width)
    keys = {off: o.gen_rotation_key(s, s_ntt, off, 15100 + i) for i, off in enumerate(offs) if off}
    M, w_int = o.conv_operands(w, height, width, batch, level, 2.0 ** 28, p.moduli[level] / 2.0 ** 28)
    plan = o.downsample_plan(height, width, batch, 2, 3)
    dkeys = downsample_keys(o, s, s_ntt, plan, 15200)
    sts2 = batch * height * width // 4
    tiles, refs = [], []
    for t in range(g):
        img = image_batch(batch, c_in, height, width, seed=15300 + t)
        cts = [o.encrypt(o.pack_channel(img, c), scale, level, s_ntt, 15400 + 10 * t + c) for c in range(c_in)]
        conv = o.he_conv(cts, level, width, keys, M, w_int)[0]                       # level-1
        tiles.append(o.downsample_compact(conv, level - 1, plan, dkeys))            # level-3
        refs.append(conv2d_reference(img, w)[:, 0, ::2, ::2].reshape(-1))
    lm = level - 3
    Mc = o.encode_ntt(o.cleaning_mask(sts2), float(p.moduli[lm]), lm)
    mkeys = {-i * sts2: o.gen_rotation_key(s, s_ntt, -i * sts2, 15500 + i) for i in range(1, g)}
    joined = o.accumulator_merge(tiles, lm, sts2, Mc, mkeys)
    got = o.decrypt(joined, lm - 1, s_ntt, scale)
    want = np.concatenate(refs)
    assert want.size == g * sts2 == batch * height * width                            # the ciphertext's images are full again
    assert np.abs(got[:want.size] - want).max() < 1e-4
    assert np.abs(got[want.size:]).max() < 1e-4


def test_activation_polynomial_pins():
    assert activation_reference(np.array([0.0, 1.0, -1.0])).tolist() == [0.0, 1.0, -1.0]
    # p'(x) = 35/16 (1-x^2)^3: flat at +-1
    h = 1e-4
    assert abs(activation_reference(np.array([1 - h]))[0] - 1) < 1e-10
    assert abs(sum(ACT_COEFFS) - 1) < 1e-15


def test_encrypted_activation_matches_float():
    wl = CONFIGS["small_block"]
    p = wl.params()
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(4000)
    rlk = o.gen_relin_key(s_ntt, 4001)
    x = np.random.default_rng(5).uniform(-1, 1, o.n)
    scale = 2.0 ** 50
    ct = o.encrypt(x, scale, level, s_ntt, 4002)
    plan = o.act_schedule(level, scale)
    out = o.poly_activation(ct, level, plan["k"], rlk)
    assert out.shape == (2, plan["out_level"] + 1, o.N)
    got = o.decrypt(out, plan["out_level"], s_ntt, plan["out_scale"])
    assert np.abs(got - activation_reference(x)).max() < 1e-3


def test_merged_division_product_and_activation_match_float():
    """Rescale(a*b + addend) with one division by P*q_level: decrypts to the slot-wise product plus the
    addend, agrees with the two-step version up to rounding noise, and the activation built on it
    matches the float64 polynomial."""
    wl = CONFIGS["small_block"]
    p = wl.params()
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(11000)
    rlk = o.gen_relin_key(s_ntt, 11001)
    rng = np.random.default_rng(8)
    xa, xb, xc = (rng.uniform(-1, 1, o.n) for _ in range(3))
    scale = 2.0 ** 50
    a, b = o.encrypt(xa, scale, level, s_ntt, 11002), o.encrypt(xb, scale, level, s_ntt, 11003)
    # an addend at the product's scale 2^100: an encryption at 2^50 times the integer 2^50
    add = o.scalar_mul(o.encrypt(xc, scale, level, s_ntt, 11004), o.scalar_residues(2 ** 50, level), level)
    out = o.ctct_mul_relin_rescale(a, b, rlk, level, addend=add)
    assert out.shape == (2, level, o.N)
    out_scale = scale * scale / p.moduli[level]
    assert np.abs(o.decrypt(out, level - 1, s_ntt, out_scale) - (xa * xb + xc)).max() < 1e-6
    two_step = o.rescale(o.add(o.ctct_mul_relin(a, b, rlk, level), add, level), level)
    assert np.abs(o.decrypt(out, level - 1, s_ntt, out_scale) - o.decrypt(two_step, level - 1, s_ntt, out_scale)).max() < 1e-7
    assert not np.array_equal(out, two_step)
    plan = o.act_schedule(level, scale)
    y = o.poly_activation_merged(a, level, plan["k"], rlk)
    assert y.shape == (2, plan["out_level"] + 1, o.N)
    assert np.abs(o.decrypt(y, plan["out_level"], s_ntt, plan["out_scale"]) - activation_reference(xa)).max() < 1e-3


def test_he_conv_deferred_with_merged_division_decrypts_to_float_conv():
    wl, p, o, level, s, s_ntt, img, w, scale, cts, keys = _conv_setup("small_conv", 12000)
    delta_m = 2.0 ** 28
    M_ext, w_int = o.conv_operands_ext(w, wl.height, wl.width, wl.batch, level, delta_m, p.moduli[level] / delta_m)
    outs = o.he_conv_deferred(cts, level, wl.width, keys, M_ext, w_int, merged=True)
    two = o.he_conv_deferred(cts, level, wl.width, keys, M_ext, w_int)
    want = conv2d_reference(img, w)
    for oc, ct in outs.items():
        z = o.decrypt(ct, level - 1, s_ntt, scale)
        assert np.abs(o.unpack_channel(z, wl.batch, wl.height, wl.width) - want[:, oc]).max() < 1e-4
        assert np.abs(z - o.decrypt(two[oc], level - 1, s_ntt, scale)).max() < 1e-6


@pytest.mark.parametrize("d_in,d_out,batch,base", [(16, 4, 8, 3), (8, 8, 4, 2), (32, 10, 16, 4)])
def test_fc_batched_decrypts_to_the_affine_map(d_in, d_out, batch, base):
    """y = W x + b for every batch element, outputs packed at stride d_out (float64 reference: numpy matmul)."""
    p = make_params(10, 6, 2, 3)
    o = Oracle(p)
    level = p.num_q - 1
    s, s_ntt = o.gen_secret(13000)
    rng = np.random.default_rng(9)
    W = rng.normal(0, 0.3, (d_out, d_in))
    bias = rng.uniform(-0.5, 0.5, d_out)
    X = rng.uniform(-1, 1, (batch, d_in))
    z = np.zeros(o.n)
    z[:batch * d_in] = X.reshape(-1)
    scale = 2.0 ** 40
    ct = o.encrypt(z, scale, level, s_ntt, 13001)
    delta, lo, hi = o.fc_shifts(d_in, d_out, batch, base)
    offsets = {2 ** t for t in range(d_in.bit_length() - 1)} | {-i for i in range(1, d_out)} | set(lo[1:]) | set(hi[1:])
    keys = {r: o.gen_rotation_key(s, s_ntt, r, 13100 + k) for k, r in enumerate(sorted(offsets)) if r % o.n}
    ops = o.fc_operands(W, bias, batch, level, base, scale)
    out = o.fc_batched(ct, level, d_in, d_out, batch, base, *ops, keys)
    assert out.shape == (2, level - 2, o.N)
    got = o.decrypt(out, level - 3, s_ntt, scale)
    want = (X @ W.T + bias).reshape(-1)
    assert np.abs(got[:batch * d_out] - want).max() < 1e-4
    assert np.abs(got[batch * d_out:]).max() < 1e-4             # everything else is clean
