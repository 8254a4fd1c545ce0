"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.  See the package docstring."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SRC_PATH = os.path.join(_HERE, "ckks_oracle.cpp")
_lib = None

u64p = C.POINTER(C.c_uint64)


def build(force: bool = False) -> str:
    """Compile the C++ core with g++ (plain -O2, OpenMP over independent limbs)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC_PATH):
        subprocess.check_call(["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, _SRC_PATH])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.orc_create.restype = C.c_void_p
        _lib.orc_live_digits.restype = C.c_int
    return _lib


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def round_half_away(x: np.ndarray) -> np.ndarray:
    return np.where(x >= 0, np.floor(x + 0.5), np.ceil(x - 0.5))


# odd degree-7 polynomial with p(0)=0, p(+-1)=+-1, p'(+-1)=p''(+-1)=p'''(+-1)=0
ACT_COEFFS = (35.0 / 16.0, -35.0 / 16.0, 21.0 / 16.0, -5.0 / 16.0)


def activation_reference(x: np.ndarray) -> np.ndarray:
    c1, c3, c5, c7 = ACT_COEFFS
    return c1 * x + c3 * x**3 + c5 * x**5 + c7 * x**7


def conv2d_reference(images: np.ndarray, weights: np.ndarray) -> np.ndarray:
    """float64 cross-correlation, 3x3, stride 1, zero padding 1.
    images [B, C_in, H, W], weights [C_out, C_in, 3, 3] -> [B, C_out, H, W]:
    out[b,o,y,x] = sum_c sum_{dy,dx} weights[o,c,dy+1,dx+1] * images[b,c,y+dy,x+dx]."""
    B, Ci, H, W = images.shape
    Co = weights.shape[0]
    padded = np.zeros((B, Ci, H + 2, W + 2), dtype=np.float64)
    padded[:, :, 1:H + 1, 1:W + 1] = images
    out = np.zeros((B, Co, H, W), dtype=np.float64)
    for o in range(Co):
        for c in range(Ci):
            for dy in (-1, 0, 1):
                for dx in (-1, 0, 1):
                    out[:, o] += weights[o, c, dy + 1, dx + 1] * padded[:, c, 1 + dy:1 + dy + H, 1 + dx:1 + dx + W]
    return out


class Oracle:
    """One RNS-CKKS context (ring degree, modulus chain, special primes, digit count)."""

    def __init__(self, params):
        lib = _load()
        self.lib = lib
        self.log_n = int(params.log_n)
        self.N = 1 << self.log_n
        self.n = self.N // 2
        self.num_q = int(params.num_q)
        self.num_p = int(params.num_p)
        self.dnum = int(params.dnum)
        self.alpha = -(-self.num_q // self.dnum) if self.dnum else 0
        self.moduli = [int(q) for q in params.moduli]
        self.psi = [int(x) for x in params.psi]
        self.M = self.num_q + self.num_p
        mods = np.array(self.moduli, dtype=np.uint64)
        psis = np.array(self.psi, dtype=np.uint64)
        self.h = C.c_void_p(lib.orc_create(self.log_n, self.num_q, self.num_p, self.dnum, _p(mods), _p(psis)))
        if not self.h:
            raise ValueError("psi is not a primitive 2N-th root of unity for some modulus")

    def __del__(self):
        try:
            self.lib.orc_destroy(self.h)
        except Exception:
            pass

    # ----------------------------------------------------------------------------- NTT
    def ntt_fwd(self, a, mod_idx: int) -> np.ndarray:
        a = _u64(a).copy()
        self.lib.orc_ntt_fwd(self.h, int(mod_idx), _p(a))
        return a

    def ntt_inv(self, a, mod_idx: int) -> np.ndarray:
        a = _u64(a).copy()
        self.lib.orc_ntt_inv(self.h, int(mod_idx), _p(a))
        return a

    def ntt_definition(self, a, mod_idx: int) -> np.ndarray:
        a = _u64(a)
        out = np.empty_like(a)
        self.lib.orc_ntt_definition(self.h, int(mod_idx), _p(a), _p(out))
        return out

    def ntt_many(self, polys, mod_idx: Sequence[int], inverse: bool = False) -> np.ndarray:
        """polys [..., n_limbs, N]; limb t uses modulus mod_idx[t].  Returns a new array."""
        a = _u64(polys).copy()
        n_limbs = len(mod_idx)
        assert a.shape[-2] == n_limbs and a.shape[-1] == self.N
        idx = np.array(mod_idx, dtype=np.int32)
        batch = a.size // (n_limbs * self.N)
        self.lib.orc_ntt_many(self.h, _p(a), _p(idx), n_limbs, batch, int(bool(inverse)))
        return a

    def schoolbook(self, q: int, a, b) -> np.ndarray:
        a, b = _u64(a), _u64(b)
        out = np.empty_like(a)
        self.lib.orc_negacyclic_schoolbook(C.c_uint64(q), len(a), _p(a), _p(b), _p(out))
        return out

    # -------------------------------------------------------------------- automorphism
    def galois(self, offset: int) -> int:
        """Galois element of a left rotation by `offset` slots: 5^offset mod 2N."""
        return pow(5, offset % self.n, 2 * self.N)

    def automorph_coeff(self, a, mod_idx: int, g: int) -> np.ndarray:
        a = _u64(a)
        out = np.empty_like(a)
        self.lib.orc_automorph_coeff(self.h, int(mod_idx), C.c_uint64(g), _p(a), _p(out))
        return out

    def automorph_ntt(self, a, g: int) -> np.ndarray:
        """a [..., N] in NTT form; the same gather on every limb."""
        a = _u64(a)
        out = np.empty_like(a)
        flat_in, flat_out = a.reshape(-1, self.N), out.reshape(-1, self.N)
        for i in range(flat_in.shape[0]):
            self.lib.orc_automorph_ntt(self.h, C.c_uint64(g), _p(flat_in[i]), _p(flat_out[i]))
        return out

    # -------------------------------------------------------------------- key switching
    def live_digits(self, level: int) -> int:
        return (level + self.alpha) // self.alpha

    def ext_moduli_idx(self, level: int) -> List[int]:
        return list(range(level + 1)) + list(range(self.num_q, self.M))

    def modup(self, c, level: int) -> np.ndarray:
        c = _u64(c)
        assert c.shape == (level + 1, self.N)
        out = np.empty((self.live_digits(level), level + 1 + self.num_p, self.N), dtype=np.uint64)
        self.lib.orc_modup(self.h, level, _p(c), _p(out))
        return out

    def key_inner(self, digits, key, level: int) -> np.ndarray:
        digits, key = _u64(digits), _u64(key)
        assert key.shape == (self.dnum, 2, self.M, self.N)
        out = np.empty((2, level + 1 + self.num_p, self.N), dtype=np.uint64)
        self.lib.orc_key_inner(self.h, level, _p(digits), _p(key), _p(out))
        return out

    def moddown(self, v, level: int) -> np.ndarray:
        v = _u64(v)
        assert v.shape == (level + 1 + self.num_p, self.N)
        out = np.empty((level + 1, self.N), dtype=np.uint64)
        self.lib.orc_moddown(self.h, level, _p(v), _p(out))
        return out

    def divide_by_limbs(self, v, keep_idx: Sequence[int], drop_idx: Sequence[int]) -> np.ndarray:
        """v [len(keep)+len(drop)][N] (kept limbs first) divided by the product of the dropped moduli, rounded
        (centred remainder, error below len(drop)/2): ModDown and rescale are special cases."""
        v = _u64(v)
        keep = np.array(keep_idx, dtype=np.int32)
        drop = np.array(drop_idx, dtype=np.int32)
        assert v.shape == (len(keep) + len(drop), self.N)
        out = np.empty((len(keep), self.N), dtype=np.uint64)
        self.lib.orc_divide_by_limbs(self.h, _p(keep), len(keep), _p(drop), len(drop), _p(v), _p(out))
        return out

    def moddown_rescale(self, v, level: int) -> np.ndarray:
        """ModDown and rescale in one step: v on the extended basis q_0..q_level, p_0.. divided by P * q_level
        with a single rounding; result [level][N]."""
        return self.divide_by_limbs(v, list(range(level)), [level] + list(range(self.num_q, self.M)))

    def keyswitch(self, c, key, level: int) -> np.ndarray:
        c, key = _u64(c), _u64(key)
        assert c.shape == (level + 1, self.N) and key.shape == (self.dnum, 2, self.M, self.N)
        out = np.empty((2, level + 1, self.N), dtype=np.uint64)
        self.lib.orc_keyswitch(self.h, level, _p(c), _p(key), _p(out))
        return out

    def rotate(self, ct, level: int, offset: int, key, hoisted: bool, digits=None) -> np.ndarray:
        """Rot(ct, offset): slot i of the result holds slot (i+offset) mod n of the input."""
        ct = _u64(ct)
        assert ct.shape == (2, level + 1, self.N)
        if offset % self.n == 0:
            return ct.copy()
        key = _u64(key)
        g = self.galois(offset)
        out = np.empty_like(ct)
        if hoisted:
            if digits is None:
                digits = self.modup(ct[1], level)
            digits = _u64(digits)
            self.lib.orc_rotate_hoisted(self.h, level, C.c_uint64(g), _p(ct), _p(digits), _p(key), _p(out))
        else:
            self.lib.orc_rotate_unhoisted(self.h, level, C.c_uint64(g), _p(ct), _p(key), _p(out))
        return out

    def rotate_many(self, ct, level: int, offsets: Sequence[int], keys: Sequence, hoisted: bool) -> List[np.ndarray]:
        digits = self.modup(_u64(ct)[1], level) if hoisted else None
        return [self.rotate(ct, level, r, k, hoisted, digits) for r, k in zip(offsets, keys)]

    # ------------------------------------------------------------------------ pointwise
    def ptct_mac(self, pts: Sequence[np.ndarray], cts: Sequence[np.ndarray], level: int,
                 acc: Optional[np.ndarray] = None) -> np.ndarray:
        """sum_k pt_k (.) ct_k  (+ acc): Eq. 11 with the channel sum folded into the same sum."""
        assert len(pts) == len(cts)
        pts = [_u64(p) for p in pts]
        cts = [_u64(c) for c in cts]
        for p_, c_ in zip(pts, cts):
            assert p_.shape == (level + 1, self.N) and c_.shape == (2, level + 1, self.N)
        accumulate = acc is not None
        out = _u64(acc).copy() if accumulate else np.empty((2, level + 1, self.N), dtype=np.uint64)
        n = len(pts)
        pa = (C.c_void_p * n)(*[p_.ctypes.data for p_ in pts])
        ca = (C.c_void_p * n)(*[c_.ctypes.data for c_ in cts])
        self.lib.orc_ptct_mac(self.h, level, n, pa, ca, _p(out), int(accumulate))
        return out

    def scalar_residues(self, value: int, level: int) -> np.ndarray:
        """Residues of a (signed) integer scalar modulo q_0..q_level."""
        return np.array([int(value) % self.moduli[i] for i in range(level + 1)], dtype=np.uint64)

    def scalar_mul(self, poly, scalar_res, level: int) -> np.ndarray:
        """poly [n_comp, level+1, N] (or [level+1, N]) times an integer scalar given by residues."""
        poly = _u64(poly)
        n_comp = poly.size // ((level + 1) * self.N)
        out = np.empty_like(poly)
        self.lib.orc_scalar_mul(self.h, level, n_comp, _p(poly), _p(_u64(scalar_res)), _p(out))
        return out

    def add(self, a, b, level: int) -> np.ndarray:
        a, b = _u64(a), _u64(b)
        assert a.shape == b.shape
        n_comp = a.size // ((level + 1) * self.N)
        out = np.empty_like(a)
        self.lib.orc_add(self.h, level, n_comp, _p(a), _p(b), _p(out))
        return out

    @staticmethod
    def drop_to_level(ct, level: int) -> np.ndarray:
        """Forget limbs above `level` (RNS: lower levels are a prefix of the limbs)."""
        return np.ascontiguousarray(_u64(ct)[:, :level + 1, :])

    def rescale(self, ct, level: int) -> np.ndarray:
        ct = _u64(ct)
        assert ct.shape == (2, level + 1, self.N) and level >= 1
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self.lib.orc_rescale(self.h, level, _p(ct), _p(out))
        return out

    def ctct_mul_relin(self, a, b, rlk, level: int) -> np.ndarray:
        a, b, rlk = _u64(a), _u64(b), _u64(rlk)
        assert a.shape == b.shape == (2, level + 1, self.N)
        out = np.empty_like(a)
        self.lib.orc_ctct_mul_relin(self.h, level, _p(a), _p(b), _p(rlk), _p(out))
        return out

    # ------------------------------------------------------------------- encode / decode
    def _slot_index(self) -> np.ndarray:
        """k_j with zeta^(2 k_j + 1) = zeta^(5^j), j < n."""
        idx = np.empty(self.n, dtype=np.int64)
        e = 1
        for j in range(self.n):
            idx[j] = (e - 1) // 2
            e = e * 5 % (2 * self.N)
        return idx

    def encode(self, z: np.ndarray, scale: float) -> np.ndarray:
        """Real slot vector z[n] -> int64 coefficients m with m(zeta^(5^j)) ~ scale * z_j.
        The values at all N odd powers of zeta (slot values and their conjugates) are turned into
        coefficients by one FFT: m_i zeta^i = (1/N) sum_k v_k exp(-2 pi i ik/N)."""
        z = np.asarray(z, dtype=np.float64)
        assert z.shape == (self.n,)
        idx = self._slot_index()
        v = np.zeros(self.N, dtype=np.complex128)
        v[idx] = z
        v[self.N - 1 - idx] = z  # exponent -(2k+1) = 2(N-1-k)+1 mod 2N carries the conjugate
        i = np.arange(self.N)
        twist = np.exp(-1j * np.pi * i / self.N)
        m = (np.fft.fft(v) / self.N * twist).real * scale
        return round_half_away(m).astype(np.int64)

    def decode(self, coeffs: np.ndarray, scale: float) -> np.ndarray:
        """Coefficients (float64 or integer) -> real parts of the n slots, divided by scale."""
        m = np.asarray(coeffs, dtype=np.float64)
        i = np.arange(self.N)
        v = np.fft.ifft(m * np.exp(1j * np.pi * i / self.N)) * self.N
        return v[self._slot_index()].real / scale

    def embed_definition(self, coeffs: np.ndarray) -> np.ndarray:
        """O(N^2) canonical embedding: slot j = sum_i m_i zeta^(5^j i).  For pinning only."""
        m = np.asarray(coeffs, dtype=np.float64)
        out = np.empty(self.n, dtype=np.complex128)
        e = 1
        i = np.arange(self.N)
        for j in range(self.n):
            out[j] = np.sum(m * np.exp(1j * np.pi * ((e * i) % (2 * self.N)) / self.N))
            e = e * 5 % (2 * self.N)
        return out

    def lift_ntt(self, coeffs: np.ndarray, mod_idx: Sequence[int]) -> np.ndarray:
        coeffs = np.ascontiguousarray(coeffs, dtype=np.int64)
        idx = np.array(mod_idx, dtype=np.int32)
        out = np.empty((len(idx), self.N), dtype=np.uint64)
        self.lib.orc_lift_ntt(self.h, _p(coeffs), _p(idx), len(idx), _p(out))
        return out

    def encode_ntt(self, z: np.ndarray, scale: float, level: int) -> np.ndarray:
        """Plaintext polynomial [level+1][N] in NTT form."""
        return self.lift_ntt(self.encode(z, scale), list(range(level + 1)))

    # --------------------------------------------------------------------------- client
    def gen_secret(self, seed: int) -> Tuple[np.ndarray, np.ndarray]:
        """Ternary secret: (int64 coefficients, NTT form over all num_q+num_p moduli)."""
        s8 = np.empty(self.N, dtype=np.int8)
        self.lib.orc_sample_ternary(C.c_uint64(seed), self.N, _p(s8))
        s = s8.astype(np.int64)
        return s, self.lift_ntt(s, list(range(self.M)))

    def _gen_switch_key(self, s_ntt, sp_ntt, seed: int) -> np.ndarray:
        key = np.empty((self.dnum, 2, self.M, self.N), dtype=np.uint64)
        self.lib.orc_gen_switch_key(self.h, _p(_u64(s_ntt)), _p(_u64(sp_ntt)), C.c_uint64(seed), _p(key))
        return key

    def gen_rotation_key(self, s: np.ndarray, s_ntt: np.ndarray, offset: int, seed: int) -> np.ndarray:
        """Key switching from sigma_g(s) to s, g = 5^offset."""
        g = self.galois(offset)
        # sigma_g on the small signed coefficients: index i -> i*g mod 2N with the negacyclic sign
        sp = np.zeros(self.N, dtype=np.int64)
        e = (np.arange(self.N, dtype=np.int64) * g) % (2 * self.N)
        sp[e % self.N] = np.where(e < self.N, s, -s)
        return self._gen_switch_key(s_ntt, self.lift_ntt(sp, list(range(self.M))), seed)

    # ---- staged keys: the public half a_j is a function of a 64-bit seed ("Evaluation Keys Reuse": key sets are
    # offloaded and reloaded between block groups; only b_j and the seed have to be kept and moved)
    @staticmethod
    def splitmix64_at(seed: int, index: np.ndarray) -> np.ndarray:
        """Output number `index` (0-based) of the SplitMix64 sequence started at `seed` (Steele, Lea, Flood 2014):
        the state advances by the golden-ratio constant, so any output can be computed on its own."""
        with np.errstate(over="ignore"):
            z = np.uint64(seed) + (np.asarray(index, dtype=np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            return z ^ (z >> np.uint64(31))

    def expand_key_a(self, a_seed: int) -> np.ndarray:
        """a[j][t][x], uniform modulo the t-th modulus of the key (q_0..q_L, p_0..), evaluation form: element number
        e = (j*M + t)*N + x takes the outputs 64 e, 64 e + 1, ... of the sequence; the top bitlength(q) bits of the
        first one below q are the value (rejection sampling, so the value is exactly uniform; after 64 rejections,
        probability below 2^-64, the last output is reduced modulo q)."""
        out = np.empty((self.dnum, self.M, self.N), dtype=np.uint64)
        x = np.arange(self.N, dtype=np.uint64)
        for j in range(self.dnum):
            for t in range(self.M):
                q = self.moduli[t]
                shift = np.uint64(64 - q.bit_length())
                e = np.uint64((j * self.M + t) * self.N) + x
                val = np.zeros(self.N, dtype=np.uint64)
                todo = np.ones(self.N, dtype=bool)
                for attempt in range(64):
                    z = self.splitmix64_at(a_seed, e[todo] * np.uint64(64) + np.uint64(attempt))
                    v = z >> shift
                    ok = v < np.uint64(q)
                    idx = np.flatnonzero(todo)
                    val[idx[ok]] = v[ok]
                    if attempt == 63:
                        val[idx[~ok]] = z[~ok] % np.uint64(q)
                    todo[idx[ok]] = False
                    if not todo.any():
                        break
                out[j, t] = val
        return out

    def gen_rotation_key_seeded(self, s: np.ndarray, s_ntt: np.ndarray, offset: int, seed: int, a_seed: int) -> np.ndarray:
        """As gen_rotation_key, with the public halves a_j = expand_key_a(a_seed); the errors come from `seed`."""
        g = self.galois(offset)
        sp = np.zeros(self.N, dtype=np.int64)
        e = (np.arange(self.N, dtype=np.int64) * g) % (2 * self.N)
        sp[e % self.N] = np.where(e < self.N, s, -s)
        key = np.empty((self.dnum, 2, self.M, self.N), dtype=np.uint64)
        a = self.expand_key_a(a_seed)
        self.lib.orc_gen_switch_key_with_a(self.h, _p(_u64(s_ntt)), _p(self.lift_ntt(sp, list(range(self.M)))), C.c_uint64(seed), _p(a), _p(key))
        return key

    def mul(self, a, b, mod_idx: Sequence[int]) -> np.ndarray:
        """a (.) b, limb t modulo moduli[mod_idx[t]]; a, b [len(mod_idx)][N]."""
        a, b = _u64(a), _u64(b)
        idx = np.array(mod_idx, dtype=np.int32)
        assert a.shape == b.shape == (len(idx), self.N)
        out = np.empty_like(a)
        self.lib.orc_mul(self.h, _p(idx), len(idx), _p(a), _p(b), _p(out))
        return out

    def gen_relin_key(self, s_ntt: np.ndarray, seed: int) -> np.ndarray:
        """Key switching from s^2 to s."""
        s2 = self.mul(s_ntt, s_ntt, list(range(self.M)))
        return self._gen_switch_key(s_ntt, s2, seed)

    def encrypt_coeffs(self, m: np.ndarray, level: int, s_ntt: np.ndarray, seed: int) -> np.ndarray:
        ct = np.empty((2, level + 1, self.N), dtype=np.uint64)
        m = np.ascontiguousarray(m, dtype=np.int64)
        self.lib.orc_encrypt(self.h, level, _p(m), _p(_u64(s_ntt)), C.c_uint64(seed), _p(ct))
        return ct

    def encrypt(self, z: np.ndarray, scale: float, level: int, s_ntt: np.ndarray, seed: int) -> np.ndarray:
        return self.encrypt_coeffs(self.encode(z, scale), level, s_ntt, seed)

    def decrypt_coeffs(self, ct, level: int, s_ntt: np.ndarray) -> np.ndarray:
        ct = _u64(ct)
        assert ct.shape == (2, level + 1, self.N)
        out = np.empty(self.N, dtype=np.float64)
        self.lib.orc_decrypt(self.h, level, _p(ct), _p(_u64(s_ntt)), _p(out))
        return out

    def decrypt(self, ct, level: int, s_ntt: np.ndarray, scale: float) -> np.ndarray:
        return self.decode(self.decrypt_coeffs(ct, level, s_ntt), scale)

    # ------------------------------------------------------------- batched convolution
    def pack_channel(self, images: np.ndarray, channel: int) -> np.ndarray:
        """Channel-by-channel packing (Eqs. 3 and 5): image j's flattened channel occupies slots
        [j*m, (j+1)*m), m = H*W; needs m*b <= n (Eq. 4).  Unused slots are zero."""
        B, _, H, W = images.shape
        m = H * W
        if m * B > self.n:
            raise ValueError("slot constraint m*b <= n violated")
        z = np.zeros(self.n, dtype=np.float64)
        z[:m * B] = images[:, channel].reshape(B, m).reshape(-1)
        return z

    def unpack_channel(self, z: np.ndarray, batch: int, height: int, width: int) -> np.ndarray:
        return np.asarray(z[:batch * height * width]).reshape(batch, height, width)

    def tap_masks(self, height: int, width: int, batch: int) -> np.ndarray:
        """[9][n] 0/1 vectors, tap (dy,dx) in row-major order: 1 where the neighbour (y+dy, x+dx)
        lies inside the same image.  Replicated over the batch segments (Eq. 7)."""
        masks = np.zeros((9, self.n), dtype=np.float64)
        m = height * width
        y, x = np.divmod(np.arange(m), width)
        t = 0
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                ok = ((y + dy >= 0) & (y + dy < height) & (x + dx >= 0) & (x + dx < width)).astype(np.float64)
                masks[t, :m * batch] = np.tile(ok, batch)
                t += 1
        return masks

    def conv_operands(self, weights: np.ndarray, height: int, width: int, batch: int, level: int,
                      delta_m: float, delta_w: float) -> Tuple[np.ndarray, np.ndarray]:
        """The two factors of the weight plaintexts pt[o,c,tap] = w_int[o,c,tap] * M_tap:
        M [9][level+1][N] (NTT form, masks encoded at delta_m) and the integer weights
        w_int [C_out][C_in][9] = round(w * delta_w) as int64."""
        masks = self.tap_masks(height, width, batch)
        M = np.stack([self.encode_ntt(masks[t], delta_m, level) for t in range(9)])
        w_int = round_half_away(np.asarray(weights, dtype=np.float64).reshape(weights.shape[0], weights.shape[1], 9) * delta_w).astype(np.int64)
        return M, w_int

    def align_direct(self, ct, level: int, width: int, rot_keys: Dict[int, np.ndarray], hoisted: bool = True) -> List[np.ndarray]:
        """The nine aligned copies of one channel ciphertext, tap (dy,dx) in row-major order, each by
        its own rotation Rot(ct, dy*W+dx): eight keys, one shared decomposition when hoisted."""
        ct = _u64(ct)
        digits = self.modup(ct[1], level) if hoisted else None
        row = []
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                off = dy * width + dx
                row.append(ct if off == 0 else self.rotate(ct, level, off, rot_keys[off], hoisted, digits))
        return row

    def align_four_keys(self, ct, level: int, width: int, rot_keys: Dict[int, np.ndarray]) -> List[np.ndarray]:
        """The paper's input alignment (Eqs. 8-10) with the four keys {-1, +1, -W, +W}:
        C^-1 = Rot(ct, -1), C^+1 = Rot(ct, +1), then Rot(., -W) and Rot(., +W) of C^-1, ct, C^+1.
        Returned in the order of Eq. 10, which is the row-major tap order."""
        ct = _u64(ct)
        W = width
        d0 = self.modup(ct[1], level)                       # ct is rotated four times: one decomposition
        cm = self.rotate(ct, level, -1, rot_keys[-1], True, d0)
        cp = self.rotate(ct, level, +1, rot_keys[+1], True, d0)
        dm, dp = self.modup(cm[1], level), self.modup(cp[1], level)
        up = [self.rotate(b, level, -W, rot_keys[-W], True, d) for b, d in ((cm, dm), (ct, d0), (cp, dp))]
        down = [self.rotate(b, level, +W, rot_keys[+W], True, d) for b, d in ((cm, dm), (ct, d0), (cp, dp))]
        return up + [cm, ct, cp] + down

    # ---- the same layer with the division by P taken once, after the sum (deferred ModDown) ----------
    def special_product_residues(self, level: int) -> np.ndarray:
        """[P]_{q_i} for i <= level and 0 for the special primes: P = p_0 ... p_{k-1} on the extended basis."""
        P = 1
        for t in range(self.num_q, self.M):
            P *= self.moduli[t]
        return np.array([P % self.moduli[t] for t in self.ext_moduli_idx(level)], dtype=np.uint64)

    def scalar_residues_ext(self, value: int, level: int) -> np.ndarray:
        return np.array([int(value) % self.moduli[t] for t in self.ext_moduli_idx(level)], dtype=np.uint64)

    def scalar_mul_ext(self, poly, scalar_res, level: int) -> np.ndarray:
        """poly [n_comp, E, N] (or [E, N]) on the extended basis times an integer scalar given by residues."""
        poly = _u64(poly)
        idx = np.array(self.ext_moduli_idx(level), dtype=np.int32)
        n_comp = poly.size // (len(idx) * self.N)
        out = np.empty_like(poly)
        self.lib.orc_scalar_mul_on_moduli(self.h, _p(idx), len(idx), n_comp, _p(poly), _p(_u64(scalar_res)), _p(out))
        return out

    def mac_ext(self, pts: Sequence[np.ndarray], xs: Sequence[np.ndarray], level: int) -> np.ndarray:
        """sum_k pt_k (.) x_k on the extended basis Q_level P: pts [E][N], xs [2][E][N]."""
        idx = np.array(self.ext_moduli_idx(level), dtype=np.int32)
        E = len(idx)
        pts = [_u64(p_) for p_ in pts]
        xs = [_u64(x_) for x_ in xs]
        for p_, x_ in zip(pts, xs):
            assert p_.shape == (E, self.N) and x_.shape == (2, E, self.N)
        n = len(pts)
        out = np.empty((2, E, self.N), dtype=np.uint64)
        pa = (C.c_void_p * n)(*[p_.ctypes.data for p_ in pts])
        xa = (C.c_void_p * n)(*[x_.ctypes.data for x_ in xs])
        self.lib.orc_mac_on_moduli(self.h, _p(idx), E, n, pa, xa, _p(out), 0)
        return out

    def conv_operands_ext(self, weights: np.ndarray, height: int, width: int, batch: int, level: int,
                          delta_m: float, delta_w: float) -> Tuple[np.ndarray, np.ndarray]:
        """As conv_operands, with the mask plaintexts on the extended basis: M [9][level+1+k][N]."""
        masks = self.tap_masks(height, width, batch)
        ext = self.ext_moduli_idx(level)
        M = np.stack([self.lift_ntt(self.encode(masks[t], delta_m), ext) for t in range(9)])
        w_int = round_half_away(np.asarray(weights, dtype=np.float64).reshape(weights.shape[0], weights.shape[1], 9) * delta_w).astype(np.int64)
        return M, w_int

    def align_deferred(self, ct, level: int, width: int, rot_keys: Dict[int, np.ndarray]) -> List[np.ndarray]:
        """The nine aligned copies of one channel ciphertext BEFORE their division by P, on the
        extended basis Q_level P ([2][level+1+k][N] each): for tap offset r != 0 with g = 5^r
            X_r = (P * sigma_g(c0) + v_0,  v_1),   v = < sigma_g(ModUp(c1)), key_g >,
        so that ModDown(X_r) = Rot(ct, r); the centre tap is P * ct (zero on the special primes)."""
        ct = _u64(ct)
        digits = self.modup(ct[1], level)
        return [self.aligned_ext(ct, level, dy * width + dx, rot_keys.get(dy * width + dx), digits) for dy in (-1, 0, 1) for dx in (-1, 0, 1)]

    def aligned_ext(self, ct, level: int, off: int, key, digits) -> np.ndarray:
        """X = (P * sigma_g(c0) + v_0, v_1) on the extended basis Q_level P, v = < sigma_g(digits), key >, g = 5^off:
        Rot(ct, off) before its division by P.  off = 0: P * ct.  digits = ModUp(ct[1])."""
        ct = _u64(ct)
        L1, E = level + 1, level + 1 + self.num_p
        Pres = self.special_product_residues(level)
        x = np.zeros((2, E, self.N), dtype=np.uint64)
        if off % self.n == 0:
            x[:, :L1] = self.scalar_mul(ct, Pres[:L1], level)
        else:
            g = self.galois(off)
            v = self.key_inner(self.automorph_ntt(digits, g), key, level)
            pc0 = self.scalar_mul(self.automorph_ntt(ct[0], g), Pres[:L1], level)
            x[:] = v
            x[0, :L1] = self.add(v[0, :L1], pc0, level)
        return x

    def add_ext(self, a, b, level: int) -> np.ndarray:
        """a + b on the extended basis Q_level P, [..., level+1+k, N]."""
        a, b = _u64(a), _u64(b)
        out = np.empty_like(a)
        for e, t in enumerate(self.ext_moduli_idx(level)):
            out[..., e, :] = (a[..., e, :] + b[..., e, :]) % np.uint64(self.moduli[t])
        return out

    def he_conv_deferred(self, cts: Sequence[np.ndarray], level: int, width: int, rot_keys: Dict[int, np.ndarray],
                         M_ext: np.ndarray, w_int: np.ndarray, out_channels: Optional[Iterable[int]] = None,
                         merged: bool = False) -> Dict[int, np.ndarray]:
        """The batched convolution layer (Eqs. 10-11) with one division by P per OUTPUT channel
        instead of one per rotation:
            out_o = Rescale( ModDown( sum_c sum_tap pt[o,c,tap] (.) X_tap(ct_c) ) ),
        the sum taken on the extended basis Q_level P, X_tap as in align_deferred, the plaintexts
        pt = w_int * M_tap on that basis too.  Same slots as he_conv up to rounding noise (a little
        less of it: one rounding after the sum instead of one per term), different residues."""
        C_in = len(cts)
        aligned = [self.align_deferred(cts[c], level, width, rot_keys) for c in range(C_in)]
        outs = {}
        chans = range(w_int.shape[0]) if out_channels is None else out_channels
        for o in chans:
            pts, terms = [], []
            for c in range(C_in):
                for t in range(9):
                    pts.append(self.scalar_mul_ext(M_ext[t], self.scalar_residues_ext(int(w_int[o, c, t]), level), level))
                    terms.append(aligned[c][t])
            acc = self.mac_ext(pts, terms, level)
            if merged:   # ModDown and rescale as one division by P * q_level
                outs[o] = np.stack([self.moddown_rescale(acc[0], level), self.moddown_rescale(acc[1], level)])
            else:
                u = np.stack([self.moddown(acc[0], level), self.moddown(acc[1], level)])
                outs[o] = self.rescale(u, level)
        return outs

    def he_conv(self, cts: Sequence[np.ndarray], level: int, width: int, rot_keys: Dict[int, np.ndarray],
                M: np.ndarray, w_int: np.ndarray, out_channels: Optional[Iterable[int]] = None,
                hoisted: bool = True, four_keys: bool = False) -> Dict[int, np.ndarray]:
        """Batched 3x3 convolution layer on channel-packed ciphertexts:
        out_o = Rescale( sum_c sum_tap pt[o,c,tap] (.) R_tap(ct_c) )   (Eqs. 10-11),
        R_tap by eight direct rotations, or by the paper's four-key two-stage alignment.
        rot_keys maps the slot offset to its rotation key.  Returns {o: ct at level-1}."""
        C_in = len(cts)
        aligned = [self.align_four_keys(cts[c], level, width, rot_keys) if four_keys
                   else self.align_direct(cts[c], level, width, rot_keys, hoisted) for c in range(C_in)]
        outs = {}
        chans = range(w_int.shape[0]) if out_channels is None else out_channels
        for o in chans:
            pts, terms = [], []
            for c in range(C_in):
                for t in range(9):
                    pts.append(self.scalar_mul(M[t], self.scalar_residues(int(w_int[o, c, t]), level), level))
                    terms.append(aligned[c][t])
            acc = self.ptct_mac(pts, terms, level)
            outs[o] = self.rescale(acc, level)
        return outs

    # ---------------------------------------------------------------- accumulator (pipeline)
    def cleaning_mask(self, sts: int) -> np.ndarray:
        """The plaintext cleaning mask M of the accumulator: ones on the first `sts` slots, zeros on the rest."""
        m = np.zeros(self.n, dtype=np.float64)
        m[:sts] = 1.0
        return m

    def accumulator_merge(self, cts: Sequence[np.ndarray], level: int, sts: int, M: np.ndarray,
                          rot_keys: Dict[int, np.ndarray]) -> np.ndarray:
        """The accumulator of the optimised pipeline ("Optimized Inference Pipeline", the merge equation):
            C_joined = Rescale( sum_{i<g} Rot(C_i (.) M, -i*sts) ),
        g = len(cts) down-sampled intermediate ciphertexts whose data sit in slots [0, sts); M is the
        cleaning mask in NTT form [level+1][N]; rot_keys maps the offset -i*sts to its key.  The mask
        multiplication is followed by the rescale every plaintext product needs (the paper leaves
        scale management to the library).  Result at level-1, block i in slots [i*sts, (i+1)*sts)."""
        g = len(cts)
        if g * sts > self.n:
            raise ValueError("g * sts exceeds the slot count")
        total = None
        for i, ct in enumerate(cts):
            t = self.ptct_mac([M], [_u64(ct)], level)
            if i:
                t = self.rotate(t, level, -i * sts, rot_keys[-i * sts], True)
            total = t if total is None else self.add(total, t, level)
        return self.rescale(total, level)

    # ------------------------------------------------- slot re-layout with two rotations per element
    def relayout_two_rotations(self, ct, level: int, lo: Sequence[int], hi: Sequence[int], masks, keys: Dict[int, np.ndarray]) -> np.ndarray:
        """The two-rotation placement of the FC layer's output reconstruction ("Fully Connected Layer": every
        element moves by base_idx + mod_idx), as an operation of its own:
            out = sum_h Rot( Rescale( sum_l M[h][l] (.) Rot(ct, lo[l]) ), hi[h] ),
        an element that has to move left by lo[l] + hi[h] is selected by the mask M[h][l] (given in NTT form
        [level+1][N], or None when no element takes that pair) after its first rotation.  The first rotations
        share one decomposition of ct.  Result [2][level][N] at level-1."""
        ct = _u64(ct)
        digits = self.modup(ct[1], level)
        R = [self.rotate(ct, level, r, keys.get(r), True, digits) for r in lo]
        out = None
        for h in range(len(hi)):
            ls = [l for l in range(len(lo)) if masks[h][l] is not None]
            V = self.rescale(self.ptct_mac([masks[h][l] for l in ls], [R[l] for l in ls], level), level)
            V = self.rotate(V, level - 1, hi[h], keys.get(hi[h]), True)
            out = V if out is None else self.add(out, V, level - 1)
        return out

    def relayout_two_rotations_deferred(self, ct, level: int, lo: Sequence[int], hi: Sequence[int], masks_ext, keys: Dict[int, np.ndarray]) -> np.ndarray:
        """The same re-layout with the divisions by P deferred past the sums, as in the convolution's deferred schedule:
            X_l  = Rot(ct, lo[l]) before its division (aligned_ext, one decomposition of ct for all l);
            V_h  = ( sum_l M[h][l] (.) X_l ) / (P * q_level)           one merged division per h, level-1;
            out  = ModDown( sum_h X'_h ),  X'_h = Rot(V_h, hi[h]) before its division          one ModDown.
        masks_ext[h][l]: [level+1+k][N] on the extended basis, or None.  A first rotation costs an inner product only, so
        plans with many first and few second rotations are cheap here.  Same slots as relayout_two_rotations up to
        rounding noise, different residues.  Result [2][level][N]."""
        ct = _u64(ct)
        digits = self.modup(ct[1], level)
        X = [self.aligned_ext(ct, level, r, keys.get(r), digits) for r in lo]
        W = None
        for h in range(len(hi)):
            ls = [l for l in range(len(lo)) if masks_ext[h][l] is not None]
            acc = self.mac_ext([masks_ext[h][l] for l in ls], [X[l] for l in ls], level)
            V = np.stack([self.moddown_rescale(acc[0], level), self.moddown_rescale(acc[1], level)])
            Xh = self.aligned_ext(V, level - 1, hi[h], keys.get(hi[h]), self.modup(V[1], level - 1))
            W = Xh if W is None else self.add_ext(W, Xh, level - 1)
        return np.stack([self.moddown(W[0], level - 1), self.moddown(W[1], level - 1)])

    def downsample_plan(self, height: int, width: int, batch: int, r: int = 2, base: int = 0, rows_per_group: int = 1):
        """Slot compaction after a stride-r layer ("Optimized Inference Pipeline": H' = H/r, W' = W/r, sts' = sts/r^2;
        the paper leaves the compaction itself to its library).  Input layout: image j at slots [j*H*W, (j+1)*H*W)
        with the kept elements (y, x) = (r y', r x') at j*H*W + r*y'*W + r*x'.  Output layout: image j at slots
        [j*H'*W', (j+1)*H'*W'), everything else zero.  Two re-layouts of two rotations each:
          A (inside every image):  element (y', x') moves left by x'*(r-1) + y'*(r*W - W'); with rows_per_group = G
                                   (a divisor of H') the first rotation takes x'*(r-1) + (y' % G)*(r*W - W') and the
                                   second (y' // G)*G*(r*W - W'): G*W' first and H'/G second rotations (G = 1: W' and H');
          B (whole images):        image j moves left by j*(H*W - H'*W') = (j % base)*d [lo] + (j // base)*base*d [hi].
        Returns [(lo, hi, slot_masks)] for A and B; slot_masks[h][l] is a 0/1 vector over the n slots (the positions of
        the selected elements after their first rotation) or None."""
        assert height % r == 0 and width % r == 0 and batch * height * width <= self.n
        hw, h2, w2 = height * width, height // r, width // r
        G = rows_per_group
        assert h2 % G == 0
        base = base or int(np.ceil(np.sqrt(batch)))
        j0 = np.arange(batch) * hw
        dy = r * width - w2
        lo_a = [yl * dy + x * (r - 1) for yl in range(G) for x in range(w2)]
        hi_a = [yh * G * dy for yh in range(h2 // G)]
        masks_a = []
        for yh in range(h2 // G):
            row = []
            for yl in range(G):
                for x in range(w2):
                    m = np.zeros(self.n)
                    m[j0 + r * (yh * G + yl) * width + r * x - lo_a[yl * w2 + x]] = 1.0
                    row.append(m)
            masks_a.append(row)
        d = hw - h2 * w2
        lo_b = [l * d for l in range(min(base, batch))]
        hi_b = [h * base * d for h in range(-(-batch // base))]
        masks_b = []
        for h in range(len(hi_b)):
            row = []
            for l in range(len(lo_b)):
                j = h * base + l
                if j >= batch:
                    row.append(None)
                    continue
                m = np.zeros(self.n)
                start = j * hw - lo_b[l]
                m[start:start + h2 * w2] = 1.0
                row.append(m)
            masks_b.append(row)
        return [(lo_a, hi_a, masks_a), (lo_b, hi_b, masks_b)]

    def downsample_compact(self, ct, level: int, plan, keys: Dict[int, np.ndarray], deferred: bool = False) -> np.ndarray:
        """Runs the two re-layouts of downsample_plan; every mask is encoded at the scale of the limb its product
        drops, so the ciphertext's scale is unchanged.  Input at `level`, output [2][level-1][N] at level-2."""
        ct = _u64(ct)
        for stage, (lo, hi, slot_masks) in enumerate(plan):
            lv = level - stage
            if deferred:
                ext = self.ext_moduli_idx(lv)
                masks = [[None if m is None else self.lift_ntt(self.encode(m, float(self.moduli[lv])), ext) for m in row] for row in slot_masks]
                ct = self.relayout_two_rotations_deferred(ct, lv, lo, hi, masks, keys)
            else:
                masks = [[None if m is None else self.encode_ntt(m, float(self.moduli[lv]), lv) for m in row] for row in slot_masks]
                ct = self.relayout_two_rotations(ct, lv, lo, hi, masks, keys)
        return ct

    # ------------------------------------------- ciphertext product with the merged division
    def ctct_mul_relin_rescale(self, a, b, rlk, level: int, addend=None) -> np.ndarray:
        """Rescale(a*b + addend) with the relinearisation's division by P and the rescale's division by
        q_level merged into one (a single rounding, 48 fewer limb transforms at 24 limbs):
            (d0, d1, d2) = (a0 b0, a0 b1 + a1 b0, a1 b1),   v = < ModUp(d2), rlk >  on Q_level P,
            out_c = (v_c + P * (d_c + addend_c)) / (P * q_level),   c = 0, 1.
        a, b, addend: [2][level+1][N]; result [2][level][N]."""
        a, b = _u64(a), _u64(b)
        L1 = level + 1
        idx = list(range(L1))
        d0 = self.mul(a[0], b[0], idx)
        d1 = self.add(self.mul(a[0], b[1], idx), self.mul(a[1], b[0], idx), level)
        d2 = self.mul(a[1], b[1], idx)
        if addend is not None:
            addend = _u64(addend)
            d0, d1 = self.add(d0, addend[0], level), self.add(d1, addend[1], level)
        v = self.key_inner(self.modup(d2, level), rlk, level)
        Pres = self.special_product_residues(level)[:L1]
        out = []
        for comp, dpart in enumerate((d0, d1)):
            vc = v[comp].copy()
            vc[:L1] = self.add(vc[:L1], self.scalar_mul(dpart, Pres, level), level)
            out.append(self.moddown_rescale(vc, level))
        return np.stack(out)

    def poly_activation_merged(self, x, level: int, k: Sequence[int], rlk) -> np.ndarray:
        """The degree-7 activation of poly_activation with every relinearise-then-rescale pair replaced by
        the merged division (same levels, scales and integer scalars; other residues: one rounding per product)."""
        k1, k3, k5, k7 = [int(v) for v in k]
        x = _u64(x)
        x2 = self.ctct_mul_relin_rescale(x, x, rlk, level)                                       # level-1
        xd1 = self.drop_to_level(x, level - 1)
        x3 = self.ctct_mul_relin_rescale(x2, xd1, rlk, level - 1)                                # level-2
        x4 = self.ctct_mul_relin_rescale(x2, x2, rlk, level - 1)                                 # level-2
        l2, l3 = level - 2, level - 3
        Bp = self.add(self.scalar_mul(self.drop_to_level(x, l2), self.scalar_residues(k5, l2), l2),
                      self.scalar_mul(x3, self.scalar_residues(k7, l2), l2), l2)
        B = self.rescale(Bp, l2)                                                                 # level-3
        A = self.add(self.scalar_mul(self.drop_to_level(x, l3), self.scalar_residues(k1, l3), l3),
                     self.scalar_mul(self.drop_to_level(x3, l3), self.scalar_residues(k3, l3), l3), l3)
        return self.ctct_mul_relin_rescale(self.drop_to_level(x4, l3), B, rlk, l3, addend=A)     # level-4

    # ------------------------------------------------------------------ fully connected layer
    @staticmethod
    def fc_shifts(d_in: int, d_out: int, batch: int, base: int):
        """Offsets of the layout rotations: block j moves left by j*(d_in - d_out) = base_idx + mod_idx with
        mod_idx = (j % base) * delta and base_idx = (j // base) * base * delta (the two-key decomposition)."""
        delta = d_in - d_out
        lo = [jl * delta for jl in range(min(base, batch))]
        hi = [jh * base * delta for jh in range(-(-batch // base))]
        return delta, lo, hi

    def fc_operands(self, W: np.ndarray, bias: np.ndarray, batch: int, level: int, base: int, scale: float):
        """Plaintext operands of the batched FC layer for an input at (level, scale):
        w_enc [d_out][level+1][N]   row i of W replicated over the batch blocks, at scale q_level;
        merge_mask [level][N]       ones at the slots j*d_in (where the inner sums land), at scale q_{level-1};
        place_masks [batch][level-1][N]  block j's d_out slots after its first layout rotation, at scale q_{level-2};
        bias_pt [level-2][N]        the bias replicated at stride d_out, at the ciphertext's scale."""
        d_out, d_in = W.shape
        q = self.moduli
        delta, lo, hi = self.fc_shifts(d_in, d_out, batch, base)
        w_enc = []
        for i in range(d_out):
            z = np.zeros(self.n)
            z[:batch * d_in] = np.tile(W[i], batch)
            w_enc.append(self.encode_ntt(z, float(q[level]), level))
        z = np.zeros(self.n)
        z[np.arange(batch) * d_in] = 1.0
        merge_mask = self.encode_ntt(z, float(q[level - 1]), level - 1)
        place = []
        for j in range(batch):
            z = np.zeros(self.n)
            start = j * d_in - lo[j % base]
            z[start:start + d_out] = 1.0
            place.append(self.encode_ntt(z, float(q[level - 2]), level - 2))
        z = np.zeros(self.n)
        z[:batch * d_out] = np.tile(bias, batch)
        bias_pt = self.encode_ntt(z, scale, level - 3)
        return np.stack(w_enc), merge_mask, np.stack(place), bias_pt

    def fc_batched(self, ct, level: int, d_in: int, d_out: int, batch: int, base: int, w_enc, merge_mask, place_masks, bias_pt,
                   keys: Dict[int, np.ndarray]) -> np.ndarray:
        """Batched fully connected layer ("Fully Connected Layer": FC evaluation and output reconstruction).
        Input: block j of d_in slots holds x^(j); output (level-3): block j of d_out slots holds W x^(j) + bias.
          1. C_i = Rescale(C_in (.) w_i^enc);  S_i = Sum_{d_in}(C_i) by log2(d_in) steps T <- T + Rot(T, 2^s):
             slot j*d_in of S_i is the inner product of output i for batch element j (all j at once);
          2. Merge: U = Rescale( sum_i Rot(S_i (.) E, -i) ): element (j, i) at slot j*d_in + i, zeros elsewhere;
          3. layout: block j moves left by j*(d_in-d_out) in two rotations (mod_idx, then base_idx):
             R_l = Rot(U, l*delta) for l < base (one shared decomposition);
             V_h = Rescale( sum_l R_l (.) E'_{h*base+l} );   out = sum_h Rot(V_h, h*base*delta);
          4. out += bias^enc.
        keys maps every offset used (2^s; -i; l*delta; h*base*delta) to its rotation key."""
        ct = _u64(ct)
        assert d_in & (d_in - 1) == 0 and d_out <= d_in and batch * d_in <= self.n
        delta, lo, hi = self.fc_shifts(d_in, d_out, batch, base)
        # 1. per-output products and inner sums
        S = []
        for i in range(d_out):
            t = self.rescale(self.ptct_mac([w_enc[i]], [ct], level), level)
            step = 1
            while step < d_in:
                t = self.add(t, self.rotate(t, level - 1, step, keys[step], True), level - 1)
                step *= 2
            S.append(t)
        # 2. merge over the outputs
        U = self.accumulator_merge(S, level - 1, 1, merge_mask, {-i: keys[-i] for i in range(1, d_out)})
        # 3. layout
        l2 = level - 2
        masks = [[place_masks[h * base + l] if h * base + l < batch else None for l in range(len(lo))] for h in range(len(hi))]
        out = self.relayout_two_rotations(U, l2, lo, hi, masks, keys)
        # 4. bias
        out = out.copy()
        for i in range(l2):
            out[0, i] = (out[0, i] + bias_pt[i]) % np.uint64(self.moduli[i])
        return out

    # ----------------------------------------------------------------------- activation
    def act_schedule(self, level: int, scale: float) -> dict:
        """Levels, scales and integer scalars of the degree-7 activation evaluated on a
        ciphertext at (level, scale) with four ciphertext products:
            x2 = x*x, x3 = x2*x, x4 = x2*x2   (each rescaled once)
            B  = Rescale(k5*x + k7*x3)
            y  = Rescale((k1*x + k3*x3) + x4*B)
        The integer scalars fold the polynomial coefficients and equalise the scales."""
        q = self.moduli
        c1, c3, c5, c7 = ACT_COEFFS
        s1 = float(scale)
        s2 = s1 * s1 / q[level]            # x2 at level-1
        s3 = s2 * s1 / q[level - 1]        # x3 at level-2
        s4 = s2 * s2 / q[level - 1]        # x4 at level-2
        tB = s3 * q[level - 2]             # B before its rescale (level-2)
        k5 = int(round_half_away(np.float64(c5 * tB / s1)))
        k7 = int(round_half_away(np.float64(c7 * tB / s3)))
        sB = tB / q[level - 2]             # B at level-3
        tY = s4 * sB                       # y before its rescale (level-3)
        k1 = int(round_half_away(np.float64(c1 * tY / s1)))
        k3 = int(round_half_away(np.float64(c3 * tY / s3)))
        return dict(k=(k1, k3, k5, k7), out_level=level - 4, out_scale=tY / q[level - 3])

    def poly_activation(self, x, level: int, k: Sequence[int], rlk) -> np.ndarray:
        """Degree-7 odd polynomial with integer scalars k = (k1, k3, k5, k7) as produced by
        act_schedule; input at `level`, output at level-4."""
        k1, k3, k5, k7 = [int(v) for v in k]
        x = _u64(x)
        x2 = self.rescale(self.ctct_mul_relin(x, x, rlk, level), level)                    # level-1
        xd1 = self.drop_to_level(x, level - 1)
        x3 = self.rescale(self.ctct_mul_relin(x2, xd1, rlk, level - 1), level - 1)          # level-2
        x4 = self.rescale(self.ctct_mul_relin(x2, x2, rlk, level - 1), level - 1)           # level-2
        xd2 = self.drop_to_level(x, level - 2)
        l2 = level - 2
        Bp = self.add(self.scalar_mul(xd2, self.scalar_residues(k5, l2), l2),
                      self.scalar_mul(x3, self.scalar_residues(k7, l2), l2), l2)
        B = self.rescale(Bp, l2)                                                            # level-3
        l3 = level - 3
        A = self.add(self.scalar_mul(self.drop_to_level(x, l3), self.scalar_residues(k1, l3), l3),
                     self.scalar_mul(self.drop_to_level(x3, l3), self.scalar_residues(k3, l3), l3), l3)
        prod = self.ctct_mul_relin(self.drop_to_level(x4, l3), B, rlk, l3)
        return self.rescale(self.add(A, prod, l3), l3)                                      # level-4
