"""RNS-CKKS parameter sets for the synthetic workloads.

The paper fixes only the ring (X^N + 1, N a power of two; Background, "The CKKS Scheme"), that
the modulus is a chain of word-size NTT-friendly primes ("RNS Decomposition and NTT
Optimization") and that key switching uses digits (Experiments, "HE Security Parameters").  The
concrete primes and roots are conventions chosen here and handed, explicitly, to both the CPU
oracle and the HIP library, so neither side derives them on its own:

* primes: walk downwards from 2^bits over the candidates that are 1 mod 2N, keep the ones that
  pass a deterministic Miller-Rabin test; the first ``num_p`` found are the special primes (the
  largest ones, so that P exceeds every digit product), the next ``num_q`` are q_0 .. q_L;
* root: for each prime the smallest x >= 2 whose power x^((q-1)/2N) has order exactly 2N.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List

_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)  # deterministic below 3.3e24


def is_prime(n: int) -> bool:
    if n < 2:
        return False
    for p in _MR_BASES:
        if n % p == 0:
            return n == p
    d, s = n - 1, 0
    while d % 2 == 0:
        d //= 2
        s += 1
    for a in _MR_BASES:
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(s - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def ntt_primes(log_n: int, count: int, bits: int = 50) -> List[int]:
    """The ``count`` largest primes below 2^bits that are 1 modulo 2N, in decreasing order."""
    two_n = 2 << log_n
    cand = ((1 << bits) - 1) // two_n * two_n + 1
    if cand >= (1 << bits):
        cand -= two_n
    out: List[int] = []
    while len(out) < count:
        if cand < (1 << (bits - 1)):
            raise ValueError("ran out of candidates")
        if is_prime(cand):
            out.append(cand)
        cand -= two_n
    return out


def primitive_2n_root(q: int, log_n: int) -> int:
    """Smallest-generator choice of a primitive 2N-th root of unity modulo the prime q."""
    two_n = 2 << log_n
    n = 1 << log_n
    assert (q - 1) % two_n == 0
    x = 2
    while True:
        psi = pow(x, (q - 1) // two_n, q)
        if pow(psi, n, q) == q - 1:
            return psi
        x += 1


@dataclass(frozen=True)
class CkksParams:
    log_n: int
    num_q: int          # ciphertext limbs L+1
    num_p: int          # special primes k
    dnum: int           # key-switch digits
    moduli: tuple       # q_0..q_L, p_0..p_{k-1}
    psi: tuple          # primitive 2N-th root per modulus
    log_scale: int = 40

    @property
    def n(self) -> int:
        return 1 << self.log_n

    @property
    def slots(self) -> int:
        return 1 << (self.log_n - 1)

    @property
    def alpha(self) -> int:
        return -(-self.num_q // self.dnum) if self.dnum else 0

    @property
    def top_level(self) -> int:
        return self.num_q - 1


def make_params(log_n: int, num_q: int, num_p: int, dnum: int, bits: int = 50,
                log_scale: int = 40) -> CkksParams:
    primes = ntt_primes(log_n, num_q + num_p, bits)
    special, chain = primes[:num_p], primes[num_p:]
    moduli = tuple(chain + special)
    psi = tuple(primitive_2n_root(q, log_n) for q in moduli)
    return CkksParams(log_n, num_q, num_p, dnum, moduli, psi, log_scale)


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload (the five benchmark configurations plus scaled-down
    versions of them that the CPU oracle finishes in seconds)."""
    name: str
    log_n: int
    num_q: int
    num_p: int
    dnum: int
    height: int = 0
    width: int = 0
    batch: int = 0
    c_in: int = 0
    c_out: int = 0
    n_rot: int = 0
    ntt_batch: int = 0
    extra: dict = field(default_factory=dict)

    def params(self) -> CkksParams:
        return make_params(self.log_n, self.num_q, self.num_p, self.dnum)


CONFIGS: Dict[str, Workload] = {
    # single 3x3 conv on one 8x8 image; two special primes so that alpha = 2 digits are covered by P
    "cfg1_single_conv": Workload("cfg1_single_conv", 12, 4, 2, 2, 8, 8, 1, 1, 1),
    # the same with the single special prime of the literal statement (limb parity only)
    "cfg1_single_conv_k1": Workload("cfg1_single_conv_k1", 12, 4, 1, 2, 8, 8, 1, 1, 1),
    "cfg2_ntt": Workload("cfg2_ntt", 16, 30, 0, 0, ntt_batch=64),
    "cfg3_rotations": Workload("cfg3_rotations", 16, 24, 8, 3, n_rot=64),
    "cfg4_resnet20_stage1": Workload("cfg4_resnet20_stage1", 16, 20, 7, 3, 32, 32, 32, 16, 16),
    "cfg5_resnet20_stage3": Workload("cfg5_resnet20_stage3", 16, 24, 8, 3, 8, 8, 512, 64, 64),
    # scaled-down shapes for element-by-element parity (several tiles, ragged digit, seconds on CPU)
    "small_rotations": Workload("small_rotations", 13, 7, 3, 3, n_rot=6),
    "small_conv": Workload("small_conv", 13, 5, 2, 3, 8, 8, 64, 3, 2),
    "small_block": Workload("small_block", 12, 8, 3, 3, 8, 8, 32, 2, 2),
    # 64 input channels (9 * 64 = 576 terms, a whole number of 64-term blocks) and 40 outputs (both 32-channel output tiles live):
    # the instantiation of the multiply-accumulate that the block-slice benchmark runs, at a size the oracle affords
    "small_conv_c64": Workload("small_conv_c64", 12, 4, 2, 2, 8, 8, 32, 64, 40),
    # a ring below the transforms' tile size (N = 2^10: single-kernel transforms, stand-alone conversions) with 50-bit primes
    "tiny_ring_conv": Workload("tiny_ring_conv", 10, 4, 2, 2, 8, 8, 8, 2, 2),
    # six one-limb digits: more than the fused multi-rotation launches take (the one-launch-per-tap paths)
    "small_conv_d6": Workload("small_conv_d6", 12, 6, 2, 6, 8, 8, 32, 3, 2),
}
