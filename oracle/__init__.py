"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Python face of the plain CPU RNS-CKKS in ``ckks_oracle.cpp`` plus the floating-point client
side (slot encoding / decoding with numpy's FFT as a library step, float64 reference
convolution, the odd degree-7 activation polynomial).  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the HIP library never does.

Paper passages followed: Background ("The CKKS Scheme": slots through the canonical embedding;
"Rotations and Key Switching"), Methodology ("Encrypted Input Representation", Eqs. 2-5: channel-
by-channel packing; "Weights Encoding", Eqs. 6-7: batch-replicated weights; "Convolution Layer",
Eqs. 8-11: aligned rotations, multiply, accumulate), "Other Layers" (polynomial activation).

Readings fixed here where the paper is silent:
  * slot j is the value of the plaintext polynomial at zeta^(5^j), zeta = exp(i*pi/N); real data
    are encoded with conjugate symmetry; Rot(ct, r) moves slot (i+r) mod n into slot i and is the
    automorphism X -> X^(5^r);
  * rounding to integers is half-away-from-zero;
  * convolution is cross-correlation with zero padding 1 and stride 1; the zero padding, the
    separation between images of a batch and the cyclic wrap are realised by 0/1 masks folded
    into the weight plaintexts: pt[o,c,tap] = w_int[o,c,tap] * M_tap with M_tap the NTT-form
    encoding of the tap's mask at scale delta_m and w_int = round(w * delta_w);
  * the activation is p(x) = (35x - 35x^3 + 21x^5 - 5x^7)/16 evaluated as
    (c1 x + c3 x^3) + x^4 (c5 x + c7 x^3) with four ciphertext products.

Parity unpinned: prime list, roots of unity and sampler streams (conventions passed explicitly).
"""
from .core import Oracle, build, conv2d_reference, activation_reference, ACT_COEFFS  # noqa: F401
