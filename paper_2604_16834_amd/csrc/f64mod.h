// Exact modular arithmetic on integers held in doubles, for moduli below 2^50.
//
// This is the one copy of the arithmetic that the double-precision butterflies, the basis conversions inside the
// transforms and the fused inner products are made of.  It has no dependency but <stdint.h> and compiles for the GPU
// (hipcc) and for the host (any C++ compiler, with floating-point contraction switched off: -ffp-contract=off), so that
// a CPU test can compare every routine with 128-bit integer arithmetic on boundary values and on random ones.
//
//   y * w - q * round(y * w / q) is computed without rounding error from the rounded product h = y*w, its exact error
//   l = fma(y, w, -h), and a quotient c that is an integer within 3/4 of y*w/q:  fma(-c, q, h) + l.
//   The quotient comes from y * (w / q) when w / q is precomputed (a twiddle, a conversion constant: mulmod), or from
//   h * (1 / q) when the multiplier is data (a key word, a ciphertext residue: mulmod_any).  Adding 1.5 * 2^52 inside a
//   fused multiply-add rounds the exact product to the nearest integer, so c is off by at most 1/2 plus the error of the
//   factor w / q (relative 2^-53) or of h and 1 / q (relative 2^-53 each).
// Bounds (q < 2^50, all values integers):
//   mulmod      |y| < 2^51, 0 <= w < q, wq = w / q rounded to nearest   ->  |result| <= (1/2 + |y| / 2^53) q  < 3/4 q
//   mulmod_any  |y| < q,    0 <= w < q, qinv = 1 / q rounded to nearest ->  |result| <= (1/2 + |y| / 2^52) q  < 3/4 q
//   reduce      |v| < 2^53                                              ->  |result| <= q/2 + 1
// (for reduced multiplicands, |y| <= q/2 + 1: below 0.57 q and 0.63 q).  h - c q is an integer below 2^51 and l one below
// 2^48, so the last two operations are exact.  A sum of up to eight products stays below 2^53 and is exact, and three
// forward butterfly stages after a reduce keep every multiplicand below 2q + 1 < 2^51.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define F64M_FN __host__ __device__ __forceinline__
#pragma clang fp contract(off)  // every product and sum as written
#else
#define F64M_FN static inline
#endif

#define F64M_MAGIC 6755399441055744.0  // 1.5 * 2^52: adding it rounds to the nearest integer (magnitudes below 2^51)
#define F64M_2P52 4503599627370496.0

// a constant multiplier as a double with its quotient by the modulus (w / q rounded to nearest), one 16-byte word
struct __attribute__((aligned(16))) TwF {
    double w, wq;
};

F64M_FN double f64m_bits_to_double(uint64_t b) {
    double d;
    __builtin_memcpy(&d, &b, 8);
    return d;
}
F64M_FN uint64_t f64m_double_to_bits(double d) {
    uint64_t b;
    __builtin_memcpy(&b, &d, 8);
    return b;
}

// the integer nearest to v * c (|v * c| < 2^51), from the exact product: one rounding only
F64M_FN double f64m_round_mul(double v, double c) { return __builtin_fma(v, c, F64M_MAGIC) - F64M_MAGIC; }

// v - q * round(v / q) for an integer |v| < 2^53: magnitude at most q/2 + 1
F64M_FN double f64m_reduce(double v, double q, double qinv) { return __builtin_fma(-f64m_round_mul(v, qinv), q, v); }

// y * w - q * c with c the integer nearest to y * wq
F64M_FN double f64m_mulmod(double y, double w, double wq, double q) {
    const double h = y * w;
    const double l = __builtin_fma(y, w, -h);
    const double c = f64m_round_mul(y, wq);
    return __builtin_fma(-c, q, h) + l;
}

// the same for a multiplier without a precomputed w / q: the quotient comes from the rounded product (|y| < 2q: the quotient
// is at most 1/2 + |y| / 2^52 off, the result at most q in magnitude)
F64M_FN double f64m_mulmod_any(double y, double w, double q, double qinv) {
    const double h = y * w;
    const double l = __builtin_fma(y, w, -h);
    const double c = f64m_round_mul(h, qinv);
    return __builtin_fma(-c, q, h) + l;
}

// canonical residues below 2^52 <-> doubles through the mantissa of 2^52 + v
F64M_FN double f64m_from_u64(uint64_t v) { return f64m_bits_to_double(v | 0x4330000000000000ull) - F64M_2P52; }
F64M_FN uint64_t f64m_to_u64(double v) { return f64m_double_to_bits(v + F64M_2P52) & 0x000fffffffffffffull; }

// |v| <= q/2 + 1 (more generally -q <= v < q) -> the canonical residue in [0, q)
F64M_FN uint64_t f64m_canonical(double v, double q) { return f64m_to_u64(v < 0.0 ? v + q : v); }

// |t| < q (the result of a product) -> the centred representative in (-q/2, q/2); q is odd: no residue on the boundary
F64M_FN double f64m_centre(double t, double q) {
    const double half = 0.5 * q;
    return t > half ? t - q : (t < -half ? t + q : t);
}

// sum_{a < ND} y[a] * cw[a].w  mod q  as a reduced double, for centred operands: |y[a]| < 2^49 (centred residues of a
// modulus below 2^50) and |cw[a].w| < 2^49 (the constant's centred representative; cw[a].wq is not read): the basis-conversion
// sum.  Terms are taken in chains of up to eight.  A chain's running sum T starts at 1.5 * 2^102 and takes each product
// with one fused multiply-add: the chain's sum stays below 2^101 in magnitude, so T stays in its binade and every step rounds
// the exact sum to a multiple of 2^50.  D = T_new - T_old is exact; the step's remainder y w - D is an integer of magnitude at
// most 2^49, which a second fused multiply-add gives exactly, and eight of them add up exactly (at most 2^52).  The chain's
// high part T - 1.5 * 2^102, an exact multiple of 2^50, has a quotient by q below 2^51 in magnitude (2 max|y|), which
// rint(high * (1/q)) misses by at most one; high - quotient * q, below 2q, is exact, the low part is added (below 2^53:
// exact) and the sum reduced.  Four instructions per term, where a product reduced on its own takes seven.
// A row of nine terms (the division by P q_l: eight special primes and the dropped limb) is one chain too: only the ninth
// step can take T past 2^103, where it rounds to a multiple of 2^51 and leaves a remainder of at most 2^50; D, the high
// part and the sum of the remainders (at most 8 * 2^49 + 2^50) are still exact, the quotient stays below 2^52.
#define F64M_DOT_BASE 0x1.8p+102  /* 1.5 * 2^102 */
template <int ND>
F64M_FN double f64m_dot_w(const double* y, const double* w, double q, double qinv) {  // w[a]: the centred constants
    constexpr int CHAIN = ND == 9 ? 9 : 8;
    double r = 0.0;
#pragma unroll
    for (int a0 = 0; a0 < ND; a0 += CHAIN) {
        double t = F64M_DOT_BASE, lo = 0.0;
#pragma unroll
        for (int a = a0; a < a0 + CHAIN && a < ND; a++) {
            const double tn = __builtin_fma(y[a], w[a], t);
            const double d = tn - t;
            lo += __builtin_fma(y[a], w[a], -d);
            t = tn;
        }
        const double hi = t - F64M_DOT_BASE;
        const double c = __builtin_rint(hi * qinv);
        const double v = f64m_reduce(__builtin_fma(-c, q, hi) + lo, q, qinv);
        r = a0 == 0 ? v : f64m_reduce(r + v, q, qinv);
    }
    return r;
}
template <int ND>
F64M_FN double f64m_dot(const double* y, const TwF* cw, double q, double qinv) {
    double w[ND];
#pragma unroll
    for (int a = 0; a < ND; a++) w[a] = cw[a].w;
    return f64m_dot_w<ND>(y, w, q, qinv);
}

// sum_s D[s] * c[s]  mod q  as a reduced double, for 32-bit signed D[s] and ND <= 13 constants c[s] < q given in three
// parts, c[s] = c0[s] + 2^17 c1[s] + 2^34 c2[s] with c0, c1 < 2^17 and c2 < 2^16 (the digit diagonals of a sum of 8-bit
// digit products and the powers of 256 they stand for).  Each of the three sums of ND products is below
// 13 * 2^31 * 2^17 < 2^52 in magnitude, so it is exact; the sums are joined by Horner's rule with the multiplier
// w17 = 2^17 mod q (w17q = w17 / q rounded to nearest), every multiplicand reduced first so that any modulus from 3 up works.
// cparts: [ND][3] doubles.
template <int ND>
F64M_FN double f64m_fold_diagonals(const int* D, const double* cparts, double w17, double w17q, double q, double qinv) {
    static_assert(ND <= 13, "the three partial sums must stay below 2^52");
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int s = 0; s < ND; s++) {
        const double ds = (double)D[s];
        s0 = __builtin_fma(ds, cparts[3 * s], s0);
        s1 = __builtin_fma(ds, cparts[3 * s + 1], s1);
        s2 = __builtin_fma(ds, cparts[3 * s + 2], s2);
    }
    const double t = f64m_mulmod(f64m_reduce(s2, q, qinv), w17, w17q, q);
    const double u = f64m_mulmod(f64m_reduce(t + s1, q, qinv), w17, w17q, q);
    return f64m_reduce(u + s0, q, qinv);
}
