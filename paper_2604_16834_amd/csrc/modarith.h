// 64-bit modular arithmetic for gfx950 (device) and for table building (host).
//
// Everything the NTT, the basis conversions and the pointwise kernels do is made of these few
// routines (RNS limbs of word size: Background, "RNS Decomposition and NTT Optimization").
// Moduli are primes below 2^58.  Two reduction schemes:
//   * Shoup: multiplication by a constant w with a precomputed quotient w' = floor(w * 2^64 / q);
//     result in [0, 2q) for any 64-bit multiplicand (twiddles, conversion constants, scalars);
//   * Barrett on a 128-bit value: x < 2^(62 + bits(q)), quotient estimated from the top 64 bits
//     with mu = floor(2^(62 + bits(q)) / q); estimate is at most 2 too small, result made canonical.
//     Sums of products are accumulated unreduced in 128 bits and reduced once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;

// Per-modulus constants, passed to kernels by value or read from a device table.
struct ModConst {
    u64 q;
    u64 mu;      // floor(2^(64 + sh) / q)
    u32 sh;      // bits(q) - 2
    u32 pad;
    u64 n_inv;   // N^-1 mod q
    u64 n_inv_sh;
};

__host__ __device__ __forceinline__ u64 mulhi64(u64 a, u64 b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (u64)(((unsigned __int128)a * b) >> 64);
#endif
}

struct U128 {
    u64 lo, hi;
};

__host__ __device__ __forceinline__ U128 mul_wide(u64 a, u64 b) {
    U128 r;
    r.lo = a * b;
    r.hi = mulhi64(a, b);
    return r;
}

__host__ __device__ __forceinline__ void acc_wide(U128& acc, u64 a, u64 b) {
    u64 lo = a * b;
    u64 hi = mulhi64(a, b);
    acc.lo += lo;
    acc.hi += hi + (acc.lo < lo ? 1ull : 0ull);
}

// canonical residue of a 128-bit value below 2^(62 + bits(q))
__host__ __device__ __forceinline__ u64 barrett_reduce(U128 x, const ModConst& m) {
    u64 x1 = (x.hi << (64 - m.sh)) | (x.lo >> m.sh);
    u64 qe = mulhi64(x1, m.mu);
    u64 r = x.lo - qe * m.q;  // true value is below 3q, so the low word is all of it
    if (r >= 2 * m.q) r -= 2 * m.q;
    if (r >= m.q) r -= m.q;
    return r;
}

__host__ __device__ __forceinline__ u64 mulmod_barrett(u64 a, u64 b, const ModConst& m) {
    return barrett_reduce(mul_wide(a, b), m);
}

// reduce a single word (any 64-bit value) to [0, q)
__host__ __device__ __forceinline__ u64 reduce_word(u64 a, const ModConst& m) {
    U128 x;
    x.lo = a;
    x.hi = 0;
    return barrett_reduce(x, m);
}

// a * w mod q up to one extra q: result in [0, 2q); w_sh = floor(w * 2^64 / q)
__host__ __device__ __forceinline__ u64 mul_shoup_lazy(u64 a, u64 w, u64 w_sh, u64 q) {
    u64 t = mulhi64(a, w_sh);
    return a * w - t * q;
}

__host__ __device__ __forceinline__ u64 mul_shoup(u64 a, u64 w, u64 w_sh, u64 q) {
    u64 r = mul_shoup_lazy(a, w, w_sh, q);
    return r >= q ? r - q : r;
}

__host__ __device__ __forceinline__ u64 add_mod(u64 a, u64 b, u64 q) {
    u64 s = a + b;
    return s >= q ? s - q : s;
}

__host__ __device__ __forceinline__ u64 sub_mod(u64 a, u64 b, u64 q) {
    return a >= b ? a - b : a + q - b;
}

// ---- carry-free accumulation of products of residues below 2^50 ------------------------------
// Each operand is split into 25-bit halves (l, h) and their sum s; one product costs three
// 32x32+64 multiply-adds (Karatsuba) into three plain 64-bit sums, so up to 4096 products can be
// accumulated without a single carry:  sum xl*wl, sum xh*wh, sum (xl+xh)*(wl+wh) < 2^64.
struct Split50 {
    u32 l, h, s;
};
struct Acc50 {
    u64 ll, hh, kk;
};
#define ACC50_MAX_TERMS 4096u

__host__ __device__ __forceinline__ Split50 split50(u64 v) {
    Split50 r;
    r.l = (u32)v & 0x1ffffffu;
    r.h = (u32)(v >> 25);
    r.s = r.l + r.h;
    return r;
}

__host__ __device__ __forceinline__ void acc50_mad(Acc50& a, const Split50& x, const Split50& w) {
    a.ll += (u64)x.l * w.l;
    a.hh += (u64)x.h * w.h;
    a.kk += (u64)x.s * w.s;
}

// the accumulated sum as a 128-bit integer: hh*2^50 + (kk - ll - hh)*2^25 + ll
__host__ __device__ __forceinline__ U128 acc50_value(const Acc50& a) {
    const u64 mid = a.kk - a.ll - a.hh;
    U128 r;
    r.lo = a.ll;
    r.hi = 0;
    u64 t = mid << 25;
    r.lo += t;
    r.hi += (mid >> 39) + (r.lo < t ? 1ull : 0ull);
    t = a.hh << 50;
    r.lo += t;
    r.hi += (a.hh >> 14) + (r.lo < t ? 1ull : 0ull);
    return r;
}
