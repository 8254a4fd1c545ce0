// Exact modular arithmetic on integers held in doubles, for moduli below 2^50 (device code only).
// y * w - q * round(y * w / q) is computed without rounding error from the rounded product h = y*w, its exact error
// l = fma(y, w, -h), and the quotient c = the integer nearest to y * (w / q): fma(-c, q, h) + l, of magnitude below
// 0.63 q.  Needs |y| < 2^51, 0 <= w < q < 2^50, wq = w / q rounded to nearest.  Sums of such terms stay exact below 2^53.
#pragma once
#include "ctx.h"

#pragma clang fp contract(off)  // every product and sum as written

#define F64M_MAGIC 6755399441055744.0  // 1.5 * 2^52: adding it rounds to the nearest integer (magnitudes below 2^51)
#define F64M_2P52 4503599627370496.0

__device__ __forceinline__ double f64m_mulmod(double y, double w, double wq, double q) {
    const double h = y * w;
    const double l = __builtin_fma(y, w, -h);
    const double c = __builtin_fma(y, wq, F64M_MAGIC) - F64M_MAGIC;
    return __builtin_fma(-c, q, h) + l;
}
// v - q * round(v / q) for an integer |v| < 2^53: magnitude at most q/2 + 1
__device__ __forceinline__ double f64m_reduce(double v, double q, double qinv) {
    return __builtin_fma(-(__builtin_fma(v, qinv, F64M_MAGIC) - F64M_MAGIC), q, v);
}
// a residue below 2^52 as a double, through the mantissa of 2^52 + v
__device__ __forceinline__ double f64m_from_u64(u64 v) { return __longlong_as_double((long long)(v | 0x4330000000000000ull)) - F64M_2P52; }
// |v| <= q/2 + 1 -> the canonical residue in [0, q)
__device__ __forceinline__ u64 f64m_canonical(double v, double q) {
    const double p = v < 0.0 ? v + q : v;
    return (u64)__double_as_longlong(p + F64M_2P52) & 0x000fffffffffffffull;
}
