// Host-side checker of the library's double-precision modular arithmetic (paper_2604_16834_amd/csrc/f64mod.h) against
// 128-bit integer arithmetic.  Built by tests/test_f64mod.py with  g++ -O2 -ffp-contract=off -shared -fPIC.
// Two kinds of entry points:
//   run_*   evaluate the header's routines on the host (the very source the GPU kernels compile) for arrays of inputs;
//   chk_*   judge results, wherever they were computed (host or GPU), with signed 128-bit integers.
#include <stddef.h>
#include <stdint.h>

#include "../paper_2604_16834_amd/csrc/f64mod.h"

typedef __int128 i128;

static int64_t as_int(double v) { return (int64_t)v; }  // every value in play is an integer below 2^63

extern "C" {

// r[i] = mulmod(y[i], w[i], w[i] / q, q)
void run_mulmod(const int64_t* y, const uint64_t* w, uint64_t q, double* r, size_t n) {
    const double qd = (double)q;
    for (size_t i = 0; i < n; i++) r[i] = f64m_mulmod((double)y[i], (double)w[i], (double)w[i] / qd, qd);
}
void run_mulmod_any(const int64_t* y, const uint64_t* w, uint64_t q, double* r, size_t n) {
    const double qd = (double)q, qinv = 1.0 / qd;
    for (size_t i = 0; i < n; i++) r[i] = f64m_mulmod_any((double)y[i], (double)w[i], qd, qinv);
}
void run_reduce(const int64_t* v, uint64_t q, double* r, size_t n) {
    const double qd = (double)q, qinv = 1.0 / qd;
    for (size_t i = 0; i < n; i++) r[i] = f64m_reduce((double)v[i], qd, qinv);
}
// canonical(reduce(v)) as the kernels' last store does
void run_canonical(const int64_t* v, uint64_t q, uint64_t* r, size_t n) {
    const double qd = (double)q, qinv = 1.0 / qd;
    for (size_t i = 0; i < n; i++) r[i] = f64m_canonical(f64m_reduce((double)v[i], qd, qinv), qd);
}
void run_from_to_u64(const uint64_t* v, uint64_t* r, size_t n) {
    for (size_t i = 0; i < n; i++) r[i] = f64m_to_u64(f64m_from_u64(v[i]));
}
// the centred store of the inverse transform in front of a basis conversion: centre(mulmod(v, k, k/q, q))
void run_centre(const int64_t* v, uint64_t k, uint64_t q, double* r, size_t n) {
    const double qd = (double)q;
    for (size_t i = 0; i < n; i++) r[i] = f64m_centre(f64m_mulmod((double)v[i], (double)k, (double)k / qd, qd), qd);
}
// the basis-conversion sum of nd terms (rows of y: [n][nd]; one row of constants cw[nd]), nd in {1, 4, 8, 9, 12, 16}
int run_dot(const int64_t* y, const uint64_t* cw, uint32_t nd, uint64_t q, double* r, size_t n) {
    const double qd = (double)q, qinv = 1.0 / qd;
    TwF c[16];
    double yv[16];
    if (nd > 16) return -1;
    for (uint32_t a = 0; a < nd; a++) {  // the constant's centred representative, as the library's tables hold it
        const double w = cw[a] > (q >> 1) ? -(double)(q - cw[a]) : (double)cw[a];
        c[a] = TwF{w, w / qd};
    }
    for (size_t i = 0; i < n; i++) {
        for (uint32_t a = 0; a < nd; a++) yv[a] = (double)y[i * nd + a];
        switch (nd) {
            case 1: r[i] = f64m_dot<1>(yv, c, qd, qinv); break;
            case 4: r[i] = f64m_dot<4>(yv, c, qd, qinv); break;
            case 8: r[i] = f64m_dot<8>(yv, c, qd, qinv); break;
            case 9: r[i] = f64m_dot<9>(yv, c, qd, qinv); break;
            case 12: r[i] = f64m_dot<12>(yv, c, qd, qinv); break;
            case 16: r[i] = f64m_dot<16>(yv, c, qd, qinv); break;
            default: return -1;
        }
    }
    return 0;
}
// three forward butterfly stages on eight values (a round of the transforms), then the round's reduction; returns the
// largest multiplicand magnitude seen, so that the caller can check the "below 2^51" precondition along the way
static double fwd_round(int64_t* v8, const uint64_t* tw7, uint64_t q, bool value_only);
double run_fwd_round(int64_t* v8, const uint64_t* tw7, uint64_t q) { return fwd_round(v8, tw7, q, false); }
// the same with twiddles given as values alone (the quotient from the rounded product: f64m_mulmod_any)
double run_fwd_round_any(int64_t* v8, const uint64_t* tw7, uint64_t q) { return fwd_round(v8, tw7, q, true); }
static double fwd_round(int64_t* v8, const uint64_t* tw7, uint64_t q, bool value_only) {
    const double qd = (double)q, qinv = 1.0 / qd;
    double v[8], worst = 0.0;
    for (int j = 0; j < 8; j++) v[j] = (double)v8[j];
    for (int a = 0; a < 3; a++) {
        const int half = 8 >> (a + 1);
        for (int rr = 0; rr < 8; rr++) {
            if (rr & half) continue;
            const double w = (double)tw7[(1 << a) - 1 + (rr >> (3 - a))];
            const double y = v[rr + half];
            if (__builtin_fabs(y) > worst) worst = __builtin_fabs(y);
            const double t = value_only ? f64m_mulmod_any(y, w, qd, qinv) : f64m_mulmod(y, w, w / qd, qd);
            v[rr + half] = v[rr] - t;
            v[rr] = v[rr] + t;
        }
    }
    for (int j = 0; j < 8; j++) v8[j] = as_int(f64m_reduce(v[j], qd, qinv));
    return worst;
}

// ---- judges ----------------------------------------------------------------------------------------------------
// r[i] must be an integer with r = y*w (mod q) and |r| * den <= num * q (the documented bound num/den of q).
// Returns the index of the first failure, or -1; *worst_ratio = max |r| / q seen.
long chk_product(const int64_t* y, const uint64_t* w, const double* r, uint64_t q, size_t n, uint32_t num, uint32_t den, double* worst_ratio) {
    double worst = 0.0;
    for (size_t i = 0; i < n; i++) {
        const int64_t ri = as_int(r[i]);
        if ((double)ri != r[i]) return (long)i;
        const i128 diff = (i128)y[i] * (i128)w[i] - (i128)ri;
        if (diff % (i128)q != 0) return (long)i;
        const i128 mag = ri < 0 ? -(i128)ri : (i128)ri;
        if (mag * den > (i128)num * q) return (long)i;
        const double ratio = (double)mag / (double)q;
        if (ratio > worst) worst = ratio;
    }
    if (worst_ratio) *worst_ratio = worst;
    return -1;
}
// r[i] = v[i] (mod q), |r| <= q/2 + 1
long chk_reduce(const int64_t* v, const double* r, uint64_t q, size_t n) {
    for (size_t i = 0; i < n; i++) {
        const int64_t ri = as_int(r[i]);
        if ((double)ri != r[i]) return (long)i;
        if (((i128)v[i] - ri) % (i128)q != 0) return (long)i;
        const i128 mag = ri < 0 ? -(i128)ri : (i128)ri;
        if (2 * mag > (i128)q + 2) return (long)i;
    }
    return -1;
}
// r[i] = v[i] mod q in [0, q)
long chk_canonical(const int64_t* v, const uint64_t* r, uint64_t q, size_t n) {
    for (size_t i = 0; i < n; i++) {
        i128 m = (i128)v[i] % (i128)q;
        if (m < 0) m += q;
        if ((i128)r[i] != m) return (long)i;
    }
    return -1;
}
// r[i] = v[i]*k (mod q), -q/2 < r < q/2
long chk_centre(const int64_t* v, uint64_t k, const double* r, uint64_t q, size_t n) {
    for (size_t i = 0; i < n; i++) {
        const int64_t ri = as_int(r[i]);
        if ((double)ri != r[i]) return (long)i;
        if (((i128)v[i] * k - ri) % (i128)q != 0) return (long)i;
        const i128 mag = ri < 0 ? -(i128)ri : (i128)ri;
        if (2 * mag > (i128)q) return (long)i;
    }
    return -1;
}
// r[i] = sum_a y[i][a] * cw[a] (mod q), |r| <= q/2 + 1
long chk_dot(const int64_t* y, const uint64_t* cw, uint32_t nd, const double* r, uint64_t q, size_t n) {
    for (size_t i = 0; i < n; i++) {
        i128 s = 0;
        for (uint32_t a = 0; a < nd; a++) s += (i128)y[i * nd + a] * (i128)cw[a] % (i128)q;
        const int64_t ri = as_int(r[i]);
        if ((double)ri != r[i]) return (long)i;
        if ((s - ri) % (i128)q != 0) return (long)i;
        const i128 mag = ri < 0 ? -(i128)ri : (i128)ri;
        if (2 * mag > (i128)q + 2) return (long)i;
    }
    return -1;
}
// the same round with exact integers: out8 = the eight results mod q in [0, q)
void ref_fwd_round(const int64_t* v8, const uint64_t* tw7, uint64_t q, uint64_t* out8) {
    i128 v[8];
    for (int j = 0; j < 8; j++) v[j] = v8[j];
    for (int a = 0; a < 3; a++) {
        const int half = 8 >> (a + 1);
        for (int rr = 0; rr < 8; rr++) {
            if (rr & half) continue;
            const i128 t = v[rr + half] * (i128)tw7[(1 << a) - 1 + (rr >> (3 - a))] % (i128)q;
            v[rr + half] = v[rr] - t;
            v[rr] = v[rr] + t;
        }
    }
    for (int j = 0; j < 8; j++) {
        i128 m = v[j] % (i128)q;
        if (m < 0) m += q;
        out8[j] = (uint64_t)m;
    }
}

// three inverse butterfly stages on eight reduced values (a round of the inverse transforms: sum re-centred, difference
// times the twiddle), with the twiddle's quotient precomputed or with its value alone; returns the largest multiplicand seen
static double inv_round(int64_t* v8, const uint64_t* tw7, uint64_t q, bool value_only) {
    const double qd = (double)q, qinv = 1.0 / qd;
    double v[8], worst = 0.0;
    for (int j = 0; j < 8; j++) v[j] = (double)v8[j];
    for (int a = 2; a >= 0; a--) {
        const int half = 8 >> (a + 1);
        for (int rr = 0; rr < 8; rr++) {
            if (rr & half) continue;
            const double w = (double)tw7[(1 << a) - 1 + (rr >> (3 - a))];
            const double s = v[rr] + v[rr + half], d = v[rr] - v[rr + half];
            if (__builtin_fabs(d) > worst) worst = __builtin_fabs(d);
            v[rr] = f64m_reduce(s, qd, qinv);
            v[rr + half] = value_only ? f64m_mulmod_any(d, w, qd, qinv) : f64m_mulmod(d, w, w / qd, qd);
        }
    }
    for (int j = 0; j < 8; j++) v8[j] = as_int(v[j]);
    return worst;
}
double run_inv_round(int64_t* v8, const uint64_t* tw7, uint64_t q) { return inv_round(v8, tw7, q, false); }
double run_inv_round_any(int64_t* v8, const uint64_t* tw7, uint64_t q) { return inv_round(v8, tw7, q, true); }
void ref_inv_round(const int64_t* v8, const uint64_t* tw7, uint64_t q, uint64_t* out8) {
    i128 v[8];
    for (int j = 0; j < 8; j++) v[j] = v8[j];
    for (int a = 2; a >= 0; a--) {
        const int half = 8 >> (a + 1);
        for (int rr = 0; rr < 8; rr++) {
            if (rr & half) continue;
            const i128 s = v[rr] + v[rr + half], d = v[rr] - v[rr + half];
            v[rr] = s % (i128)q;
            v[rr + half] = d % (i128)q * (i128)tw7[(1 << a) - 1 + (rr >> (3 - a))] % (i128)q;
        }
    }
    for (int j = 0; j < 8; j++) {
        i128 m = v[j] % (i128)q;
        if (m < 0) m += q;
        out8[j] = (uint64_t)m;
    }
}

// the fold of nd digit diagonals (rows of D: [n][nd] 32-bit signed; constants c[nd] < q), nd in {9, 10, 13}: the parts
// of the constants and the multiplier 2^17 mod q are formed here the way the library's table holds them
int run_fold(const int32_t* D, const uint64_t* c, uint32_t nd, uint64_t q, double* r, size_t n) {
    const double qd = (double)q, qinv = 1.0 / qd;
    double cp[39];
    if (nd > 13) return -1;
    for (uint32_t s = 0; s < nd; s++) {
        cp[3 * s] = (double)(c[s] & 0x1ffffu);
        cp[3 * s + 1] = (double)((c[s] >> 17) & 0x1ffffu);
        cp[3 * s + 2] = (double)(c[s] >> 34);
    }
    const uint64_t w17 = 131072 % q;
    const double w17d = (double)w17, w17q = w17d / qd;
    for (size_t i = 0; i < n; i++) {
        const int* row = (const int*)(D + i * nd);
        switch (nd) {
            case 9: r[i] = f64m_fold_diagonals<9>(row, cp, w17d, w17q, qd, qinv); break;
            case 10: r[i] = f64m_fold_diagonals<10>(row, cp, w17d, w17q, qd, qinv); break;
            case 13: r[i] = f64m_fold_diagonals<13>(row, cp, w17d, w17q, qd, qinv); break;
            default: return -1;
        }
    }
    return 0;
}

// r[i] is an integer, |r[i]| <= q/2 + 1, congruent to sum_s D[i][s] * c[s]; returns the number of failures
long chk_fold(const int32_t* D, const uint64_t* c, uint32_t nd, const double* r, uint64_t q, size_t n) {
    long bad = 0;
    for (size_t i = 0; i < n; i++) {
        i128 want = 0;
        for (uint32_t s = 0; s < nd; s++) want += (i128)D[i * nd + s] * (i128)c[s];
        const i128 got = (i128)as_int(r[i]);
        const bool integral = (double)as_int(r[i]) == r[i];
        const bool small = got <= (i128)(q / 2 + 1) && got >= -(i128)(q / 2 + 1);
        const bool congruent = ((want - got) % (i128)q) == 0;
        if (!(integral && small && congruent)) bad++;
    }
    return bad;
}

}  // extern "C"
