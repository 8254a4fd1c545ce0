// Hybrid (digit-decomposed) key switching for gfx950: the arithmetic behind every Rot and every
// relinearisation (Background, "Rotations and Key Switching"; Experiments, "HE Security
// Parameters": key switching with digits).
//
//   ModUp      digit j's limbs (coefficient form) -> all live q-limbs and the special primes:
//              y_a = [c_a * (Q_j/q_a)^-1] mod q_a  taken centred in [-(q_a-1)/2, (q_a-1)/2],
//              d_j[t] = sum_a y_a * [Q_j/q_a]_t  mod t          (plain sum, no correction term).
//              Computed on the unsigned residues plus  (#negative y_a) * (-Q_j mod t), which is
//              the same integer modulo t because q_a * (Q_j/q_a) = Q_j.
//   inner      v_comp[t] = sum_j sigma_g(d_j)[t] * key[j][comp][t]   (sigma_g = gather, g = 1: none)
//   ModDown    z_a = [v_{p_a} * (P/p_a)^-1] mod p_a centred,  w[i] = sum_a z_a * [P/p_a]_{q_i}
//              (coefficient form, same negative-count trick with -P mod q_i), then in NTT form
//              u[i] = (v[q_i] - w[i]) * P^-1  (+ an optional addend)
// Sums of products are accumulated unreduced in 128 bits and reduced once.
#include "ctx.h"
#include "f64mod.h"
#include "galois.h"

#define KS_THREADS 256
#define KS_MAX_DIGIT 16  // limbs per digit / special primes handled in registers

// row [N] of (batch item b, digit j, extended-basis position e): see DigitSrc
__device__ __forceinline__ const u64* digit_row(const DigitSrc& D, u32 b, u32 j, u32 e, u32 E, u32 N, u32 level) {
    if (e <= level && e / D.alpha == j) return D.own.p[b] + (size_t)e * N;
    return D.digits + b * D.bstride + ((size_t)j * E + e) * N;
}

// ---- ModUp: basis extension of one digit --------------------------------------------------------
// y     [nd][N]      digit limbs in coefficient form (canonical)
// c_in  [level+1][N] the polynomial being switched, NTT form (source of the digit's own limbs)
// digit [E][N]       out: own limbs copied (NTT form), other limbs in coefficient form
__global__ __launch_bounds__(KS_THREADS) void modup_conv_kernel(const u64* __restrict__ y, size_t y_bstride, PtrList8 c_list,
                                                                u64* __restrict__ digit, size_t digit_bstride,
                                                                const u64* __restrict__ tab, const ModConst* __restrict__ mc, u32 N,
                                                                u32 level, u32 num_q, u32 lo, u32 nd, u32 alpha, u32 M, u32 E, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    y += blockIdx.z * y_bstride;
    digit += blockIdx.z * digit_bstride;
    const u64* __restrict__ c_in = c_list.p[blockIdx.z];
    u64 yv[KS_MAX_DIGIT];
    u64 n_neg = 0;
#pragma unroll
    for (u32 a = 0; a < KS_MAX_DIGIT; a++)
        if (a < nd) {
            const u64 qa = mc[lo + a].q;
            yv[a] = mul_shoup(y[(size_t)a * N + x], tab[a], tab[alpha + a], qa);
            n_neg += yv[a] > (qa >> 1) ? 1 : 0;
        }
    const u64* negq = tab + (size_t)alpha * (2 + M);  // alpha = padded row length here
    const u32 e0 = blockIdx.y * lpb;
    for (u32 e = e0; e < e0 + lpb && e < E; e++) {
        const u32 t = e <= level ? e : num_q + (e - level - 1);
        if (t >= lo && t < lo + nd) continue;  // the digit's own limbs are read from the polynomial itself (DigitSrc)
        U128 acc = {0, 0};
#pragma unroll
        for (u32 a = 0; a < KS_MAX_DIGIT; a++)
            if (a < nd) acc_wide(acc, yv[a], tab[2 * alpha + (size_t)e * alpha + a]);
        acc_wide(acc, n_neg, negq[e]);
        digit[(size_t)e * N + x] = barrett_reduce(acc, mc[t]);
    }
}

// ModUp for moduli below 2^50: carry-free 25-bit-split accumulation (three multiply-adds per term).
// AP = padded digit size: the AP constants of a target limb are one aligned run (wide scalar load).
template <int AP>
__global__ __launch_bounds__(KS_THREADS) void modup_conv50_kernel(const u64* __restrict__ y, size_t y_bstride, PtrList8 c_list,
                                                                  u64* __restrict__ digit, size_t digit_bstride,
                                                                  const u64* __restrict__ tab, const ModConst* __restrict__ mc, u32 N,
                                                                  u32 level, u32 num_q, u32 lo, u32 nd, u32 M, u32 E, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    y += blockIdx.z * y_bstride;
    digit += blockIdx.z * digit_bstride;
    const u64* __restrict__ c_in = c_list.p[blockIdx.z];
    Split50 yv[AP];
    u32 n_neg = 0;
#pragma unroll
    for (u32 a = 0; a < AP; a++) {
        yv[a] = {0, 0, 0};
        if (a < nd) {
            const u64 qa = mc[lo + a].q;
            const u64 v = mul_shoup(y[(size_t)a * N + x], tab[a], tab[AP + a], qa);
            n_neg += v > (qa >> 1) ? 1 : 0;
            yv[a] = split50(v);
        }
    }
    const u64* conv = (const u64*)__builtin_assume_aligned(tab + 2 * AP, 8 * AP);
    const u64* negq = tab + (size_t)AP * (2 + M);
    const u32 e0 = blockIdx.y * lpb;
    for (u32 e = e0; e < e0 + lpb && e < E; e++) {
        const u32 t = e <= level ? e : num_q + (e - level - 1);
        if (t >= lo && t < lo + nd) continue;  // the digit's own limbs are read from the polynomial itself (DigitSrc)
        const u64* ce = (const u64*)__builtin_assume_aligned(conv + (size_t)e * AP, 8 * AP);
        u64 cv[AP];
#pragma unroll
        for (u32 a = 0; a < AP; a++) cv[a] = ce[a];
        Acc50 acc = {0, 0, 0};
#pragma unroll
        for (u32 a = 0; a < AP; a++) acc50_mad(acc, yv[a], split50(cv[a]));
        U128 v = acc50_value(acc);
        acc_wide(v, n_neg, negq[e]);
        digit[(size_t)e * N + x] = barrett_reduce(v, mc[t]);
    }
}

// ModUp for moduli below 2^50 in double precision: the centred residues of the digit as doubles, every term reduced by
// an exact fused-multiply-add product (f64mod.h), the sum of at most 8 terms (below 2^53) reduced once.  About 60
// full-rate instructions per target residue where the split integer sum takes about 90; no correction for the negative
// terms is needed, their representatives are negative doubles.  convf: [E][AP] (constant, constant / target modulus).
template <int AP>
__global__ __launch_bounds__(KS_THREADS) void modup_conv_f64_kernel(const u64* __restrict__ y, size_t y_bstride, PtrList8 c_list,
                                                                    u64* __restrict__ digit, size_t digit_bstride,
                                                                    const u64* __restrict__ tab, const TwF* __restrict__ convf,
                                                                    const ModConst* __restrict__ mc, const ModConstF* __restrict__ mcf,
                                                                    u32 N, u32 level, u32 num_q, u32 lo, u32 nd, u32 E, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    y += blockIdx.z * y_bstride;
    digit += blockIdx.z * digit_bstride;
    const u64* __restrict__ c_in = c_list.p[blockIdx.z];
    double yd[AP];
#pragma unroll
    for (u32 a = 0; a < AP; a++) {
        yd[a] = 0.0;
        if (a < nd) {
            const u64 qa = mc[lo + a].q;
            const u64 v = mul_shoup(y[(size_t)a * N + x], tab[a], tab[AP + a], qa);
            yd[a] = v > (qa >> 1) ? -f64m_from_u64(qa - v) : f64m_from_u64(v);
        }
    }
    const u32 e0 = blockIdx.y * lpb;
    for (u32 e = e0; e < e0 + lpb && e < E; e++) {
        const u32 t = e <= level ? e : num_q + (e - level - 1);
        if (t >= lo && t < lo + nd) continue;  // the digit's own limbs are read from the polynomial itself (DigitSrc)
        const TwF* ce = (const TwF*)__builtin_assume_aligned(convf + (size_t)e * AP, 16 * AP);
        const double q = mcf[t].q, qinv = mcf[t].qinv;
        digit[(size_t)e * N + x] = f64m_canonical(f64m_dot<AP>(yd, ce, q, qinv), q);
    }
}

// n <= KS_MAX_BATCH polynomials at once: item b reads y + b*y_bstride and c_in.p[b], writes digit + b*digit_bstride
hipError_t launch_modup_conv(const ckks_ctx* c, u32 level, u32 j, const u64* y, size_t y_bstride, const PtrList8& c_in, u64* digit,
                             size_t digit_bstride, u32 n, hipStream_t st) {
    const u32 E = c->ext_limbs(level), lo = c->digit_lo(j), nd = c->digit_hi(j, level) - lo;
    // target limbs per thread: the digit's prepared residues are reused for all of them, but a small batch needs the
    // limbs spread over more workgroups to fill the chip
    const u32 x_wgs = (c->N + KS_THREADS - 1) / KS_THREADS;
    const u32 lpb = x_wgs * n >= 1024 ? 32 : (x_wgs * n >= 512 ? 8 : 4);
    dim3 grid(x_wgs, (E + lpb - 1) / lpb, n);
    const u64* tab = c->modup_table(level, j);
    ProfScope ps__(c, K_MODUP_CONV, st, 8.0 * n * c->N * (2.0 * nd + E), (double)n * c->N * nd * (1.0 + E - nd));
    if (c->ntt_f64 && c->d_modup_f) {
        const TwF* tf = c->modup_table_f(level, j);
        if (c->alpha_pad == 4)
            hipLaunchKernelGGL(modup_conv_f64_kernel<4>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, tf, c->d_mc, c->d_mcf, c->N, level, c->num_q, lo, nd, E, lpb);
        else if (c->alpha_pad == 8)
            hipLaunchKernelGGL(modup_conv_f64_kernel<8>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, tf, c->d_mc, c->d_mcf, c->N, level, c->num_q, lo, nd, E, lpb);
        else
            hipLaunchKernelGGL(modup_conv_f64_kernel<16>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, tf, c->d_mc, c->d_mcf, c->N, level, c->num_q, lo, nd, E, lpb);
    } else if (c->small_q) {
        if (c->alpha_pad == 4)
            hipLaunchKernelGGL(modup_conv50_kernel<4>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, c->d_mc, c->N, level, c->num_q, lo, nd, c->M, E, lpb);
        else if (c->alpha_pad == 8)
            hipLaunchKernelGGL(modup_conv50_kernel<8>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, c->d_mc, c->N, level, c->num_q, lo, nd, c->M, E, lpb);
        else
            hipLaunchKernelGGL(modup_conv50_kernel<16>, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, c->d_mc, c->N, level, c->num_q, lo, nd, c->M, E, lpb);
    } else {
        hipLaunchKernelGGL(modup_conv_kernel, grid, dim3(KS_THREADS), 0, st, y, y_bstride, c_in, digit, digit_bstride, tab, c->d_mc,
                           c->N, level, c->num_q, lo, nd, c->alpha_pad, c->M, E, lpb);
    }
    return hipGetLastError();
}

// ---- inner product with the switching key ------------------------------------------------------
// digits [beta][E][N], key [dnum][2][M][N], v [2][E][N]
__global__ __launch_bounds__(KS_THREADS) void key_inner_kernel(DigitSrc digits, const u64* __restrict__ key,
                                                               u64* __restrict__ v, const ModConst* __restrict__ mc, u32 log_n,
                                                               u32 level, u32 num_q, u32 M, u32 E, u32 beta, u32 g) {
    const u32 N = 1u << log_n;
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y;
    const u32 t = e <= level ? e : num_q + (e - level - 1);
    const u32 xs = g == 1 ? x : galois_gather_index(x, g, log_n);
    U128 acc0 = {0, 0}, acc1 = {0, 0};
    const ModConst m = mc[t];
    for (u32 j = 0; j < beta; j++) {
        const u64 d = digit_row(digits, 0, j, e, E, N, level)[xs];
        acc_wide(acc0, d, key[(((size_t)j * 2 + 0) * M + t) * N + x]);
        acc_wide(acc1, d, key[(((size_t)j * 2 + 1) * M + t) * N + x]);
        if ((j & 15) == 15) {  // keep the unreduced sums inside the Barrett input range
            acc0.lo = barrett_reduce(acc0, m); acc0.hi = 0;
            acc1.lo = barrett_reduce(acc1, m); acc1.hi = 0;
        }
    }
    v[((size_t)0 * E + e) * N + x] = barrett_reduce(acc0, m);
    v[((size_t)1 * E + e) * N + x] = barrett_reduce(acc1, m);
}

hipError_t launch_key_inner(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g, u64* v, hipStream_t st) {
    const u32 E = c->ext_limbs(level);
    dim3 grid((c->N + KS_THREADS - 1) / KS_THREADS, E);
    { ProfScope ps__(c, K_KEY_INNER, st, 8.0 * c->N * E * (3.0 * c->live_digits(level) + 2.0), 2.0 * c->N * E * c->live_digits(level)); hipLaunchKernelGGL(key_inner_kernel, grid, dim3(KS_THREADS), 0, st, digits, key, v, c->d_mc, c->log_n, level, c->num_q,
                       c->M, E, c->live_digits(level), g); }
    return hipGetLastError();
}

// The same key applied to n <= KS_MAX_BATCH sets of digits (the channels of a layer share their
// rotation and relinearisation keys): every thread keeps its key words while it walks the batch, so
// the key streams from HBM once per batch instead of once per key switch.
// digits + b*digits_bstride: [beta][E][N];  v + b*v_bstride: [2][E][N]
// F64 (every modulus below 2^50, at most four digits): the sums as chains of fused multiply-adds on centred doubles
// (f64m_dot_w), as in the fused taps.
template <bool F64>
__global__ __launch_bounds__(KS_THREADS) void key_inner_multi_kernel(DigitSrc digits, const u64* __restrict__ key, u64* __restrict__ v,
                                                                     size_t v_bstride, const ModConst* __restrict__ mc, u32 log_n,
                                                                     u32 level, u32 num_q, u32 M, u32 E, u32 beta, u32 g, u32 n,
                                                                     const ModConstF* __restrict__ mcf) {
    const u32 N = 1u << log_n;
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y;
    const u32 t = e <= level ? e : num_q + (e - level - 1);
    const u32 xs = g == 1 ? x : galois_gather_index(x, g, log_n);
    const ModConst m = mc[t];
    if constexpr (F64) {  // beta <= 4: entries past the last digit are zero on both sides
        const double qd = mcf[t].q, qinv = mcf[t].qinv, halfq = 0.5 * qd;
        auto centred = [&](u64 w) {
            const double d = f64m_from_u64(w);
            return d > halfq ? d - qd : d;
        };
        double w0[4], w1[4];
#pragma unroll
        for (u32 j = 0; j < 4; j++) {
            w0[j] = j < beta ? centred(key[(((size_t)j * 2 + 0) * M + t) * N + x]) : 0.0;
            w1[j] = j < beta ? centred(key[(((size_t)j * 2 + 1) * M + t) * N + x]) : 0.0;
        }
        for (u32 b = 0; b < n; b++) {
            double y[4];
#pragma unroll
            for (u32 j = 0; j < 4; j++) y[j] = j < beta ? centred(digit_row(digits, b, j, e, E, N, level)[xs]) : 0.0;
            u64* vb = v + b * v_bstride;
            vb[((size_t)0 * E + e) * N + x] = f64m_canonical(f64m_dot_w<4>(y, w0, qd, qinv), qd);
            vb[((size_t)1 * E + e) * N + x] = f64m_canonical(f64m_dot_w<4>(y, w1, qd, qinv), qd);
        }
        return;
    }
    if (beta <= 4) {
        // the thread's key words stay in registers for the whole batch
        u64 k0[4], k1[4];
#pragma unroll
        for (u32 j = 0; j < 4; j++) {
            k0[j] = j < beta ? key[(((size_t)j * 2 + 0) * M + t) * N + x] : 0;
            k1[j] = j < beta ? key[(((size_t)j * 2 + 1) * M + t) * N + x] : 0;
        }
        for (u32 b = 0; b < n; b++) {
            U128 acc0 = {0, 0}, acc1 = {0, 0};
#pragma unroll
            for (u32 j = 0; j < 4; j++) {
                const u64 dv = j < beta ? digit_row(digits, b, j, e, E, N, level)[xs] : 0;
                acc_wide(acc0, dv, k0[j]);
                acc_wide(acc1, dv, k1[j]);
            }
            u64* vb = v + b * v_bstride;
            vb[((size_t)0 * E + e) * N + x] = barrett_reduce(acc0, m);
            vb[((size_t)1 * E + e) * N + x] = barrett_reduce(acc1, m);
        }
        return;
    }
    for (u32 b = 0; b < n; b++) {
        U128 acc0 = {0, 0}, acc1 = {0, 0};
        for (u32 j = 0; j < beta; j++) {
            const u64 dv = digit_row(digits, b, j, e, E, N, level)[xs];
            acc_wide(acc0, dv, key[(((size_t)j * 2 + 0) * M + t) * N + x]);
            acc_wide(acc1, dv, key[(((size_t)j * 2 + 1) * M + t) * N + x]);
            if ((j & 15) == 15) {
                acc0.lo = barrett_reduce(acc0, m); acc0.hi = 0;
                acc1.lo = barrett_reduce(acc1, m); acc1.hi = 0;
            }
        }
        u64* vb = v + b * v_bstride;
        vb[((size_t)0 * E + e) * N + x] = barrett_reduce(acc0, m);
        vb[((size_t)1 * E + e) * N + x] = barrett_reduce(acc1, m);
    }
}

hipError_t launch_key_inner_multi(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g,
                                  u64* v, size_t v_bstride, u32 n, hipStream_t st) {
    const u32 E = c->ext_limbs(level), beta = c->live_digits(level);
    dim3 grid((c->N + KS_THREADS - 1) / KS_THREADS, E);
    ProfScope ps__(c, K_KEY_INNER, st, 8.0 * c->N * E * (2.0 * beta + n * (beta + 2.0)), 2.0 * n * c->N * E * beta);
    if (c->small_q && beta <= 4)
        hipLaunchKernelGGL(key_inner_multi_kernel<true>, grid, dim3(KS_THREADS), 0, st, digits, key, v, v_bstride, c->d_mc,
                           c->log_n, level, c->num_q, c->M, E, beta, g, n, c->d_mcf);
    else
        hipLaunchKernelGGL(key_inner_multi_kernel<false>, grid, dim3(KS_THREADS), 0, st, digits, key, v, v_bstride, c->d_mc,
                           c->log_n, level, c->num_q, c->M, E, beta, g, n, c->d_mcf);
    return hipGetLastError();
}

// The inner product of a batch, finished for an operation that divides by P later (the convolution that
// takes one ModDown per output channel after its sum; the ciphertext product whose ModDown is merged with
// the rescale): on all E limbs of the extended basis,
//   out_b[comp][e][x] = mask[e][x] * ( v_b[comp][e][x] + (e <= level ? [P]_{q_e} * add_comp,b[e][sigma_g x] : 0) )
// add0 / add1 [level+1][N] (optional) are what the result of the key switch would have been added to
// (Rot: c0; relinearisation: d0, d1); P times them vanishes on the special primes and joins the
// unreduced 128-bit sum as one more term.  mask [E][N] (optional): a plaintext on the extended basis.
struct ExtItems {
    const u64* add0[KS_MAX_BATCH];
    const u64* add1[KS_MAX_BATCH];
    u64* out[KS_MAX_BATCH];
};

__global__ __launch_bounds__(KS_THREADS) void key_inner_ext_kernel(DigitSrc digits, const u64* __restrict__ key, ExtItems items,
                                                                   const u64* __restrict__ mask, const u64* __restrict__ negp,
                                                                   const ModConst* __restrict__ mc, u32 log_n, u32 level, u32 num_q,
                                                                   u32 M, u32 E, u32 beta, u32 g, u32 n) {
    const u32 N = 1u << log_n;
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y;
    const u32 t = e <= level ? e : num_q + (e - level - 1);
    const u32 xs = g == 1 ? x : galois_gather_index(x, g, log_n);
    const ModConst m = mc[t];
    const bool has_mask = mask != nullptr;
    const u64 mk = has_mask ? mask[(size_t)e * N + x] : 0;
    const bool has_add = e <= level;
    const u64 pres = has_add ? m.q - negp[e] : 0;  // P mod q_e
    u64 k0[4], k1[4];  // beta <= 4: the thread's key words stay in registers for the whole batch
    if (beta <= 4) {
#pragma unroll
        for (u32 j = 0; j < 4; j++) {
            k0[j] = j < beta ? key[(((size_t)j * 2 + 0) * M + t) * N + x] : 0;
            k1[j] = j < beta ? key[(((size_t)j * 2 + 1) * M + t) * N + x] : 0;
        }
    }
    for (u32 b = 0; b < n; b++) {
        U128 acc0 = {0, 0}, acc1 = {0, 0};
        if (beta <= 4) {
#pragma unroll
            for (u32 j = 0; j < 4; j++) {
                const u64 dv = j < beta ? digit_row(digits, b, j, e, E, N, level)[xs] : 0;
                acc_wide(acc0, dv, k0[j]);
                acc_wide(acc1, dv, k1[j]);
            }
        } else {
            for (u32 j = 0; j < beta; j++) {
                const u64 dv = digit_row(digits, b, j, e, E, N, level)[xs];
                acc_wide(acc0, dv, key[(((size_t)j * 2 + 0) * M + t) * N + x]);
                acc_wide(acc1, dv, key[(((size_t)j * 2 + 1) * M + t) * N + x]);
                if ((j & 15) == 15) {
                    acc0.lo = barrett_reduce(acc0, m); acc0.hi = 0;
                    acc1.lo = barrett_reduce(acc1, m); acc1.hi = 0;
                }
            }
        }
        if (has_add && items.add0[b]) acc_wide(acc0, items.add0[b][(size_t)e * N + xs], pres);
        if (has_add && items.add1[b]) acc_wide(acc1, items.add1[b][(size_t)e * N + xs], pres);
        u64 r0 = barrett_reduce(acc0, m), r1 = barrett_reduce(acc1, m);
        if (has_mask) {
            r0 = mulmod_barrett(r0, mk, m);
            r1 = mulmod_barrett(r1, mk, m);
        }
        u64* ob = items.out[b];
        ob[((size_t)0 * E + e) * N + x] = r0;
        ob[((size_t)1 * E + e) * N + x] = r1;
    }
}

// add0s / add1s / outs: host arrays of n <= KS_MAX_BATCH device pointers ([level+1][N], [level+1][N], [2][E][N]);
// add0s, add1s or single entries of them may be null
hipError_t launch_key_inner_ext(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g,
                                const u64* const* add0s, const u64* const* add1s, const u64* mask, u64* const* outs, u32 n,
                                hipStream_t st) {
    const u32 E = c->ext_limbs(level), beta = c->live_digits(level);
    ExtItems items;
    double n_add = 0.0;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) {
        items.add0[b] = (b < n && add0s) ? add0s[b] : nullptr;
        items.add1[b] = (b < n && add1s) ? add1s[b] : nullptr;
        items.out[b] = b < n ? outs[b] : nullptr;
        n_add += (items.add0[b] ? 1.0 : 0.0) + (items.add1[b] ? 1.0 : 0.0);
    }
    const u64* negp = c->d_moddown + 2 * c->k_pad + (size_t)c->k_pad * c->num_q + 2 * c->num_q;
    dim3 grid((c->N + KS_THREADS - 1) / KS_THREADS, E);
    ProfScope ps__(c, K_KEY_INNER, st, 8.0 * c->N * (E * (2.0 * beta + (mask ? 1.0 : 0.0) + n * (beta + 2.0)) + n_add * (level + 1.0)),
                   2.0 * n * c->N * E * (beta + 1.0));
    hipLaunchKernelGGL(key_inner_ext_kernel, grid, dim3(KS_THREADS), 0, st, digits, key, items, mask, negp, c->d_mc,
                       c->log_n, level, c->num_q, c->M, E, beta, g, n);
    return hipGetLastError();
}

// All the taps of a convolution for a batch of input channels in one launch: the same arithmetic as
// key_inner_ext_kernel (P * sigma_g(c0) added, tap mask multiplied in) for up to 8 (key, Galois element,
// mask) triples, organised by SOURCE point: a thread loads the digits and c0 of one evaluation point of
// every batch item once (coalesced) and, for each tap, sends them to the point sigma_g^-1 maps it to,
// where it reads the key and the mask and writes the result.  sigma_g maps every aligned run of 2^m
// points onto an aligned run of 2^m points, so a wavefront's 64 destinations are one 512-byte run,
// permuted inside: key reads and result writes are as coalesced as unpermuted ones.  The digits stream
// from HBM once per batch instead of once per tap, with no reliance on a cache.
// result of (item b, tap i): term k0 + b * k_bstride + tap[i] of xs in layout xl
struct TapSet {
    const u64* key[8];
    const u64* mask[8];
    u32 ginv[8];  // inverse Galois elements: the destination of source point x under sigma_g is gather(x, g^-1)
    u32 tap[8];
    u32 n_taps;
    const u64* centre_mask;  // the tap without a rotation (P * ct times this mask), or null
    u32 centre_tap;
};

// The tap's mask is folded into the key before the batch runs: mk[i][j][comp][e][x] = mask_i[e][x] * key_i[j][comp][t(e)][x]
// on the live digits and limbs, mp[i][e][x] = mask_i[e][x] * [P]_{q_e} for e <= level.  Then
//   mask * (sum_j d_j key_j + P c0) = sum_j d_j mk_j + c0 mp
// is one unreduced sum with one reduction per result: the per-result mask product (half of the arithmetic)
// is gone.  Costs one pass over the eight keys per call.
__global__ __launch_bounds__(KS_THREADS) void mask_keys_kernel(TapSet T, u64* __restrict__ mk, u64* __restrict__ mp,
                                                               const u64* __restrict__ negp, const ModConst* __restrict__ mc, u32 N,
                                                               u32 level, u32 num_q, u32 M, u32 E, u32 beta) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y, i = blockIdx.z;
    const u32 t = e <= level ? e : num_q + (e - level - 1);
    const ModConst m = mc[t];
    if (i == T.n_taps) {  // the centre tap has no key: only mask * P
        if (e <= level) mp[((size_t)i * (level + 1) + e) * N + x] = mulmod_barrett(T.centre_mask[(size_t)e * N + x], m.q - negp[e], m);
        return;
    }
    const u64 mv = T.mask[i] ? T.mask[i][(size_t)e * N + x] : 1;  // no mask: the key as it is, and P
    for (u32 j = 0; j < beta; j++)
        for (u32 comp = 0; comp < 2; comp++)
            mk[((((size_t)i * beta + j) * 2 + comp) * E + e) * N + x] = mulmod_barrett(mv, T.key[i][(((size_t)j * 2 + comp) * M + t) * N + x], m);
    if (e <= level) mp[((size_t)i * (level + 1) + e) * N + x] = mulmod_barrett(mv, m.q - negp[e], m);
}

// F64: every modulus below 2^50: the sums of BETA + 1 products as chains of fused multiply-adds on centred doubles (f64m_dot_w:
// four full-rate operations per term where a split integer sum takes three quarter-rate 64-bit multiply-adds and the splits:
// 117 registers instead of 232, 776 us instead of 904 for eight ciphertexts and nine taps at N = 2^16); the digits and the
// ciphertext's words are centred once per thread, a tap's key words once per tap.  Otherwise 128-bit integer sums.
template <int BETA, bool F64>
__global__ __launch_bounds__(KS_THREADS) void key_inner_taps_kernel(DigitSrc digits, TapSet T,
                                                                    const u64* __restrict__ mk, const u64* __restrict__ mp,
                                                                    PtrList8 c0s, u64* __restrict__ xs, XLayout xl, u32 k0base,
                                                                    u32 k_bstride, const ModConst* __restrict__ mc, u32 log_n,
                                                                    u32 level, u32 num_q, u32 E, u32 n, u32 M, const u64* __restrict__ negp,
                                                                    const ModConstF* __restrict__ mcf) {
    // negp != nullptr: no masks; the keys are read where they are (T.key[i]: [dnum][2][M][N]) and mask * P is P itself
    const u32 N = 1u << log_n;
    const u32 xsrc = blockIdx.x * KS_THREADS + threadIdx.x;
    if (xsrc >= N) return;
    const u32 e = blockIdx.y;
    const u32 t = e <= level ? e : num_q + (e - level - 1);
    const ModConst m = mc[t];
    const bool has_add = e <= level;
    const bool direct = negp != nullptr;
    const u64 pres = (direct && has_add) ? m.q - negp[e] : 0;  // P mod q_e
    u64 dv[CT_BATCH][BETA], cv[CT_BATCH];
#pragma unroll
    for (u32 b = 0; b < CT_BATCH; b++) {
        const bool on = b < n;
        cv[b] = (on && has_add) ? c0s.p[b][(size_t)e * N + xsrc] : 0;
#pragma unroll
        for (u32 j = 0; j < BETA; j++) dv[b][j] = on ? digit_row(digits, b, j, e, E, N, level)[xsrc] : 0;
    }
    // F64: the centred representative of a residue as a double
    const double qd = F64 ? mcf[t].q : 0.0, qinv = F64 ? mcf[t].qinv : 0.0, halfq = 0.5 * qd;
    auto centred = [&](u64 v) {
        const double d = f64m_from_u64(v);
        return d > halfq ? d - qd : d;
    };
    double yd[CT_BATCH][BETA + 1];  // F64: digits and the ciphertext's word of every batch item
    if (F64) {
#pragma unroll
        for (u32 b = 0; b < CT_BATCH; b++) {
#pragma unroll
            for (u32 j = 0; j < BETA; j++) yd[b][j] = centred(dv[b][j]);
            yd[b][BETA] = centred(cv[b]);
        }
    }
    for (u32 i = 0; i < T.n_taps; i++) {
        const u32 x = galois_gather_index(xsrc, T.ginv[i], log_n);  // destination point
        u64 k0[BETA], k1[BETA];
#pragma unroll
        for (u32 j = 0; j < BETA; j++) {
            const u64* kb = direct ? T.key[i] + (((size_t)j * 2) * M + t) * N + x : mk + ((((size_t)i * BETA + j) * 2) * E + e) * N + x;
            k0[j] = kb[0];
            k1[j] = kb[(size_t)(direct ? M : E) * N];
        }
        const u64 kp = direct ? pres : (has_add ? mp[((size_t)i * (level + 1) + e) * N + x] : 0);
        u64* ot = xs + xl.at(k0base + T.tap[i], 0, e, x);
        if (F64) {
            double w0[BETA + 1], w1[BETA];
#pragma unroll
            for (u32 j = 0; j < BETA; j++) { w0[j] = centred(k0[j]); w1[j] = centred(k1[j]); }
            w0[BETA] = centred(kp);  // zero on the special primes
#pragma unroll
            for (u32 b = 0; b < CT_BATCH; b++) {
                if (b < n) {
                    u64* ob = ot + (size_t)b * k_bstride * xl.s_k;
                    ob[0] = f64m_canonical(f64m_dot_w<BETA + 1>(yd[b], w0, qd, qinv), qd);
                    ob[xl.s_comp] = f64m_canonical(f64m_dot_w<BETA>(yd[b], w1, qd, qinv), qd);
                }
            }
        } else {
#pragma unroll
            for (u32 b = 0; b < CT_BATCH; b++) {
                if (b < n) {
                    U128 acc0 = {0, 0}, acc1 = {0, 0};
#pragma unroll
                    for (u32 j = 0; j < BETA; j++) {
                        acc_wide(acc0, dv[b][j], k0[j]);
                        acc_wide(acc1, dv[b][j], k1[j]);
                    }
                    acc_wide(acc0, cv[b], kp);
                    u64* ob = ot + (size_t)b * k_bstride * xl.s_k;
                    ob[0] = barrett_reduce(acc0, m);
                    ob[xl.s_comp] = barrett_reduce(acc1, m);
                }
            }
        }
    }
    if (T.centre_mask) {  // no rotation: mask * P * ct on the live limbs, zero on the special primes
        const u64 kp = has_add ? mp[((size_t)T.n_taps * (level + 1) + e) * N + xsrc] : 0;
        u64* ot = xs + xl.at(k0base + T.centre_tap, 0, e, xsrc);
#pragma unroll
        for (u32 b = 0; b < CT_BATCH; b++) {
            if (b < n) {
                const u64 c1 = has_add ? c0s.p[b][((size_t)(level + 1) + e) * N + xsrc] : 0;
                u64* ob = ot + (size_t)b * k_bstride * xl.s_k;
                ob[0] = has_add ? mulmod_barrett(cv[b], kp, m) : 0;
                ob[xl.s_comp] = has_add ? mulmod_barrett(c1, kp, m) : 0;
            }
        }
    }
}

// words of scratch launch_key_inner_taps needs (the masked keys)
size_t key_inner_taps_scratch_elems(const ckks_ctx* c, u32 level, u32 n_taps) {
    return (size_t)n_taps * c->N * ((size_t)c->live_digits(level) * 2 * c->ext_limbs(level) + level + 1) + (size_t)c->N * (level + 1);
}

// keys / gs / masks / taps: n_taps <= 8 entries (taps[i] = position of tap i in the output's tap stride);
// c0s: n <= CT_BATCH device pointers [level+1][N]; scratch: key_inner_taps_scratch_elems() words, filled by
// prepare (once per set of taps) and read by every later call with prepare = false.
// Needs beta <= 4 (returns hipErrorNotSupported otherwise: the caller then falls back to one launch per tap).
hipError_t launch_key_inner_taps(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* const* keys,
                                 const u32* gs, const u64* const* masks, const u32* taps, u32 n_taps, const u64* const* c0s,
                                 u64* xs, XLayout xl, u32 k0, u32 k_bstride, u32 n, u64* scratch, bool prepare, hipStream_t st,
                                 const u64* centre_mask, u32 centre_tap, bool direct_keys) {
    if (n_taps == 0 || n == 0) return hipSuccess;
    if (n_taps > 8 || n > CT_BATCH) return hipErrorInvalidValue;
    if (direct_keys) {  // no masks, no prepared copies: the keys are read where they are
        if (centre_mask) return hipErrorInvalidValue;
        for (u32 i = 0; i < n_taps; i++)
            if (masks && masks[i]) return hipErrorInvalidValue;
    } else if (!scratch || !masks) {
        return hipErrorInvalidValue;
    }
    const u32 E = c->ext_limbs(level), beta = c->live_digits(level);
    if (beta > 4) return hipErrorNotSupported;
    TapSet T;
    const u64 two_n = 2ull * c->N;
    for (u32 i = 0; i < 8; i++) {
        T.key[i] = i < n_taps ? keys[i] : nullptr;
        T.mask[i] = (i < n_taps && masks) ? masks[i] : nullptr;
        T.tap[i] = i < n_taps ? taps[i] : 0;
        u64 inv = 1;
        if (i < n_taps) {  // g^-1 mod 2N: g is odd, the group has exponent N/2
            u64 base = gs[i] % two_n;
            for (u64 ex = c->N / 2 - 1; ex; ex >>= 1) {
                if (ex & 1) inv = inv * base % two_n;
                base = base * base % two_n;
            }
        }
        T.ginv[i] = (u32)inv;
    }
    T.n_taps = n_taps;
    T.centre_mask = centre_mask;
    T.centre_tap = centre_tap;
    PtrList8 cl;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) cl.p[b] = b < n ? c0s[b] : nullptr;
    u64* mk = scratch;
    u64* mp = direct_keys ? nullptr : scratch + (size_t)n_taps * beta * 2 * E * c->N;
    const u32 nxb = (c->N + KS_THREADS - 1) / KS_THREADS;
    const u64* negp = c->d_moddown + 2 * c->k_pad + (size_t)c->k_pad * c->num_q + 2 * c->num_q;
    const u64* negp_direct = direct_keys ? negp : nullptr;
    if (prepare && !direct_keys) {
        ProfScope ps__(c, K_MASK_MUL, st, 8.0 * c->N * n_taps * (E * (4.0 * beta + 1.0) + level + 1.0), 2.0 * c->N * n_taps * E * beta);
        hipLaunchKernelGGL(mask_keys_kernel, dim3(nxb, E, n_taps + (centre_mask ? 1 : 0)), dim3(KS_THREADS), 0, st, T, mk, mp, negp, c->d_mc, c->N, level, c->num_q,
                           c->M, E, beta);
    }
    dim3 grid(nxb, E);
    // digits and c0 once per batch, per tap one masked key and the outputs
    ProfScope ps__(c, K_KEY_INNER, st, 8.0 * c->N * (E * (n * (double)beta + n_taps * (2.0 * beta + 2.0 * n)) + (n + n_taps) * (level + 1.0)),
                   2.0 * n_taps * n * c->N * E * (beta + 1.0));
#define KI_TAPS(B_)                                                                                                                  \
    do {                                                                                                                             \
        if (c->small_q)                                                                                                              \
            hipLaunchKernelGGL((key_inner_taps_kernel<B_, true>), grid, dim3(KS_THREADS), 0, st, digits, T, mk, mp, cl, xs, xl, \
                               k0, k_bstride, c->d_mc, c->log_n, level, c->num_q, E, n, c->M, negp_direct, c->d_mcf);                \
        else                                                                                                                         \
            hipLaunchKernelGGL((key_inner_taps_kernel<B_, false>), grid, dim3(KS_THREADS), 0, st, digits, T, mk, mp, cl, xs, xl, \
                               k0, k_bstride, c->d_mc, c->log_n, level, c->num_q, E, n, c->M, negp_direct, c->d_mcf);                \
    } while (0)
    if (beta == 1) KI_TAPS(1);
    else if (beta == 2) KI_TAPS(2);
    else if (beta == 3) KI_TAPS(3);
    else KI_TAPS(4);
#undef KI_TAPS
    return hipGetLastError();
}

// ---- ModDown, conversion of the P-part ----------------------------------------------------------
// v [2][E][N]: limbs level+1.. hold the P-part in coefficient form.  w [2][level+1][N] (coefficients)
// Dropped limbs: positions first..first+k-1 of v's E limbs; their moduli: `merged` ? (q_level, p_0, ...) : (p_0, ...).
// Results on limbs 0..n_out-1 (n_out = level+1, or level when merged).
__device__ __forceinline__ u32 dropped_modulus(u32 a, u32 level, u32 num_q, bool merged) {
    return merged ? (a == 0 ? level : num_q + a - 1) : num_q + a;
}

__global__ __launch_bounds__(KS_THREADS) void moddown_conv_kernel(const u64* __restrict__ v, u64* __restrict__ w,
                                                                  const u64* __restrict__ tab, const ModConst* __restrict__ mc,
                                                                  u32 N, u32 level, u32 num_q, u32 k, u32 kp, u32 E, u32 first,
                                                                  u32 n_out, bool merged, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 comp = blockIdx.z;
    u64 z[KS_MAX_DIGIT];
    u64 n_neg = 0;
#pragma unroll
    for (u32 a = 0; a < KS_MAX_DIGIT; a++)
        if (a < k) {
            const u64 pa = mc[dropped_modulus(a, level, num_q, merged)].q;
            z[a] = mul_shoup(v[((size_t)comp * E + first + a) * N + x], tab[a], tab[kp + a], pa);
            n_neg += z[a] > (pa >> 1) ? 1 : 0;
        }
    const u64* phat_q = tab + 2 * kp;  // [num_q][kp]
    const u64* negp = tab + 2 * kp + (size_t)kp * num_q + 2 * num_q;
    const u32 i0 = blockIdx.y * lpb;
    for (u32 i = i0; i < i0 + lpb && i < n_out; i++) {
        U128 acc = {0, 0};
#pragma unroll
        for (u32 a = 0; a < KS_MAX_DIGIT; a++)
            if (a < k) acc_wide(acc, z[a], phat_q[(size_t)i * kp + a]);
        acc_wide(acc, n_neg, negp[i]);
        w[((size_t)comp * n_out + i) * N + x] = barrett_reduce(acc, mc[i]);
    }
}

// KP: padded row length of the tables; KR: how many of the row's entries are real (the rest are zeros that need no arithmetic)
template <int KP, int KR = KP>
__global__ __launch_bounds__(KS_THREADS) void moddown_conv50_kernel(const u64* __restrict__ v, u64* __restrict__ w,
                                                                    const u64* __restrict__ tab, const ModConst* __restrict__ mc,
                                                                    u32 N, u32 level, u32 num_q, u32 k, u32 E, u32 first, u32 n_out,
                                                                    bool merged, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 comp = blockIdx.z;
    Split50 z[KR];
    u32 n_neg = 0;
#pragma unroll
    for (u32 a = 0; a < KR; a++) {
        z[a] = {0, 0, 0};
        if (a < k) {
            const u64 pa = mc[dropped_modulus(a, level, num_q, merged)].q;
            const u64 zv = mul_shoup(v[((size_t)comp * E + first + a) * N + x], tab[a], tab[KP + a], pa);
            n_neg += zv > (pa >> 1) ? 1 : 0;
            z[a] = split50(zv);
        }
    }
    constexpr int ROW_ALIGN = (KP & (KP - 1)) == 0 ? 8 * KP : 32;  // rows of 12 words are 32-byte aligned
    const u64* phat_q = (const u64*)__builtin_assume_aligned(tab + 2 * KP, ROW_ALIGN);  // [num_q][KP]
    const u64* negp = tab + 2 * KP + (size_t)KP * num_q + 2 * num_q;
    const u32 i0 = blockIdx.y * lpb;
    for (u32 i = i0; i < i0 + lpb && i < n_out; i++) {
        const u64* pe = (const u64*)__builtin_assume_aligned(phat_q + (size_t)i * KP, ROW_ALIGN);
        u64 cv[KP];
#pragma unroll
        for (u32 a = 0; a < KP; a++) cv[a] = pe[a];
        Acc50 acc = {0, 0, 0};
#pragma unroll
        for (u32 a = 0; a < KR; a++) acc50_mad(acc, z[a], split50(cv[a]));
        U128 s = acc50_value(acc);
        acc_wide(s, n_neg, negp[i]);
        w[((size_t)comp * n_out + i) * N + x] = barrett_reduce(s, mc[i]);
    }
}

// The same conversion in double precision (see modup_conv_f64_kernel).  phf: [num_q][KP] (constant, constant / q_i).
template <int KP, int KR = KP>
__global__ __launch_bounds__(KS_THREADS) void moddown_conv_f64_kernel(const u64* __restrict__ v, u64* __restrict__ w,
                                                                      const u64* __restrict__ tab, const TwF* __restrict__ phf,
                                                                      const ModConst* __restrict__ mc, const ModConstF* __restrict__ mcf,
                                                                      u32 N, u32 level, u32 num_q, u32 k, u32 E, u32 first, u32 n_out,
                                                                      bool merged, u32 lpb) {
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 comp = blockIdx.z;
    double z[KR];
#pragma unroll
    for (u32 a = 0; a < KR; a++) {
        z[a] = 0.0;
        if (a < k) {
            const u64 pa = mc[dropped_modulus(a, level, num_q, merged)].q;
            const u64 zv = mul_shoup(v[((size_t)comp * E + first + a) * N + x], tab[a], tab[KP + a], pa);
            z[a] = zv > (pa >> 1) ? -f64m_from_u64(pa - zv) : f64m_from_u64(zv);
        }
    }
    const u32 i0 = blockIdx.y * lpb;
    for (u32 i = i0; i < i0 + lpb && i < n_out; i++) {
        const TwF* pe = phf + (size_t)i * KP;
        const double q = mcf[i].q, qinv = mcf[i].qinv;
        w[((size_t)comp * n_out + i) * N + x] = f64m_canonical(f64m_dot<KR>(z, pe, q, qinv), q);
    }
}

hipError_t launch_moddown_conv(const ckks_ctx* c, u32 level, bool merged, const u64* v, u64* w, u32 batch, hipStream_t st) {
    const u32 n_out = merged ? level : level + 1, k = merged ? c->num_p + 1 : c->num_p, kp = merged ? c->k2_pad : c->k_pad;
    const u32 first = merged ? level : level + 1, E = c->ext_limbs(level);
    const u64* tab = merged ? c->moddown_rs_table(level) : c->d_moddown;
    const u32 x_wgs = (c->N + KS_THREADS - 1) / KS_THREADS;
    const u32 lpb = x_wgs * batch >= 2048 ? 12 : 6;  // as in launch_modup_conv
    dim3 grid(x_wgs, (n_out + lpb - 1) / lpb, batch);
    ProfScope ps__(c, K_MODDOWN_CONV, st, 8.0 * batch * c->N * (k + n_out), 1.0 * batch * c->N * k * (n_out + 1.0));
    if (c->ntt_f64 && c->d_moddown_f) {
        const TwF* pf = merged ? c->moddown_rs_table_f(level) : c->d_moddown_f;
#define MD_F64(KP_, KR_) hipLaunchKernelGGL((moddown_conv_f64_kernel<KP_, KR_>), grid, dim3(KS_THREADS), 0, st, v, w, tab, pf, c->d_mc, c->d_mcf, c->N, level, c->num_q, k, E, first, n_out, merged, lpb)
        if (kp == 4) MD_F64(4, 4);
        else if (kp == 8) MD_F64(8, 8);
        else if (kp == 12 && k == 9) MD_F64(12, 9);
        else if (kp == 12) MD_F64(12, 12);
        else MD_F64(16, 16);
#undef MD_F64
        return hipGetLastError();
    }
    if (c->small_q) {
        if (kp == 4)
            hipLaunchKernelGGL(moddown_conv50_kernel<4>, grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, E, first, n_out, merged, lpb);
        else if (kp == 8)
            hipLaunchKernelGGL(moddown_conv50_kernel<8>, grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, E, first, n_out, merged, lpb);
        else if (kp == 12 && k == 9)
            hipLaunchKernelGGL((moddown_conv50_kernel<12, 9>), grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, E, first, n_out, merged, lpb);
        else if (kp == 12)
            hipLaunchKernelGGL(moddown_conv50_kernel<12>, grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, E, first, n_out, merged, lpb);
        else
            hipLaunchKernelGGL(moddown_conv50_kernel<16>, grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, E, first, n_out, merged, lpb);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(moddown_conv_kernel, grid, dim3(KS_THREADS), 0, st, v, w, tab, c->d_mc, c->N, level, c->num_q, k, kp, E, first, n_out, merged, lpb);
    return hipGetLastError();
}

// ---- ModDown, last step, for a batch of key switches -------------------------------------------
// out_r[comp][i] = ((v_r[comp][i] - w_r[comp][i]) * P^-1 + addend) * mask, r < n (grid.z = 2n).
// add0 / add1: optional polynomials [level+1][N] added to component 0 / 1; when g != 1 the addend is
// read through the sigma_g gather (Rot: c0' = sigma_g(c0) + u0).  mask: optional plaintext
// [level+1][N] multiplied into both components (the tap's validity mask of the convolution).
__global__ __launch_bounds__(KS_THREADS) void moddown_final_kernel(const u64* __restrict__ v, const u64* __restrict__ w,
                                                                   FinalBatch B, const u64* __restrict__ tab,
                                                                   const ModConst* __restrict__ mc, u32 log_n, u32 n_out,
                                                                   u32 num_q, u32 kp, u32 E) {
    const u32 N = 1u << log_n;
    const u32 x = blockIdx.x * KS_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, b = blockIdx.z, comp = b & 1;
    const FinalItem it = B.it[b >> 1];
    const ModConst m = mc[i];
    const u64* pinv = tab + 2 * kp + (size_t)kp * num_q;
    u64 d = sub_mod(v[((size_t)b * E + i) * N + x], w[((size_t)b * n_out + i) * N + x], m.q);
    u64 r = mul_shoup(d, pinv[i], pinv[num_q + i], m.q);
    const u64* add = comp == 0 ? it.add0 : it.add1;
    if (add) {
        const u32 xs = it.g == 1 ? x : galois_gather_index(x, it.g, log_n);
        r = add_mod(r, add[(size_t)i * N + xs], m.q);
    }
    if (it.mask) r = mulmod_barrett(r, it.mask[(size_t)i * N + x], m);
    if (it.acc) r = add_mod(r, it.acc[((size_t)comp * n_out + i) * N + x], m.q);
    it.out[((size_t)comp * n_out + i) * N + x] = r;
}

// merged: division by P*q_level (results on limbs 0..level-1; addends and masks, if any, are [level][N])
hipError_t launch_moddown_final(const ckks_ctx* c, u32 level, bool merged, const u64* v, const u64* w, const FinalItem* items, u32 n,
                                hipStream_t st) {
    FinalBatch B;
    double extra = 0.0;
    for (u32 r = 0; r < KS_MAX_BATCH; r++) {
        if (r < n) {
            B.it[r] = items[r];
            extra += (items[r].add0 ? 1.0 : 0.0) + (items[r].add1 ? 1.0 : 0.0) + (items[r].mask ? 1.0 : 0.0) + (items[r].acc ? 2.0 : 0.0);
        } else {
            B.it[r] = FinalItem{nullptr, nullptr, nullptr, nullptr, 1, 0, nullptr};
        }
    }
    const u32 n_out = merged ? level : level + 1;
    dim3 grid((c->N + KS_THREADS - 1) / KS_THREADS, n_out, 2 * n);
    ProfScope ps__(c, K_MODDOWN_FINAL, st, 8.0 * c->N * n_out * (6.0 * n + extra), 2.0 * c->N * n_out * n);
    hipLaunchKernelGGL(moddown_final_kernel, grid, dim3(KS_THREADS), 0, st, v, w, B, merged ? c->moddown_rs_table(level) : c->d_moddown,
                       c->d_mc, c->log_n, n_out, c->num_q, merged ? c->k2_pad : c->k_pad, c->ext_limbs(level));
    return hipGetLastError();
}
