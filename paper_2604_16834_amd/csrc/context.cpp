// Context creation: validates the parameter set and builds every table the kernels read
// (twiddles with Shoup companions, Barrett constants, basis-conversion constants for ModUp at every
// level, ModDown and rescale constants).  Host-side integer arithmetic with 128-bit products.
#include <cstring>
#include <new>

#include "ctx.h"

typedef unsigned __int128 u128;

static u64 h_mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }
static u64 h_powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = h_mulmod(r, a, q);
        a = h_mulmod(a, a, q);
    }
    return r;
}
static u64 h_invmod(u64 a, u64 q) { return h_powmod(a, q - 2, q); }
static u64 h_shoup(u64 w, u64 q) { return (u64)(((u128)w << 64) / q); }
static u32 h_bits(u64 v) { u32 b = 0; while (v) { b++; v >>= 1; } return b; }
static u32 h_bitrev(u32 x, u32 bits) {
    u32 r = 0;
    for (u32 i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}
static bool h_is_prime(u64 n) {
    if (n < 2) return false;
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 p : bases) { if (n % p == 0) return n == p; }
    u64 d = n - 1; u32 s = 0;
    while (!(d & 1)) { d >>= 1; s++; }
    for (u64 a : bases) {
        u64 x = h_powmod(a, d, n);
        if (x == 1 || x == n - 1) continue;
        bool comp = true;
        for (u32 r = 1; r < s; r++) { x = h_mulmod(x, x, n); if (x == n - 1) { comp = false; break; } }
        if (comp) return false;
    }
    return true;
}

template <class T>
static hipError_t upload(const std::vector<T>& h, T** d) {
    *d = nullptr;
    if (h.empty()) return hipSuccess;
    hipError_t e = hipMalloc((void**)d, h.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
}

static thread_local std::string g_create_error;

extern "C" const char* ckks_last_error_string(const ckks_ctx* ctx) {
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

extern "C" void ckks_ctx_destroy(ckks_ctx* c) {
    if (!c) return;
    (void)hipFree(c->d_mc);
    (void)hipFree(c->d_tw);
    (void)hipFree(c->d_itw);
    (void)hipFree(c->d_twf);
    (void)hipFree(c->d_twf_val);
    (void)hipFree(c->d_itwf_val);
    (void)hipFree(c->d_itwf);
    (void)hipFree(c->d_mcf);
    (void)hipFree(c->d_pow256);
    (void)hipFree(c->d_modup);
    (void)hipFree(c->d_moddown);
    (void)hipFree(c->d_moddown_rs);
    (void)hipFree(c->d_modup_f);
    (void)hipFree(c->d_modup_prep_f);
    (void)hipFree(c->d_moddown_f);
    (void)hipFree(c->d_moddown_rs_f);
    (void)hipFree(c->d_moddown_prep_f);
    (void)hipFree(c->d_rescale_prep_f);
    (void)hipFree(c->d_rescale_conv_f);
    (void)hipFree(c->d_rescale_ep);
    (void)hipFree(c->d_moddown_rs_prep_f);
    (void)hipFree(c->d_rescale);
    (void)hipFree(c->d_check);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->side) (void)hipStreamDestroy(c->side);
    delete c;
}

extern "C" int ckks_ctx_create(const ckks_params* p, ckks_ctx** out) {
    auto fail = [&](int code, const char* msg) { g_create_error = msg; return code; };
    if (!p || !out || !p->moduli || !p->psi) return fail(CKKS_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    if (p->log_n < 4 || p->log_n > 17) return fail(CKKS_ERR_UNSUPPORTED_PARAMS, "log_n must be in [4, 17]");
    const u32 M = p->num_q + p->num_p;
    if (p->num_q < 1 || M > CKKS_MAX_MODULI) return fail(CKKS_ERR_UNSUPPORTED_PARAMS, "need 1 <= num_q and num_q + num_p <= 64");
    if (p->dnum == 0 && p->num_p != 0) return fail(CKKS_ERR_INVALID_ARG, "special primes given but dnum = 0");
    if (p->dnum != 0 && (p->dnum > p->num_q || p->num_p < 1)) return fail(CKKS_ERR_INVALID_ARG, "need 1 <= dnum <= num_q and num_p >= 1");
    const u32 N = 1u << p->log_n;
    const u32 alpha = p->dnum ? (p->num_q + p->dnum - 1) / p->dnum : 0;
    if (alpha > 16 || p->num_p > 15) return fail(CKKS_ERR_UNSUPPORTED_PARAMS, "at most 16 limbs per digit and 15 special primes");
    u32 bmin = 64, bmax = 0;
    for (u32 t = 0; t < M; t++) {
        const u64 q = p->moduli[t];
        if (q >= (1ull << 58) || q < 1024) return fail(CKKS_ERR_UNSUPPORTED_PARAMS, "moduli must lie in [2^10, 2^58)");
        if ((q - 1) % (2ull * N) != 0) return fail(CKKS_ERR_INVALID_ARG, "modulus is not 1 mod 2N");
        if (!h_is_prime(q)) return fail(CKKS_ERR_INVALID_ARG, "modulus is not prime");
        for (u32 u = 0; u < t; u++)
            if (p->moduli[u] == q) return fail(CKKS_ERR_INVALID_ARG, "moduli must be distinct");
        if (p->psi[t] >= q || h_powmod(p->psi[t], N, q) != q - 1) return fail(CKKS_ERR_INVALID_ARG, "psi is not a primitive 2N-th root of unity");
        const u32 b = h_bits(q);
        bmin = b < bmin ? b : bmin;
        bmax = b > bmax ? b : bmax;
    }
    // products of two residues are below 2^(2*bmax); a Barrett input must stay below 2^(62+bmin)
    const int lazy_log = 62 + (int)bmin - 2 * (int)bmax;
    if (lazy_log < 5) return fail(CKKS_ERR_UNSUPPORTED_PARAMS, "moduli sizes too uneven for 128-bit lazy accumulation");

    ckks_ctx* c = new (std::nothrow) ckks_ctx;
    if (!c) return fail(CKKS_ERR_INVALID_ARG, "out of host memory");
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return fail(CKKS_ERR_HIP, "no current HIP device"); }
    c->log_n = p->log_n; c->N = N; c->num_q = p->num_q; c->num_p = p->num_p; c->dnum = p->dnum; c->alpha = alpha; c->M = M;
    c->log_lo = p->log_n < CKKS_TILE_LOG ? p->log_n : CKKS_TILE_LOG;
    c->log_hi = p->log_n - c->log_lo;
    c->lazy_terms = 1u << (lazy_log > 12 ? 12 : lazy_log);
    c->small_q = bmax <= 50;
    c->ntt_f64 = c->small_q && p->log_n >= CKKS_TILE_LOG;
    auto pad = [](u32 v) { return v <= 4 ? 4u : (v <= 8 ? 8u : 16u); };
    c->alpha_pad = pad(alpha);
    c->k_pad = pad(p->num_p);
    c->k2_pad = p->num_p + 1 > 8 && p->num_p + 1 <= 12 ? 12u : pad(p->num_p + 1);  // 9..12 dropped limbs: rows of 12
    c->mod.assign(p->moduli, p->moduli + M);
    c->psi.assign(p->psi, p->psi + M);

    c->mc.resize(M);
    // one pair of twiddle tables: integers with Shoup companions, or doubles with twiddle / q
    std::vector<TwPair> tw, itw;
    std::vector<TwF> twf, itwf;
    std::vector<ModConstF> mcf;
    if (c->ntt_f64) { twf.resize((size_t)M * N); itwf.resize((size_t)M * N); }
    else { tw.resize((size_t)M * N); itw.resize((size_t)M * N); }
    if (c->small_q) mcf.resize(M);  // also read by the kernels that are double-precision at any ring size (inner products, matrix-core sum)
    for (u32 t = 0; t < M; t++) {
        const u64 q = c->mod[t];
        ModConst& m = c->mc[t];
        m.q = q;
        m.sh = h_bits(q) - 2;
        m.mu = (u64)((((u128)1) << (64 + m.sh)) / q);
        m.pad = 0;
        m.n_inv = h_invmod(N % q, q);
        m.n_inv_sh = h_shoup(m.n_inv, q);
        if (c->small_q) {  // every value below is an integer below 2^50: exact as a double; the quotients are correctly rounded
            mcf[t].q = (double)q;
            mcf[t].qinv = 1.0 / (double)q;
            mcf[t].ninv = (double)m.n_inv;
            mcf[t].ninv_q = (double)m.n_inv / (double)q;
        }
        std::vector<u64> pw(N);
        pw[0] = 1;
        for (u32 i = 1; i < N; i++) pw[i] = h_mulmod(pw[i - 1], c->psi[t], q);
        const u64 psi_inv = h_invmod(c->psi[t], q);
        std::vector<u64> ipw(N);
        ipw[0] = 1;
        for (u32 i = 1; i < N; i++) ipw[i] = h_mulmod(ipw[i - 1], psi_inv, q);
        for (u32 i = 0; i < N; i++) {
            const u32 r = h_bitrev(i, p->log_n);
            const size_t o = (size_t)t * N + i;
            if (c->ntt_f64) {
                twf[o].w = (double)pw[r]; twf[o].wq = (double)pw[r] / (double)q;
                itwf[o].w = (double)ipw[r]; itwf[o].wq = (double)ipw[r] / (double)q;
            } else {
                tw[o].w = pw[r]; tw[o].s = h_shoup(pw[r], q);
                itw[o].w = ipw[r]; itw[o].s = h_shoup(ipw[r], q);
            }
        }
    }

    // powers of 256 modulo every modulus, in parts of 17, 17 and 16 bits: the matrix-core multiply-accumulate folds its 13
    // digit diagonals with them in exact double-precision sums (f64m_fold_diagonals)
    std::vector<double> pow256;
    if (c->small_q) {
        pow256.assign((size_t)M * POW256_ROW, 0.0);
        for (u32 t = 0; t < M; t++) {
            double* row = &pow256[(size_t)t * POW256_ROW];
            u64 v = 1 % c->mod[t];
            for (u32 s = 0; s < 13; s++) {
                row[3 * s] = (double)(v & 0x1ffffu);
                row[3 * s + 1] = (double)((v >> 17) & 0x1ffffu);
                row[3 * s + 2] = (double)(v >> 34);
                v = h_mulmod(v, 256, c->mod[t]);
            }
            const u64 w17 = 131072 % c->mod[t];
            row[39] = (double)w17;
            row[40] = (double)w17 / (double)c->mod[t];
        }
    }
    // ModUp tables, one per (level, digit): the digit modulus is the product of the digit's LIVE limbs
    std::vector<u64> modup;
    if (c->dnum) {
        modup.assign((size_t)c->num_q * c->modup_level_stride(), 0);
        for (u32 level = 0; level < c->num_q; level++)
            for (u32 j = 0; j < c->live_digits(level); j++) {
                u64* tab = modup.data() + level * c->modup_level_stride() + j * c->modup_digit_stride();
                const u32 lo = c->digit_lo(j), hi = c->digit_hi(j, level), E = c->ext_limbs(level);
                for (u32 a = 0; a < hi - lo; a++) {
                    const u64 qa = c->mod[lo + a];
                    u64 qhat = 1;
                    for (u32 b = lo; b < hi; b++) if (b != lo + a) qhat = h_mulmod(qhat, c->mod[b] % qa, qa);
                    const u64 inv = h_invmod(qhat, qa);
                    tab[a] = inv;
                    tab[c->alpha_pad + a] = h_shoup(inv, qa);
                    for (u32 e = 0; e < E; e++) {
                        const u64 qt = c->mod[c->ext_modulus(level, e)];
                        u64 v = 1;
                        for (u32 b = lo; b < hi; b++) if (b != lo + a) v = h_mulmod(v, c->mod[b] % qt, qt);
                        tab[2 * c->alpha_pad + (size_t)e * c->alpha_pad + a] = v;
                    }
                }
                for (u32 e = 0; e < E; e++) {  // -Q_j mod t: one per centred digit limb that is negative
                    const u64 qt = c->mod[c->ext_modulus(level, e)];
                    u64 Q = 1;
                    for (u32 b = lo; b < hi; b++) Q = h_mulmod(Q, c->mod[b] % qt, qt);
                    tab[c->modup_negq_off() + e] = (qt - Q) % qt;
                }
            }
    }
    // ModDown table
    std::vector<u64> moddown;
    if (c->dnum) {
        const u32 k = c->num_p, nq = c->num_q, kp = c->k_pad;
        moddown.assign(2 * kp + (size_t)kp * nq + 3 * nq, 0);
        for (u32 a = 0; a < k; a++) {
            const u64 pa = c->mod[nq + a];
            u64 phat = 1;
            for (u32 b = 0; b < k; b++) if (b != a) phat = h_mulmod(phat, c->mod[nq + b] % pa, pa);
            const u64 inv = h_invmod(phat, pa);
            moddown[a] = inv;
            moddown[kp + a] = h_shoup(inv, pa);
            for (u32 i = 0; i < nq; i++) {
                const u64 qi = c->mod[i];
                u64 v = 1;
                for (u32 b = 0; b < k; b++) if (b != a) v = h_mulmod(v, c->mod[nq + b] % qi, qi);
                moddown[2 * kp + (size_t)i * kp + a] = v;
            }
        }
        for (u32 i = 0; i < nq; i++) {
            const u64 qi = c->mod[i];
            u64 P = 1;
            for (u32 b = 0; b < k; b++) P = h_mulmod(P, c->mod[nq + b] % qi, qi);
            const u64 pinv = h_invmod(P, qi);
            moddown[2 * kp + (size_t)kp * nq + i] = pinv;
            moddown[2 * kp + (size_t)kp * nq + nq + i] = h_shoup(pinv, qi);
            moddown[2 * kp + (size_t)kp * nq + 2 * nq + i] = (qi - P) % qi;  // -P mod q_i
        }
    }
    // the same constants for the dropped set D(l) = {q_l, p_0..p_{k-1}} of every level l >= 1
    std::vector<u64> moddown_rs;
    if (c->dnum) {
        const u32 k = c->num_p, nq = c->num_q, kp = c->k2_pad;
        moddown_rs.assign((size_t)nq * c->moddown_rs_stride(), 0);
        for (u32 l = 1; l < nq; l++) {
            u64* tab = moddown_rs.data() + l * c->moddown_rs_stride();
            std::vector<u64> drop(1, c->mod[l]);
            for (u32 b = 0; b < k; b++) drop.push_back(c->mod[nq + b]);
            for (u32 a = 0; a <= k; a++) {
                const u64 da = drop[a];
                u64 dhat = 1;
                for (u32 b = 0; b <= k; b++) if (b != a) dhat = h_mulmod(dhat, drop[b] % da, da);
                const u64 inv = h_invmod(dhat, da);
                tab[a] = inv;
                tab[kp + a] = h_shoup(inv, da);
                for (u32 i = 0; i < l; i++) {
                    const u64 qi = c->mod[i];
                    u64 v = 1;
                    for (u32 b = 0; b <= k; b++) if (b != a) v = h_mulmod(v, drop[b] % qi, qi);
                    tab[2 * kp + (size_t)i * kp + a] = v;
                }
            }
            for (u32 i = 0; i < l; i++) {
                const u64 qi = c->mod[i];
                u64 D = 1;
                for (u32 b = 0; b <= k; b++) D = h_mulmod(D, drop[b] % qi, qi);
                const u64 dinv = h_invmod(D, qi);
                tab[2 * kp + (size_t)kp * nq + i] = dinv;
                tab[2 * kp + (size_t)kp * nq + nq + i] = h_shoup(dinv, qi);
                tab[2 * kp + (size_t)kp * nq + 2 * nq + i] = (qi - D) % qi;
            }
        }
    }
    // the conversion constants as doubles for the double-precision conversions: the centred representative (f64m_dot takes
    // centred operands) and its quotient by the target modulus
    auto centred = [](u64 w, u64 q) {
        const double v = w > (q >> 1) ? -(double)(q - w) : (double)w;
        return TwF{v, v / (double)q};
    };
    std::vector<TwF> modup_f, modup_prep_f, moddown_f, moddown_rs_f, moddown_prep_f, moddown_rs_prep_f, rescale_prep_f, rescale_conv_f;
    if (c->dnum && c->ntt_f64) {
        const u32 nq = c->num_q;
        modup_f.assign((size_t)nq * c->dnum * M * c->alpha_pad, TwF{0.0, 0.0});
        for (u32 level = 0; level < nq; level++)
            for (u32 j = 0; j < c->live_digits(level); j++) {
                const u64* tab = modup.data() + level * c->modup_level_stride() + j * c->modup_digit_stride();
                TwF* tf = modup_f.data() + ((size_t)level * c->dnum + j) * M * c->alpha_pad;
                for (u32 e = 0; e < c->ext_limbs(level); e++) {
                    const u64 qt = c->mod[c->ext_modulus(level, e)];
                    for (u32 a = 0; a < c->alpha_pad; a++)
                        tf[(size_t)e * c->alpha_pad + a] = centred(tab[2 * c->alpha_pad + (size_t)e * c->alpha_pad + a], qt);
                }
            }
        modup_prep_f.assign((size_t)nq * nq, TwF{0.0, 0.0});
        for (u32 level = 0; level < nq; level++)
            for (u32 j = 0; j < c->live_digits(level); j++) {
                const u64* tab = modup.data() + level * c->modup_level_stride() + j * c->modup_digit_stride();
                for (u32 i = c->digit_lo(j); i < c->digit_hi(j, level); i++) {
                    const u64 qi = c->mod[i];
                    const double w = (double)h_mulmod(tab[i - c->digit_lo(j)], c->mc[i].n_inv, qi);
                    modup_prep_f[(size_t)level * nq + i] = TwF{w, w / (double)qi};
                }
            }
        moddown_f.assign((size_t)nq * c->k_pad, TwF{0.0, 0.0});
        for (u32 i = 0; i < nq; i++)
            for (u32 a = 0; a < c->k_pad; a++) moddown_f[(size_t)i * c->k_pad + a] = centred(moddown[2 * c->k_pad + (size_t)i * c->k_pad + a], c->mod[i]);
        // what the inverse transform in front of ModDown scales a dropped limb by: 1/N times the limb's conversion constant
        auto prep = [&](u64 inv, u32 m) {
            const u64 q = c->mod[m];
            const double w = (double)h_mulmod(inv, c->mc[m].n_inv, q);
            return TwF{w, w / (double)q};
        };
        // the rescale as a one-limb conversion: the inverse transform scales by 1/N only, the conversion constant is 1
        rescale_prep_f.assign(M, TwF{0.0, 0.0});
        for (u32 m = 0; m < M; m++) rescale_prep_f[m] = TwF{(double)c->mc[m].n_inv, (double)c->mc[m].n_inv / (double)c->mod[m]};
        rescale_conv_f.assign((size_t)nq * 4, TwF{0.0, 0.0});
        for (u32 i = 0; i < nq; i++) rescale_conv_f[(size_t)i * 4] = TwF{1.0, 1.0 / (double)c->mod[i]};
        moddown_prep_f.assign(M, TwF{0.0, 0.0});
        for (u32 a = 0; a < c->num_p; a++) moddown_prep_f[nq + a] = prep(moddown[a], nq + a);
        moddown_rs_prep_f.assign((size_t)nq * M, TwF{0.0, 0.0});
        for (u32 l = 1; l < nq; l++) {
            const u64* tab = moddown_rs.data() + l * c->moddown_rs_stride();
            moddown_rs_prep_f[(size_t)l * M + l] = prep(tab[0], l);
            for (u32 a = 0; a < c->num_p; a++) moddown_rs_prep_f[(size_t)l * M + nq + a] = prep(tab[1 + a], nq + a);
        }
        moddown_rs_f.assign((size_t)nq * nq * c->k2_pad, TwF{0.0, 0.0});
        for (u32 l = 1; l < nq; l++) {
            const u64* tab = moddown_rs.data() + l * c->moddown_rs_stride();
            for (u32 i = 0; i < l; i++)
                for (u32 a = 0; a < c->k2_pad; a++)
                    moddown_rs_f[((size_t)l * nq + i) * c->k2_pad + a] = centred(tab[2 * c->k2_pad + (size_t)i * c->k2_pad + a], c->mod[i]);
        }
    }
    // rescale table [l][i] = (q_l^-1 mod q_i, Shoup companion, q_l mod q_i)
    std::vector<u64> resc((size_t)c->num_q * c->num_q * 3, 0);
    for (u32 l = 0; l < c->num_q; l++)
        for (u32 i = 0; i < l; i++) {
            const u64 qi = c->mod[i], ql = c->mod[l] % qi;
            const u64 inv = h_invmod(ql, qi);
            u64* t = resc.data() + ((size_t)l * c->num_q + i) * 3;
            t[0] = inv; t[1] = h_shoup(inv, qi); t[2] = ql;
        }

    // the rescale constants once more, in the layout the transforms' division epilogue reads
    std::vector<u64> resc_ep((size_t)c->num_q * 2 * c->num_q, 0);
    for (u32 l = 0; l < c->num_q; l++)
        for (u32 i = 0; i < l; i++) {
            resc_ep[((size_t)l * 2 + 0) * c->num_q + i] = resc[((size_t)l * c->num_q + i) * 3 + 0];
            resc_ep[((size_t)l * 2 + 1) * c->num_q + i] = resc[((size_t)l * c->num_q + i) * 3 + 1];
        }

    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = upload(c->mc, &c->d_mc);
    if (e == hipSuccess) e = upload(resc_ep, &c->d_rescale_ep);
    if (e == hipSuccess) e = upload(rescale_prep_f, &c->d_rescale_prep_f);
    if (e == hipSuccess) e = upload(rescale_conv_f, &c->d_rescale_conv_f);
    if (e == hipSuccess) e = upload(tw, &c->d_tw);
    if (e == hipSuccess) e = upload(itw, &c->d_itw);
    if (e == hipSuccess) e = upload(twf, &c->d_twf);
    {
        std::vector<double> twf_val(twf.size());
        for (size_t i = 0; i < twf.size(); i++) twf_val[i] = twf[i].w;
        if (e == hipSuccess) e = upload(twf_val, &c->d_twf_val);
        for (size_t i = 0; i < itwf.size(); i++) twf_val[i] = itwf[i].w;
        if (e == hipSuccess) e = upload(twf_val, &c->d_itwf_val);
    }
    if (e == hipSuccess) e = upload(itwf, &c->d_itwf);
    if (e == hipSuccess) e = upload(mcf, &c->d_mcf);
    if (e == hipSuccess) e = upload(pow256, &c->d_pow256);
    if (e == hipSuccess) e = upload(modup, &c->d_modup);
    if (e == hipSuccess) e = upload(moddown, &c->d_moddown);
    if (e == hipSuccess) e = upload(moddown_rs, &c->d_moddown_rs);
    if (e == hipSuccess) e = upload(modup_f, &c->d_modup_f);
    if (e == hipSuccess) e = upload(modup_prep_f, &c->d_modup_prep_f);
    if (e == hipSuccess) e = upload(moddown_f, &c->d_moddown_f);
    if (e == hipSuccess) e = upload(moddown_rs_f, &c->d_moddown_rs_f);
    if (e == hipSuccess) e = upload(moddown_prep_f, &c->d_moddown_prep_f);
    if (e == hipSuccess) e = upload(moddown_rs_prep_f, &c->d_moddown_rs_prep_f);
    if (e == hipSuccess) e = upload(resc, &c->d_rescale);
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_check, 256);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        g_create_error = std::string("HIP error while building tables: ") + hipGetErrorString(e);
        ckks_ctx_destroy(c);
        return CKKS_ERR_HIP;
    }
    // the built-in scratch of the call that takes no workspace: its address on this device, looked up once, here
    if ((e = noalloc_scratch_current_device(nullptr, nullptr)) != hipSuccess) {
        g_create_error = std::string("HIP error while looking up the built-in scratch buffer: ") + hipGetErrorString(e);
        ckks_ctx_destroy(c);
        return CKKS_ERR_HIP;
    }
    // the side stream is an optimisation: without it everything runs on the caller's stream
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) c->side = nullptr;
    if (c->side && (hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
                    hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess)) {
        if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
        (void)hipStreamDestroy(c->side);
        c->side = nullptr;
        c->ev_fork = c->ev_join = nullptr;
    }
    *out = c;
    return CKKS_OK;
}
