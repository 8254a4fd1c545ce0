// CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
//
// A plain, slow RNS-CKKS written step by step so that it can be checked by eye.  Only tests, the
// smoke check and the benchmark's cpu_baseline leg may call into this file; the HIP library shares
// no code, table or constant with it.
//
// What it implements is the substrate the paper uses as a black box (Background: "The CKKS
// Scheme", "Rotations and Key Switching", "RNS Decomposition and NTT Optimization"; Experiments,
// "HE Security Parameters": word-size RNS limbs, digit-decomposed key switching, rescaling) and the
// integer side of the batched convolution (Methodology, "Convolution Layer": Eq. 11, the sum over
// aligned ciphertexts times encoded weights; channel accumulation by plain additions).
//
// The paper is silent below the level of Rot / (.) / +, so the following readings are fixed here
// (the HIP side has to produce the same integers):
//   * every residue is the canonical representative in [0, q);
//   * forward NTT: natural-order coefficients in, bit-reversed evaluation order out, i.e.
//     out[k] = a(psi^(2*brv(k)+1)); the inverse is its exact inverse including 1/N;
//   * digit j of a hybrid key switch covers limbs [j*alpha, (j+1)*alpha) intersected with the live
//     limbs, alpha = ceil(num_q / dnum);
//   * the scaled residue y_i = [c_i * (Q_j/q_i)^-1] mod q_i is taken as the CENTRED representative
//     in [-(q_i-1)/2, (q_i-1)/2] and the basis extension is the plain sum
//     sum_i y_i * [Q_j/q_i]_t  mod t  (no floating-point correction), so the extended digit equals
//     c + u*Q_j with a small integer |u| <= |digit|/2 of mean zero;
//   * ModDown extends the P-part the same way (centred, uncorrected), which makes the division by
//     P a rounding to nearest with an extra error below k/2 of mean zero.  (Unsigned
//     representatives would bias every coefficient by about -k/2; times the secret that is a
//     low-frequency error of ~1e-4 in the slots at N = 2^16 and scale 2^40.)
//   * rescale takes the centred remainder of the dropped limb (round to nearest);
//   * a rotation can be computed in two orders: "unhoisted" applies the automorphism to the
//     ciphertext first and key-switches the permuted c1; "hoisted" extends c1 once and permutes the
//     extended digits.  Both are here.  Because the automorphism only permutes and negates
//     coefficients and centring commutes with negation, the two orders give the same residues
//     (with unsigned representatives they would differ by multiples of Q_j).
//   * sampling (oracle only): SplitMix64-seeded xoshiro256**, ternary secret uniform on {-1,0,1},
//     error = round(3.2 * Box-Muller normal) truncated to |e| <= 19, uniform residues by rejection.
//
// mulmod is (unsigned __int128) a * b % q everywhere: no Montgomery, no Barrett, no Shoup, no lazy
// reduction, no blocking beyond what the definitions state.  OpenMP only distributes independent
// limbs over threads.
//
// Parity unpinned: the concrete primes, roots of unity and sampler streams are conventions; they
// reach both sides as explicit inputs.

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;
typedef __int128 i128;

static inline u64 addmod(u64 a, u64 b, u64 q) { u64 s = a + b; return s >= q ? s - q : s; }
static inline u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }
static inline u64 mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }
static u64 powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    while (e) { if (e & 1) r = mulmod(r, a, q); a = mulmod(a, a, q); e >>= 1; }
    return r;
}
static inline u64 invmod(u64 a, u64 q) { return powmod(a, q - 2, q); }  // q prime

static inline uint32_t bitrev(uint32_t x, int bits) {
    uint32_t r = 0;
    for (int i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}

struct Ctx {
    int logN, N, num_q, num_p, dnum, alpha;
    std::vector<u64> mod;                  // q_0..q_L, p_0..p_{k-1}
    std::vector<u64> psi;                  // primitive 2N-th root of unity per modulus
    std::vector<std::vector<u64>> psi_brv;     // psi_brv[t][i] = psi_t ^ brv(i)
    std::vector<std::vector<u64>> psi_brv_inv; // modular inverses of the above
};

static inline int ext_modulus(const Ctx* c, int level, int e) {
    // e-th limb of the extended basis at `level`: q_0..q_level then p_0..p_{k-1}
    return e <= level ? e : c->num_q + (e - level - 1);
}
static inline int digit_lo(const Ctx* c, int j) { return j * c->alpha; }
static inline int digit_hi(const Ctx* c, int j, int level) {
    int hi = (j + 1) * c->alpha;  // exclusive
    return hi < level + 1 ? hi : level + 1;
}
static inline int live_digits(const Ctx* c, int level) { return (level + c->alpha) / c->alpha; }

extern "C" {

void* orc_create(int logN, int num_q, int num_p, int dnum, const u64* moduli, const u64* psi) {
    Ctx* c = new Ctx;
    c->logN = logN; c->N = 1 << logN; c->num_q = num_q; c->num_p = num_p; c->dnum = dnum;
    c->alpha = dnum ? (num_q + dnum - 1) / dnum : 0;
    int M = num_q + num_p;
    c->mod.assign(moduli, moduli + M);
    c->psi.assign(psi, psi + M);
    c->psi_brv.resize(M);
    c->psi_brv_inv.resize(M);
    for (int t = 0; t < M; t++) {
        u64 q = c->mod[t];
        if (powmod(psi[t], c->N, q) != q - 1) { delete c; return nullptr; }
        std::vector<u64> pw(c->N);
        pw[0] = 1;
        for (int i = 1; i < c->N; i++) pw[i] = mulmod(pw[i - 1], psi[t], q);
        c->psi_brv[t].resize(c->N);
        c->psi_brv_inv[t].resize(c->N);
        for (int i = 0; i < c->N; i++) {
            c->psi_brv[t][i] = pw[bitrev(i, logN)];
            c->psi_brv_inv[t][i] = invmod(c->psi_brv[t][i], q);
        }
    }
    return c;
}
void orc_destroy(void* h) { delete (Ctx*)h; }

// ---------------------------------------------------------------------------------------------
// Negacyclic NTT (Background, "RNS Decomposition and NTT Optimization").
// ---------------------------------------------------------------------------------------------

// The definition itself, O(N^2): out[k] = sum_i a_i * psi^((2*brv(k)+1)*i) mod q.
void orc_ntt_definition(void* h, int mod_idx, const u64* a, u64* out) {
    Ctx* c = (Ctx*)h;
    u64 q = c->mod[mod_idx];
    for (int k = 0; k < c->N; k++) {
        u64 x = powmod(c->psi[mod_idx], 2 * (u64)bitrev(k, c->logN) + 1, q);
        u64 acc = 0, xp = 1;
        for (int i = 0; i < c->N; i++) { acc = addmod(acc, mulmod(a[i], xp, q), q); xp = mulmod(xp, x, q); }
        out[k] = acc;
    }
}

// Textbook in-place radix-2 transform: stage with m groups pairs j and j+t, t = N/(2m), and
// multiplies the upper element by psi^brv(m+i) for group i.
void orc_ntt_fwd(void* h, int mod_idx, u64* a) {
    Ctx* c = (Ctx*)h;
    u64 q = c->mod[mod_idx];
    const u64* w = c->psi_brv[mod_idx].data();
    for (int m = 1, t = c->N / 2; m < c->N; m *= 2, t /= 2)
        for (int i = 0; i < m; i++)
            for (int j = 2 * i * t; j < 2 * i * t + t; j++) {
                u64 u = a[j], v = mulmod(a[j + t], w[m + i], q);
                a[j] = addmod(u, v, q);
                a[j + t] = submod(u, v, q);
            }
}

// Exact inverse: undo the stages in reverse order (u = (x+y)/2, v = (x-y)/(2w)); the halvings are
// collected into one multiplication by N^-1 at the end.
void orc_ntt_inv(void* h, int mod_idx, u64* a) {
    Ctx* c = (Ctx*)h;
    u64 q = c->mod[mod_idx];
    const u64* w_inv = c->psi_brv_inv[mod_idx].data();
    for (int m = c->N / 2, t = 1; m >= 1; m /= 2, t *= 2)
        for (int i = 0; i < m; i++) {
            u64 winv = w_inv[m + i];
            for (int j = 2 * i * t; j < 2 * i * t + t; j++) {
                u64 x = a[j], y = a[j + t];
                a[j] = addmod(x, y, q);
                a[j + t] = mulmod(submod(x, y, q), winv, q);
            }
        }
    u64 ninv = invmod((u64)c->N % q, q);
    for (int i = 0; i < c->N; i++) a[i] = mulmod(a[i], ninv, q);
}

// Several limb-polys at once: poly p uses modulus mod_idx[p % n_limbs].
void orc_ntt_many(void* h, u64* polys, const int* mod_idx, int n_limbs, int batch, int inverse) {
    Ctx* c = (Ctx*)h;
    long total = (long)n_limbs * batch;
#pragma omp parallel for schedule(dynamic)
    for (long p = 0; p < total; p++) {
        u64* a = polys + p * c->N;
        if (inverse) orc_ntt_inv(h, mod_idx[p % n_limbs], a); else orc_ntt_fwd(h, mod_idx[p % n_limbs], a);
    }
}

// Schoolbook product in Z_q[X]/(X^N+1): c_k = sum_{i+j=k} a_i b_j - sum_{i+j=k+N} a_i b_j.
void orc_negacyclic_schoolbook(u64 q, int N, const u64* a, const u64* b, u64* out) {
    for (int k = 0; k < N; k++) out[k] = 0;
    for (int i = 0; i < N; i++)
        for (int j = 0; j < N; j++) {
            u64 p = mulmod(a[i], b[j], q);
            int k = i + j;
            if (k < N) out[k] = addmod(out[k], p, q); else out[k - N] = submod(out[k - N], p, q);
        }
}

// ---------------------------------------------------------------------------------------------
// Automorphism X -> X^g (the permutation half of Rot; Background, "Rotations and Key Switching").
// ---------------------------------------------------------------------------------------------

// Coefficient form: a_i X^i -> a_i X^(i*g); X^N = -1 folds exponents >= N back with a sign flip.
void orc_automorph_coeff(void* h, int mod_idx, u64 g, const u64* a, u64* out) {
    Ctx* c = (Ctx*)h;
    u64 q = c->mod[mod_idx];
    u64 twoN = 2 * (u64)c->N;
    for (int i = 0; i < c->N; i++) {
        u64 e = ((u64)i * g) % twoN;
        if (e < (u64)c->N) out[e] = a[i]; else out[e - c->N] = a[i] ? q - a[i] : 0;
    }
}

// Evaluation form: sigma_g(a)(x) = a(x^g), so the value at psi^(2*brv(k)+1) is the value of a at
// psi^((2*brv(k)+1)*g): a gather, identical for every modulus.
void orc_automorph_ntt(void* h, u64 g, const u64* a, u64* out) {
    Ctx* c = (Ctx*)h;
    u64 twoN = 2 * (u64)c->N;
    for (int k = 0; k < c->N; k++) {
        u64 e = ((2 * (u64)bitrev(k, c->logN) + 1) * g) % twoN;
        out[k] = a[bitrev((uint32_t)((e - 1) / 2), c->logN)];
    }
}

// ---------------------------------------------------------------------------------------------
// Hybrid key switching (Experiments, "HE Security Parameters": key switching with digits).
// ---------------------------------------------------------------------------------------------

int orc_live_digits(void* h, int level) { return live_digits((Ctx*)h, level); }

// Decompose + ModUp.  in: c[level+1][N] (NTT form).  out: digits[beta][level+1+k][N] (NTT form).
void orc_modup(void* h, int level, const u64* cin, u64* digits) {
    Ctx* c = (Ctx*)h;
    int N = c->N, E = level + 1 + c->num_p, beta = live_digits(c, level);
    for (int j = 0; j < beta; j++) {
        int lo = digit_lo(c, j), hi = digit_hi(c, j, level), nd = hi - lo;
        u64* dj = digits + (size_t)j * E * N;
        // coefficient form of the digit's own limbs, scaled: y_i = [a_i * (Q_j/q_i)^-1] mod q_i
        std::vector<u64> y((size_t)nd * N);
#pragma omp parallel for
        for (int a = 0; a < nd; a++) {
            int i = lo + a;
            u64 qi = c->mod[i];
            u64 qhat = 1;  // Q_j / q_i mod q_i
            for (int b = lo; b < hi; b++) if (b != i) qhat = mulmod(qhat, c->mod[b] % qi, qi);
            u64 qhat_inv = invmod(qhat, qi);
            u64* ya = y.data() + (size_t)a * N;
            memcpy(ya, cin + (size_t)i * N, sizeof(u64) * N);
            orc_ntt_inv(h, i, ya);
            for (int x = 0; x < N; x++) ya[x] = mulmod(ya[x], qhat_inv, qi);
        }
#pragma omp parallel for
        for (int e = 0; e < E; e++) {
            int t = ext_modulus(c, level, e);
            u64* out = dj + (size_t)e * N;
            if (t >= lo && t < hi) {  // the digit's own limbs are kept as they are
                memcpy(out, cin + (size_t)t * N, sizeof(u64) * N);
                continue;
            }
            u64 qt = c->mod[t];
            std::vector<u64> qhat_t(nd);  // [Q_j / q_i] mod t
            for (int a = 0; a < nd; a++) {
                u64 v = 1;
                for (int b = lo; b < hi; b++) if (b != lo + a) v = mulmod(v, c->mod[b] % qt, qt);
                qhat_t[a] = v;
            }
            for (int x = 0; x < N; x++) {
                u64 acc = 0;
                for (int a = 0; a < nd; a++) {
                    u64 qa = c->mod[lo + a], ya = y[(size_t)a * N + x];
                    u64 yt = ya % qt;                                  // centred y_a reduced modulo t
                    if (ya > qa / 2) yt = submod(yt, qa % qt, qt);     // (y_a - q_a) mod t
                    acc = addmod(acc, mulmod(yt, qhat_t[a], qt), qt);
                }
                out[x] = acc;
            }
            orc_ntt_fwd(h, t, out);
        }
    }
}

// Inner product with a switching key.  key: [dnum][2][num_q+num_p][N] (NTT form, top level).
// digits: [beta][level+1+k][N].  out: v[2][level+1+k][N].
void orc_key_inner(void* h, int level, const u64* digits, const u64* key, u64* v) {
    Ctx* c = (Ctx*)h;
    int N = c->N, E = level + 1 + c->num_p, M = c->num_q + c->num_p, beta = live_digits(c, level);
#pragma omp parallel for collapse(2)
    for (int comp = 0; comp < 2; comp++)
        for (int e = 0; e < E; e++) {
            int t = ext_modulus(c, level, e);
            u64 qt = c->mod[t];
            u64* out = v + ((size_t)comp * E + e) * N;
            for (int x = 0; x < N; x++) out[x] = 0;
            for (int j = 0; j < beta; j++) {
                const u64* d = digits + ((size_t)j * E + e) * N;
                const u64* kk = key + (((size_t)j * 2 + comp) * M + t) * N;
                for (int x = 0; x < N; x++) out[x] = addmod(out[x], mulmod(d[x], kk[x], qt), qt);
            }
        }
}

// ModDown: v[level+1+k][N] (NTT form) -> u[level+1][N] (NTT form), u = (v - ext([v]_P centred)) / P.
void orc_moddown(void* h, int level, const u64* v, u64* u) {
    Ctx* c = (Ctx*)h;
    int N = c->N, k = c->num_p;
    std::vector<u64> z((size_t)k * N);
#pragma omp parallel for
    for (int a = 0; a < k; a++) {
        int t = c->num_q + a;
        u64 pt = c->mod[t];
        u64 phat = 1;  // P / p_t mod p_t
        for (int b = 0; b < k; b++) if (b != a) phat = mulmod(phat, c->mod[c->num_q + b] % pt, pt);
        u64 phat_inv = invmod(phat, pt);
        u64* za = z.data() + (size_t)a * N;
        memcpy(za, v + (size_t)(level + 1 + a) * N, sizeof(u64) * N);
        orc_ntt_inv(h, t, za);
        for (int x = 0; x < N; x++) za[x] = mulmod(za[x], phat_inv, pt);
    }
#pragma omp parallel for
    for (int i = 0; i <= level; i++) {
        u64 qi = c->mod[i];
        std::vector<u64> phat_i(k);  // [P / p_t] mod q_i
        u64 P_i = 1;                 // P mod q_i
        for (int a = 0; a < k; a++) {
            u64 w = 1;
            for (int b = 0; b < k; b++) if (b != a) w = mulmod(w, c->mod[c->num_q + b] % qi, qi);
            phat_i[a] = w;
            P_i = mulmod(P_i, c->mod[c->num_q + a] % qi, qi);
        }
        u64 Pinv = invmod(P_i, qi);
        std::vector<u64> w(N);
        for (int x = 0; x < N; x++) {
            u64 acc = 0;
            for (int a = 0; a < k; a++) {
                u64 pa = c->mod[c->num_q + a], za = z[(size_t)a * N + x];
                u64 zi = za % qi;                                  // centred z_a reduced modulo q_i
                if (za > pa / 2) zi = submod(zi, pa % qi, qi);     // (z_a - p_a) mod q_i
                acc = addmod(acc, mulmod(zi, phat_i[a], qi), qi);
            }
            w[x] = acc;
        }
        orc_ntt_fwd(h, i, w.data());
        const u64* vi = v + (size_t)i * N;
        u64* ui = u + (size_t)i * N;
        for (int x = 0; x < N; x++) ui[x] = mulmod(submod(vi[x], w[x], qi), Pinv, qi);
    }
}

// Exact-up-to-rounding division by the product D of a set of dropped limbs, written from its definition
// (ModDown is the case "drop the special primes", rescaling the case "drop q_level"; dropping both at
// once divides by P * q_level with a single rounding).  v: [n_keep + n_drop][N] in NTT form, the kept
// limbs first; limb t is modulo moduli[keep_idx[t]] resp. moduli[drop_idx[t - n_keep]].
//   z_a = [v_a * (D/d_a)^-1] mod d_a  centred;   w_i = sum_a z_a * [D/d_a] mod q_i;   out_i = (v_i - w_i) / D mod q_i.
void orc_divide_by_limbs(void* h, const int* keep_idx, int n_keep, const int* drop_idx, int n_drop, const u64* v, u64* out) {
    Ctx* c = (Ctx*)h;
    int N = c->N;
    std::vector<u64> z((size_t)n_drop * N);
#pragma omp parallel for
    for (int a = 0; a < n_drop; a++) {
        u64 da = c->mod[drop_idx[a]];
        u64 dhat = 1;
        for (int b = 0; b < n_drop; b++) if (b != a) dhat = mulmod(dhat, c->mod[drop_idx[b]] % da, da);
        u64 dhat_inv = invmod(dhat, da);
        u64* za = z.data() + (size_t)a * N;
        memcpy(za, v + (size_t)(n_keep + a) * N, sizeof(u64) * N);
        orc_ntt_inv(h, drop_idx[a], za);
        for (int x = 0; x < N; x++) za[x] = mulmod(za[x], dhat_inv, da);
    }
#pragma omp parallel for
    for (int i = 0; i < n_keep; i++) {
        u64 qi = c->mod[keep_idx[i]];
        std::vector<u64> dhat_i(n_drop);
        u64 D_i = 1;
        for (int a = 0; a < n_drop; a++) {
            u64 w = 1;
            for (int b = 0; b < n_drop; b++) if (b != a) w = mulmod(w, c->mod[drop_idx[b]] % qi, qi);
            dhat_i[a] = w;
            D_i = mulmod(D_i, c->mod[drop_idx[a]] % qi, qi);
        }
        u64 Dinv = invmod(D_i, qi);
        std::vector<u64> w(N);
        for (int x = 0; x < N; x++) {
            u64 acc = 0;
            for (int a = 0; a < n_drop; a++) {
                u64 da = c->mod[drop_idx[a]], za = z[(size_t)a * N + x];
                u64 zi = za % qi;
                if (za > da / 2) zi = submod(zi, da % qi, qi);     // centred z_a reduced modulo q_i
                acc = addmod(acc, mulmod(zi, dhat_i[a], qi), qi);
            }
            w[x] = acc;
        }
        orc_ntt_fwd(h, keep_idx[i], w.data());
        const u64* vi = v + (size_t)i * N;
        u64* oi = out + (size_t)i * N;
        for (int x = 0; x < N; x++) oi[x] = mulmod(submod(vi[x], w[x], qi), Dinv, qi);
    }
}

// KeySwitch(c, key): [level+1][N] -> out[2][level+1][N] with out0 + out1*s ~ c * s'.
void orc_keyswitch(void* h, int level, const u64* cin, const u64* key, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, E = level + 1 + c->num_p, beta = live_digits(c, level);
    std::vector<u64> digits(beta * E * N), v(2 * E * N);
    orc_modup(h, level, cin, digits.data());
    orc_key_inner(h, level, digits.data(), key, v.data());
    orc_moddown(h, level, v.data(), out);
    orc_moddown(h, level, v.data() + E * N, out + (size_t)(level + 1) * N);
}

// Rot with the automorphism applied to the ciphertext first (unhoisted order).
// ct: [2][level+1][N]; key switches from sigma_g(s) to s; out: [2][level+1][N].
void orc_rotate_unhoisted(void* h, int level, u64 g, const u64* ct, const u64* key, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
    std::vector<u64> pc0(L1 * N), pc1(L1 * N);
    for (size_t i = 0; i < L1; i++) {
        orc_automorph_ntt(h, g, ct + i * N, pc0.data() + i * N);
        orc_automorph_ntt(h, g, ct + (L1 + i) * N, pc1.data() + i * N);
    }
    orc_keyswitch(h, level, pc1.data(), key, out);
    for (size_t i = 0; i < L1; i++)
        for (size_t x = 0; x < N; x++)
            out[i * N + x] = addmod(out[i * N + x], pc0[i * N + x], c->mod[i]);
}

// Rot with a shared decomposition (hoisted order): digits = ModUp(c1) computed once by the caller
// (orc_modup on c1), then for each g: permute every extended limb, inner product, ModDown.
void orc_rotate_hoisted(void* h, int level, u64 g, const u64* ct, const u64* digits, const u64* key, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1, E = L1 + c->num_p, beta = live_digits(c, level);
    std::vector<u64> pd(beta * E * N), v(2 * E * N);
    for (size_t p = 0; p < beta * E; p++) orc_automorph_ntt(h, g, digits + p * N, pd.data() + p * N);
    orc_key_inner(h, level, pd.data(), key, v.data());
    orc_moddown(h, level, v.data(), out);
    orc_moddown(h, level, v.data() + E * N, out + L1 * N);
    std::vector<u64> pc0(N);
    for (size_t i = 0; i < L1; i++) {
        orc_automorph_ntt(h, g, ct + i * N, pc0.data());
        for (size_t x = 0; x < N; x++) out[i * N + x] = addmod(out[i * N + x], pc0[x], c->mod[i]);
    }
}

// ---------------------------------------------------------------------------------------------
// Pointwise ciphertext arithmetic.
// ---------------------------------------------------------------------------------------------

// acc[c][i][x] (+)= sum_k pt_k[i][x] * ct_k[c][i][x] mod q_i  (Eq. 11 and the channel sum).
// pts: n_terms pointers to [level+1][N]; cts: n_terms pointers to [2][level+1][N].
void orc_ptct_mac(void* h, int level, int n_terms, const u64* const* pts, const u64* const* cts, u64* acc, int accumulate) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
#pragma omp parallel for collapse(2)
    for (int comp = 0; comp < 2; comp++)
        for (size_t i = 0; i < L1; i++) {
            u64 q = c->mod[i];
            u64* a = acc + (comp * L1 + i) * N;
            if (!accumulate) for (size_t x = 0; x < N; x++) a[x] = 0;
            for (int k = 0; k < n_terms; k++) {
                const u64* p = pts[k] + i * N;
                const u64* t = cts[k] + (comp * L1 + i) * N;
                for (size_t x = 0; x < N; x++) a[x] = addmod(a[x], mulmod(p[x], t[x], q), q);
            }
        }
}

// poly[i][x] * scalar[i] mod q_i over limbs 0..level (an integer scalar given by its residues).
void orc_scalar_mul(void* h, int level, int n_comp, const u64* poly, const u64* scalar, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
    for (int comp = 0; comp < n_comp; comp++)
        for (size_t i = 0; i < L1; i++)
            for (size_t x = 0; x < N; x++)
                out[(comp * L1 + i) * N + x] = mulmod(poly[(comp * L1 + i) * N + x], scalar[i], c->mod[i]);
}

// a (.) b on a list of limbs: out[t][x] = a[t][x] * b[t][x] mod moduli[mod_idx[t]].
void orc_mul(void* h, const int* mod_idx, int n_mod, const u64* a, const u64* b, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N;
    for (int t = 0; t < n_mod; t++)
        for (size_t x = 0; x < N; x++) out[t * N + x] = mulmod(a[t * N + x], b[t * N + x], c->mod[mod_idx[t]]);
}

// The multiply-accumulate of Eq. 11 on an explicit list of moduli (the extended basis Q_l P of a
// convolution whose division by P comes after the sum): acc[c][t][x] (+)= sum_k pt_k[t][x] * x_k[c][t][x]
// mod moduli[mod_idx[t]].  pts: n_terms pointers to [n_mod][N]; xs: n_terms pointers to [2][n_mod][N].
void orc_mac_on_moduli(void* h, const int* mod_idx, int n_mod, int n_terms, const u64* const* pts, const u64* const* xs, u64* acc,
                       int accumulate) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N;
#pragma omp parallel for collapse(2)
    for (int comp = 0; comp < 2; comp++)
        for (int t = 0; t < n_mod; t++) {
            u64 q = c->mod[mod_idx[t]];
            u64* a = acc + ((size_t)comp * n_mod + t) * N;
            if (!accumulate) for (size_t x = 0; x < N; x++) a[x] = 0;
            for (int k = 0; k < n_terms; k++) {
                const u64* p = pts[k] + (size_t)t * N;
                const u64* v = xs[k] + ((size_t)comp * n_mod + t) * N;
                for (size_t x = 0; x < N; x++) a[x] = addmod(a[x], mulmod(p[x], v[x], q), q);
            }
        }
}

// poly[t][x] * scalar[t] mod moduli[mod_idx[t]] (an integer scalar given by its residues).
void orc_scalar_mul_on_moduli(void* h, const int* mod_idx, int n_mod, int n_comp, const u64* poly, const u64* scalar, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N;
    for (int comp = 0; comp < n_comp; comp++)
        for (int t = 0; t < n_mod; t++)
            for (size_t x = 0; x < N; x++)
                out[((size_t)comp * n_mod + t) * N + x] = mulmod(poly[((size_t)comp * n_mod + t) * N + x], scalar[t], c->mod[mod_idx[t]]);
}

void orc_add(void* h, int level, int n_comp, const u64* a, const u64* b, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
    for (int comp = 0; comp < n_comp; comp++)
        for (size_t i = 0; i < L1; i++)
            for (size_t x = 0; x < N; x++)
                out[(comp * L1 + i) * N + x] = addmod(a[(comp * L1 + i) * N + x], b[(comp * L1 + i) * N + x], c->mod[i]);
}

// Rescale: divide by the last live prime with rounding to nearest.  in [2][level+1][N] -> out
// [2][level][N].  r = centred coefficient-form remainder of limb `level`; c'_i = (c_i - r) / q_level.
void orc_rescale(void* h, int level, const u64* ct, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
    u64 ql = c->mod[level];
    for (int comp = 0; comp < 2; comp++) {
        std::vector<u64> r(ct + (comp * L1 + level) * N, ct + (comp * L1 + level + 1) * N);
        orc_ntt_inv(h, level, r.data());
#pragma omp parallel for
        for (int i = 0; i < level; i++) {
            u64 qi = c->mod[i];
            u64 qlinv = invmod(ql % qi, qi);
            std::vector<u64> w(N);
            for (size_t x = 0; x < N; x++) {
                // centred representative of r[x] modulo q_level, reduced modulo q_i
                if (r[x] > ql / 2) w[x] = submod(r[x] % qi, ql % qi, qi); else w[x] = r[x] % qi;
            }
            orc_ntt_fwd(h, i, w.data());
            const u64* ci = ct + (comp * L1 + i) * N;
            u64* oi = out + ((size_t)comp * level + i) * N;
            for (size_t x = 0; x < N; x++) oi[x] = mulmod(submod(ci[x], w[x], qi), qlinv, qi);
        }
    }
}

// ct-ct multiply + relinearise: d0 = a0 b0, d1 = a0 b1 + a1 b0, d2 = a1 b1;
// out = (d0, d1) + KeySwitch(d2, rlk), rlk switching from s^2 to s.  No rescale.
void orc_ctct_mul_relin(void* h, int level, const u64* a, const u64* b, const u64* rlk, u64* out) {
    Ctx* c = (Ctx*)h;
    size_t N = c->N, L1 = level + 1;
    std::vector<u64> d0(L1 * N), d1(L1 * N), d2(L1 * N);
    for (size_t i = 0; i < L1; i++) {
        u64 q = c->mod[i];
        for (size_t x = 0; x < N; x++) {
            size_t o = i * N + x;
            u64 a0 = a[o], a1 = a[L1 * N + o], b0 = b[o], b1 = b[L1 * N + o];
            d0[o] = mulmod(a0, b0, q);
            d1[o] = addmod(mulmod(a0, b1, q), mulmod(a1, b0, q), q);
            d2[o] = mulmod(a1, b1, q);
        }
    }
    orc_keyswitch(h, level, d2.data(), rlk, out);
    for (size_t i = 0; i < L1; i++)
        for (size_t x = 0; x < N; x++) {
            size_t o = i * N + x;
            out[o] = addmod(out[o], d0[o], c->mod[i]);
            out[L1 * N + o] = addmod(out[L1 * N + o], d1[o], c->mod[i]);
        }
}

// ---------------------------------------------------------------------------------------------
// Client side (Threat Model: the client encrypts and decrypts; the server never sees the secret).
// ---------------------------------------------------------------------------------------------

struct Rng {
    u64 s[4];
    static u64 splitmix(u64& x) {
        u64 z = (x += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    explicit Rng(u64 seed) { for (int i = 0; i < 4; i++) s[i] = splitmix(seed); }
    static u64 rotl(u64 x, int k) { return (x << k) | (x >> (64 - k)); }
    u64 next() {  // xoshiro256**
        u64 r = rotl(s[1] * 5, 7) * 9, t = s[1] << 17;
        s[2] ^= s[0]; s[3] ^= s[1]; s[1] ^= s[2]; s[0] ^= s[3]; s[2] ^= t; s[3] = rotl(s[3], 45);
        return r;
    }
    u64 below(u64 q) {  // uniform in [0, q) by rejection
        u64 lim = (~(u64)0) / q * q;
        for (;;) { u64 r = next(); if (r < lim) return r % q; }
    }
    double unit() { return ((next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }  // (0,1)
};

void orc_sample_ternary(u64 seed, int n, int8_t* out) {
    Rng r(seed);
    for (int i = 0; i < n; i++) out[i] = (int8_t)((int)r.below(3) - 1);
}
void orc_sample_gauss(u64 seed, int n, int8_t* out) {
    Rng r(seed);
    for (int i = 0; i < n; i++) {
        for (;;) {
            double z = std::sqrt(-2.0 * std::log(r.unit())) * std::cos(2.0 * M_PI * r.unit());
            long e = std::lround(3.2 * z);
            if (e >= -19 && e <= 19) { out[i] = (int8_t)e; break; }
        }
    }
}
void orc_sample_uniform(u64 seed, u64 q, int n, u64* out) {
    Rng r(seed);
    for (int i = 0; i < n; i++) out[i] = r.below(q);
}

// Signed integer coefficients -> residues modulo each listed modulus -> NTT form.
// out[n_mod][N].
void orc_lift_ntt(void* h, const i64* coeffs, const int* mod_idx, int n_mod, u64* out) {
    Ctx* c = (Ctx*)h;
#pragma omp parallel for
    for (int a = 0; a < n_mod; a++) {
        u64 q = c->mod[mod_idx[a]];
        u64* o = out + (size_t)a * c->N;
        for (int x = 0; x < c->N; x++) {
            i64 v = coeffs[x];
            o[x] = v >= 0 ? (u64)v % q : (q - ((u64)(-v) % q)) % q;
        }
        orc_ntt_fwd(h, mod_idx[a], o);
    }
}

// Switching key from s' to s over all num_q+num_p moduli, dnum digits:
//   a_j uniform, b_j = -a_j s + e_j + F_j s',  F_j = P mod q_i on the digit's own limbs, 0 elsewhere.
// s_ntt, sp_ntt: [num_q+num_p][N] NTT form.  key: [dnum][2][num_q+num_p][N] with comp 0 = b, 1 = a.
// a_in: null (a_j drawn from the key's own sequential streams) or [dnum][num_q+num_p][N] given by the caller
// (the seed-expanded public halves of a staged key).
void orc_gen_switch_key_with_a(void* h, const u64* s_ntt, const u64* sp_ntt, u64 seed, const u64* a_in, u64* key) {
    Ctx* c = (Ctx*)h;
    int N = c->N, M = c->num_q + c->num_p;
    std::vector<int> all(M);
    for (int t = 0; t < M; t++) all[t] = t;
    for (int j = 0; j < c->dnum; j++) {
        std::vector<int8_t> e8(N);
        orc_sample_gauss(seed + 1000003ull * (2 * j + 1), N, e8.data());
        std::vector<i64> e(e8.begin(), e8.end());
        std::vector<u64> e_ntt((size_t)M * N);
        orc_lift_ntt(h, e.data(), all.data(), M, e_ntt.data());
        int lo = digit_lo(c, j), hi = (j + 1) * c->alpha < c->num_q ? (j + 1) * c->alpha : c->num_q;
#pragma omp parallel for
        for (int t = 0; t < M; t++) {
            u64 q = c->mod[t];
            u64* b = key + (((size_t)j * 2 + 0) * M + t) * N;
            u64* a = key + (((size_t)j * 2 + 1) * M + t) * N;
            if (a_in) std::memcpy(a, a_in + ((size_t)j * M + t) * N, (size_t)N * sizeof(u64));
            else orc_sample_uniform(seed + 7919ull * ((u64)j * M + t + 1), q, N, a);
            u64 F = 0;
            if (t >= lo && t < hi) { F = 1; for (int p = 0; p < c->num_p; p++) F = mulmod(F, c->mod[c->num_q + p] % q, q); }
            for (int x = 0; x < N; x++) {
                size_t o = (size_t)t * N + x;
                u64 v = submod(e_ntt[o], mulmod(a[x], s_ntt[o], q), q);
                b[x] = addmod(v, mulmod(F, sp_ntt[o], q), q);
            }
        }
    }
}

void orc_gen_switch_key(void* h, const u64* s_ntt, const u64* sp_ntt, u64 seed, u64* key) {
    orc_gen_switch_key_with_a(h, s_ntt, sp_ntt, seed, nullptr, key);
}

// Symmetric encryption of integer coefficients m at `level`: ct = (-a s + m + e, a), NTT form.
void orc_encrypt(void* h, int level, const i64* m, const u64* s_ntt, u64 seed, u64* ct) {
    Ctx* c = (Ctx*)h;
    int N = c->N, L1 = level + 1;
    std::vector<int8_t> e8(N);
    orc_sample_gauss(seed, N, e8.data());
    std::vector<i64> me(N);
    for (int x = 0; x < N; x++) me[x] = m[x] + e8[x];
    std::vector<int> idx(L1);
    for (int i = 0; i < L1; i++) idx[i] = i;
    orc_lift_ntt(h, me.data(), idx.data(), L1, ct);
    for (int i = 0; i < L1; i++) {
        u64 q = c->mod[i];
        u64* c0 = ct + (size_t)i * N;
        u64* c1 = ct + (size_t)(L1 + i) * N;
        orc_sample_uniform(seed + 104729ull * (i + 1), q, N, c1);
        for (int x = 0; x < N; x++) c0[x] = submod(c0[x], mulmod(c1[x], s_ntt[(size_t)i * N + x], q), q);
    }
}

// Decrypt: c0 + c1 s, back to coefficients, centred integer via CRT over the first one or two
// limbs (the plaintext plus noise is far below q_0 q_1 / 2 in every workload here), as doubles.
void orc_decrypt(void* h, int level, const u64* ct, const u64* s_ntt, double* out) {
    Ctx* c = (Ctx*)h;
    int N = c->N, L1 = level + 1, use = L1 < 2 ? L1 : 2;
    std::vector<u64> m((size_t)use * N);
    for (int i = 0; i < use; i++) {
        u64 q = c->mod[i];
        for (int x = 0; x < N; x++)
            m[(size_t)i * N + x] = addmod(ct[(size_t)i * N + x], mulmod(ct[(size_t)(L1 + i) * N + x], s_ntt[(size_t)i * N + x], q), q);
        orc_ntt_inv(h, i, m.data() + (size_t)i * N);
    }
    if (use == 1) {
        u64 q = c->mod[0];
        for (int x = 0; x < N; x++) { u64 v = m[x]; out[x] = v > q / 2 ? -(double)(q - v) : (double)v; }
        return;
    }
    u64 q0 = c->mod[0], q1 = c->mod[1];
    u64 q0inv1 = invmod(q0 % q1, q1);
    u128 Q = (u128)q0 * q1;
    for (int x = 0; x < N; x++) {
        // v = m0 + q0 * ((m1 - m0) / q0 mod q1)
        u64 m0 = m[x], m1 = m[(size_t)N + x];
        u64 k = mulmod(submod(m1, m0 % q1, q1), q0inv1, q1);
        u128 v = (u128)m0 + (u128)q0 * k;
        out[x] = v > Q / 2 ? -(double)(Q - v) : (double)v;
    }
}

}  // extern "C"
