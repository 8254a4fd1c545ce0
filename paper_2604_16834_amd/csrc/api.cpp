// The C boundary: argument checks, workspace carving and the order of kernel launches of every
// exported operation.  No arithmetic happens on the host; no call here allocates or synchronises.
//
// Work is batched wherever operands are independent: the channel ciphertexts of a layer share their
// rotation and relinearisation keys, so up to CT_BATCH of them go through every kernel of a key
// switch together (the key streams from HBM once per batch, NTT launches are large enough to fill
// the chip); the rotations of one ciphertext share its extended digits (hoisting).
#include <cstdio>
#include <new>
#include <vector>

#include "ctx.h"

namespace {

int set_err(const ckks_ctx* c, int code, const char* msg) {
    if (c) c->err = msg;
    return code;
}

#define HIP_TRY(expr)                                                              \
    do {                                                                           \
        hipError_t e__ = (expr);                                                   \
        if (e__ != hipSuccess) {                                                   \
            c->err = std::string(#expr ": ") + hipGetErrorString(e__);             \
            return CKKS_ERR_HIP;                                                   \
        }                                                                          \
    } while (0)

// bump allocator over the caller's workspace (256-byte aligned blocks of u64)
int set_hip_err(const ckks_ctx* c, hipError_t e) {
    c->err = std::string("HIP: ") + hipGetErrorString(e);
    return CKKS_ERR_HIP;
}

struct Arena {
    char* base;
    size_t cap, used;
    Arena(void* p, size_t n) : base((char*)p), cap(n), used(0) {}
    u64* take(size_t elems) {
        size_t bytes = (elems * sizeof(u64) + 255) & ~(size_t)255;
        if (!base || used + bytes > cap) { used = cap + 1; return nullptr; }
        u64* r = (u64*)(base + used);
        used += bytes;
        return r;
    }
    bool ok() const { return used <= cap; }
    Arena rest() const { return ok() ? Arena(base + used, cap - used) : Arena(nullptr, 0); }
};
size_t blk(size_t elems) { return (elems * sizeof(u64) + 255) & ~(size_t)255; }

PolyList range_list(u32 first_pos, u32 count, u32 first_mod) {
    PolyList pl;
    pl.n = count;
    for (u32 a = 0; a < CKKS_MAX_MODULI; a++) {
        pl.spos[a] = pl.dpos[a] = (unsigned char)(a < count ? first_pos + a : 0);
        pl.mod[a] = (unsigned char)(a < count ? first_mod + a : 0);
    }
    return pl;
}

PtrList8 ptr_list(const u64* const* p, u32 n) {
    PtrList8 l;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) l.p[b] = b < n ? p[b] : nullptr;
    return l;
}
OutList8 out_list(u64* const* p, u32 n) {
    OutList8 l;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) l.p[b] = b < n ? p[b] : nullptr;
    return l;
}

bool level_ok(const ckks_ctx* c, u32 level) { return level < c->num_q; }

// ---- key-switch workspace: n_dig polynomials being decomposed, n_v key switches in flight ----------
struct KsWs {
    u64 *y, *digits, *v, *w;
    size_t y_b, dig_b, v_b, w_b;  // per-item strides in elements
    mutable const u64* own[CT_BATCH] = {};  // the polynomials run_modup decomposed last (the digits' own limbs stay there)
};
// the digits of items b0, b0 + 1, ... of the batch in ws, as the inner-product kernels take them
DigitSrc dsrc(const ckks_ctx* c, const KsWs& ws, u32 b0) {
    DigitSrc d;
    d.digits = ws.digits + b0 * ws.dig_b;
    d.bstride = ws.dig_b;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) d.own.p[b] = b0 + b < CT_BATCH ? ws.own[b0 + b] : nullptr;
    d.alpha = c->alpha;
    d.pad = 0;
    return d;
}
size_t ws_ks(const ckks_ctx* c, u32 level, u32 n_dig, u32 n_v) {
    const size_t N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    return blk(n_dig * L1 * N) + blk(n_dig * beta * E * N) + blk(n_v * 2 * E * N) + blk(n_v * 2 * L1 * N);
}
bool carve_ks(const ckks_ctx* c, u32 level, u32 n_dig, u32 n_v, Arena& ar, KsWs& b) {
    const size_t N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    b.y_b = L1 * N;
    b.dig_b = beta * E * N;
    b.v_b = 2 * E * N;
    b.w_b = 2 * L1 * N;
    b.y = ar.take(n_dig * b.y_b);
    b.digits = ar.take(n_dig * b.dig_b);
    b.v = ar.take(n_v * b.v_b);
    b.w = ar.take(n_v * b.w_b);
    return ar.ok();
}
size_t ws_rescale(const ckks_ctx* c, u32 level, u32 n) { return blk(2 * (size_t)n * c->N) + blk(2 * (size_t)n * level * c->N); }
size_t ws_ctct(const ckks_ctx* c, u32 level, u32 n) { return 3 * blk((size_t)n * (level + 1) * c->N) + ws_ks(c, level, n, n); }

// Decompose + ModUp of n <= CT_BATCH polynomials srcs[b] ([level+1][N], NTT form) into
// ws.digits + b*ws.dig_b ([beta][E][N], NTT form).
// hi_only (double-precision transforms only): the forward transforms stop after their first pass; the caller finishes them
// inside the inner product (launch_ntt_lo_mac).
// muls (with hi_only): the polynomial to decompose is srcs[b] (.) muls[b], formed as the inverse transform loads it.
int run_modup(const ckks_ctx* c, u32 level, const u64* const* srcs, u32 n, const KsWs& ws, hipStream_t st, bool hi_only = false,
              const u64* const* muls = nullptr) {
    const u32 N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    for (u32 b = 0; b < CT_BATCH; b++) ws.own[b] = (b < n && !muls) ? srcs[b] : nullptr;  // a product has no stored own limbs
    if (muls && !hi_only) return set_err(c, CKKS_ERR_INVALID_ARG, "internal: product source without the fused inner product");
    // all live limbs of every polynomial to coefficient form at once.  With double-precision transforms the inverse scales
    // limb i by N^-1 (Q_j/q_i)^-1 and leaves the centred residue as a double, and each digit's basis conversion happens
    // inside the first pass of the forward transforms of its target limbs (no conversion kernel, no coefficient-form copy
    // of the extended digit).
    const bool fused = ntt_has_modup(c);
    if (hi_only && !fused) return set_err(c, CKKS_ERR_INVALID_ARG, "internal: fused inner product without fused ModUp");
    HIP_TRY(launch_ntt(c, true, nullptr, 0, ws.y, L1, range_list(0, L1, 0), n, st, srcs, nullptr,
                       fused ? c->d_modup_prep_f + (size_t)level * c->num_q : nullptr, muls));  // (positions 0..level are moduli 0..level)
    const PtrList8 cl = ptr_list(srcs, n);
    for (u32 j = 0; j < beta; j++) {
        const u32 lo = c->digit_lo(j), hi = c->digit_hi(j, level);
        u64* digit = ws.digits + (size_t)j * E * N;
        if (!fused) HIP_TRY(launch_modup_conv(c, level, j, ws.y + (size_t)lo * N, ws.y_b, cl, digit, ws.dig_b, n, st));
        PolyList pl;
        pl.n = 0;
        for (u32 e = 0; e < E; e++) {
            const u32 t = c->ext_modulus(level, e);
            if (t >= lo && t < hi) continue;
            pl.spos[pl.n] = pl.dpos[pl.n] = (unsigned char)e;
            pl.mod[pl.n] = (unsigned char)t;
            pl.n++;
        }
        for (u32 a = pl.n; a < CKKS_MAX_MODULI; a++) pl.spos[a] = pl.dpos[a] = pl.mod[a] = 0;
        if (fused) HIP_TRY(launch_ntt_modup(c, level, j, (const double*)ws.y, ws.y_b, digit, (size_t)beta * E, pl, n, st, hi_only));
        else HIP_TRY(launch_ntt(c, false, digit, (size_t)beta * E, digit, (size_t)beta * E, pl, n, st));
    }
    return CKKS_OK;
}

// What the forward transform of the converted dropped part does to its results instead of storing them (see FwdEpilogue).
FwdEpilogue moddown_epilogue(const ckks_ctx* c, u32 level, bool merged, const u64* v, const FinalItem* items, u32 n) {
    FwdEpilogue ep;
    const u32 kp = merged ? c->k2_pad : c->k_pad;
    const u64* tab = merged ? c->moddown_rs_table(level) : c->d_moddown;
    ep.v = v;
    ep.cinv = tab + 2 * kp + (size_t)kp * c->num_q;
    ep.mci = c->d_mc;
    ep.E = c->ext_limbs(level);
    ep.n_out = merged ? level : level + 1;
    ep.num_q = c->num_q;
    ep.use_vl = 0;
    ep.v_cstride = ep.v2_cstride = 0;
    for (u32 r = 0; r < KS_MAX_BATCH; r++) ep.vl.p[r] = ep.vl2.p[r] = nullptr;
    for (u32 r = 0; r < KS_MAX_BATCH; r++) ep.B.it[r] = r < n ? items[r] : FinalItem{nullptr, nullptr, nullptr, nullptr, 1, 0};
    return ep;
}

// ModDown of the n inner products sitting in ws.v: one pass of each kernel over the whole batch.
// items[r] says what is added to / multiplied into the r-th result and where it goes ([2][level+1][N]).
// merged: the division is by P*q_level (ModDown and rescale in one): the dropped limbs are position
// level and the special primes, the results are [2][level][N].
int run_moddown(const ckks_ctx* c, u32 level, const KsWs& ws, u32 n, const FinalItem* items, hipStream_t st, bool merged = false) {
    const u32 L1 = level + 1, E = c->ext_limbs(level), k = c->num_p;
    if (merged) {
        PolyList dl = range_list(level, k + 1, c->num_q - 1);  // positions level.. ; moduli fixed up below
        dl.mod[0] = (unsigned char)level;
        for (u32 a = 1; a <= k; a++) dl.mod[a] = (unsigned char)(c->num_q + a - 1);
        if (ntt_has_modup(c)) {  // conversion inside the forward transform's first pass, last step inside its second
            HIP_TRY(launch_ntt(c, true, ws.v, E, ws.v, E, dl, 2 * n, st, nullptr, nullptr, c->d_moddown_rs_prep_f + (size_t)level * c->M));
            const FwdEpilogue ep = moddown_epilogue(c, level, true, ws.v, items, n);
            HIP_TRY(launch_ntt_moddown(c, level, true, (const double*)ws.v, ws.w, 2 * n, st, &ep));
            return CKKS_OK;
        }
        HIP_TRY(launch_ntt(c, true, ws.v, E, ws.v, E, dl, 2 * n, st));
        HIP_TRY(launch_moddown_conv(c, level, true, ws.v, ws.w, 2 * n, st));
        if (ntt_has_epilogue(c)) {  // the last step rides on the transform's stores
            const FwdEpilogue ep = moddown_epilogue(c, level, true, ws.v, items, n);
            HIP_TRY(launch_ntt(c, false, ws.w, level, ws.w, level, range_list(0, level, 0), 2 * n, st, nullptr, &ep));
            return CKKS_OK;
        }
        HIP_TRY(launch_ntt(c, false, ws.w, level, ws.w, level, range_list(0, level, 0), 2 * n, st));
        HIP_TRY(launch_moddown_final(c, level, true, ws.v, ws.w, items, n, st));
        return CKKS_OK;
    }
    if (ntt_has_modup(c)) {
        HIP_TRY(launch_ntt(c, true, ws.v, E, ws.v, E, range_list(L1, k, c->num_q), 2 * n, st, nullptr, nullptr, c->d_moddown_prep_f));
        const FwdEpilogue ep = moddown_epilogue(c, level, false, ws.v, items, n);
        HIP_TRY(launch_ntt_moddown(c, level, false, (const double*)ws.v, ws.w, 2 * n, st, &ep));
        return CKKS_OK;
    }
    HIP_TRY(launch_ntt(c, true, ws.v, E, ws.v, E, range_list(L1, k, c->num_q), 2 * n, st));  // P-part -> coefficients
    HIP_TRY(launch_moddown_conv(c, level, false, ws.v, ws.w, 2 * n, st));
    if (ntt_has_epilogue(c)) {
        const FwdEpilogue ep = moddown_epilogue(c, level, false, ws.v, items, n);
        HIP_TRY(launch_ntt(c, false, ws.w, L1, ws.w, L1, range_list(0, L1, 0), 2 * n, st, nullptr, &ep));
        return CKKS_OK;
    }
    HIP_TRY(launch_ntt(c, false, ws.w, L1, ws.w, L1, range_list(0, L1, 0), 2 * n, st));
    HIP_TRY(launch_moddown_final(c, level, false, ws.v, ws.w, items, n, st));
    return CKKS_OK;
}

// n <= CT_BATCH ciphertexts cts[b] (component stride ct_cstride) rescaled from `level` into outs[b]
int run_rescale(const ckks_ctx* c, u32 level, const u64* const* cts, size_t ct_cstride, u64* const* outs, u32 n, Arena ar,
                hipStream_t st) {
    const size_t N = c->N;
    u64* r = ar.take(2 * (size_t)n * N);
    u64* w = ar.take(2 * (size_t)n * level * N);
    if (!ar.ok()) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rescale");
    const u64* last[KS_MAX_BATCH];  // the dropped limb of every component
    for (u32 b = 0; b < n; b++) {
        last[2 * b] = cts[b] + (size_t)level * N;
        last[2 * b + 1] = cts[b] + ct_cstride + (size_t)level * N;
    }
    if (ntt_has_modup(c)) {
        // the rescale as a division by one dropped limb through the fused passes: the inverse transform leaves centred doubles,
        // the forward transform reduces them modulo each remaining limb as it loads and applies (c_i - w_i) q_level^-1 as it stores
        HIP_TRY(launch_ntt(c, true, nullptr, 0, r, 1, range_list(0, 1, level), 2 * n, st, last, nullptr, c->d_rescale_prep_f));
        FwdEpilogue ep;
        ep.v = nullptr;
        ep.cinv = c->d_rescale_ep + (size_t)level * 2 * c->num_q;
        ep.mci = c->d_mc;
        ep.E = 0;
        ep.n_out = level;
        ep.num_q = c->num_q;
        ep.use_vl = 1;
        ep.v_cstride = ct_cstride;
        ep.v2_cstride = 0;
        for (u32 b = 0; b < KS_MAX_BATCH; b++) {
            ep.vl2.p[b] = nullptr;
            ep.vl.p[b] = b < n ? cts[b] : nullptr;
            ep.B.it[b] = b < n ? FinalItem{nullptr, nullptr, nullptr, outs[b], 1, 0} : FinalItem{nullptr, nullptr, nullptr, nullptr, 1, 0};
        }
        HIP_TRY(launch_ntt_rescale(c, level, (const double*)r, w, 2 * n, st, &ep));
        return CKKS_OK;
    }
    HIP_TRY(launch_ntt(c, true, nullptr, 0, r, 1, range_list(0, 1, level), 2 * n, st, last));
    HIP_TRY(launch_rescale_conv(c, level, r, w, 2 * n, st));
    HIP_TRY(launch_ntt(c, false, w, level, w, level, range_list(0, level, 0), 2 * n, st));
    HIP_TRY(launch_rescale_final(c, level, ptr_list(cts, n), ct_cstride, w, out_list(outs, n), n, st));
    return CKKS_OK;
}

// The same for Rescale(ka * x[b] + kb * y[b]) (double-precision contexts with the fused passes): the linear combination is
// formed where it is read, in the inverse transform of the dropped limb and in the division's last step.
int run_rescale_lin(const ckks_ctx* c, u32 level, const u64* const* xs, size_t x_cstride, const u64* ka, const u64* const* ys,
                    size_t y_cstride, const u64* kb, u64* const* outs, u32 n, Arena ar, hipStream_t st) {
    if (!ntt_has_modup(c)) return set_err(c, CKKS_ERR_INVALID_ARG, "internal: fused rescale of a linear combination");
    const size_t N = c->N;
    u64* r = ar.take(2 * (size_t)n * N);
    u64* w = ar.take(2 * (size_t)n * level * N);
    if (!ar.ok()) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rescale");
    const u64 *last[KS_MAX_BATCH], *last2[KS_MAX_BATCH];
    for (u32 b = 0; b < n; b++) {
        last[2 * b] = xs[b] + (size_t)level * N;
        last[2 * b + 1] = xs[b] + x_cstride + (size_t)level * N;
        last2[2 * b] = ys[b] + (size_t)level * N;
        last2[2 * b + 1] = ys[b] + y_cstride + (size_t)level * N;
    }
    const u64 lin_k[2] = {ka[level], kb[level]};
    HIP_TRY(launch_ntt(c, true, nullptr, 0, r, 1, range_list(0, 1, level), 2 * n, st, last, nullptr, c->d_rescale_prep_f, last2, lin_k));
    FwdEpilogue ep;
    ep.v = nullptr;
    ep.cinv = c->d_rescale_ep + (size_t)level * 2 * c->num_q;
    ep.mci = c->d_mc;
    ep.E = 0;
    ep.n_out = level;
    ep.num_q = c->num_q;
    ep.use_vl = 2;
    ep.v_cstride = x_cstride;
    ep.v2_cstride = y_cstride;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) {
        ep.vl.p[b] = b < n ? xs[b] : nullptr;
        ep.vl2.p[b] = b < n ? ys[b] : nullptr;
        ep.B.it[b] = b < n ? FinalItem{nullptr, nullptr, nullptr, outs[b], 1, 0} : FinalItem{nullptr, nullptr, nullptr, nullptr, 1, 0};
    }
    for (u32 i = 0; i < CKKS_MAX_MODULI; i++) {
        ep.ka[i] = i < level ? ka[i] : 0;
        ep.kb[i] = i < level ? kb[i] : 0;
    }
    HIP_TRY(launch_ntt_rescale(c, level, (const double*)r, w, 2 * n, st, &ep));
    return CKKS_OK;
}

// n <= CT_BATCH products a[b]*b[b] with relinearisation (operands possibly at a higher level:
// component strides given); outs[b] = [2][level+1][N]
int run_ctct(const ckks_ctx* c, u32 level, const u64* const* a, size_t a_cstride, const u64* const* b, size_t b_cstride,
             const u64* d_rlk, u64* const* outs, u32 n, Arena ar, hipStream_t st) {
    const size_t N = c->N, L1 = level + 1;
    u64* d0 = ar.take(n * L1 * N);
    u64* d1 = ar.take(n * L1 * N);
    u64* d2 = ar.take(n * L1 * N);
    KsWs ws;
    if (!carve_ks(c, level, n, n, ar, ws)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for ct-ct multiply");
    HIP_TRY(launch_tensor(c, level, ptr_list(a, n), a_cstride, ptr_list(b, n), b_cstride, d0, d1, d2, n, nullptr, 0, st));
    const u64* d2s[CT_BATCH];
    FinalItem items[CT_BATCH];
    for (u32 i = 0; i < n; i++) {
        d2s[i] = d2 + i * L1 * N;
        items[i] = FinalItem{d0 + i * L1 * N, d1 + i * L1 * N, nullptr, outs[i], 1, 0};
    }
    const bool mac = ntt_has_modup(c);  // the inner product inside the forward transforms' second pass
    int rc = run_modup(c, level, d2s, n, ws, st, mac);
    if (rc) return rc;
    if (mac) {
        const u64* keys[CT_BATCH];
        u64* vs[CT_BATCH];
        for (u32 i = 0; i < n; i++) {
            keys[i] = d_rlk;
            vs[i] = ws.v + i * ws.v_b;
        }
        HIP_TRY(launch_ntt_lo_mac(c, level, dsrc(c, ws, 0), keys, vs, n, st));
    } else {
        HIP_TRY(launch_key_inner_multi(c, level, dsrc(c, ws, 0), d_rlk, 1, ws.v, ws.v_b, n, st));
    }
    return run_moddown(c, level, ws, n, items, st);
}

// n <= CT_BATCH products Rescale(a[b]*b[b] + addend[b]) with the relinearisation's ModDown and the rescale merged into
// one division by P*q_level: the tensor product's d0, d1 (plus the addend) enter the extended basis as P times
// themselves inside the inner-product kernel.  addend (optional): n ciphertexts [2][level+1][N], item stride
// add_bstride.  outs[b] = [2][level][N].
// lin (optional, contexts with the fused inner product only, instead of addend): the addend is ka * x + kb * y, formed on the fly.
struct LinAddend {
    const u64* const* x;
    size_t x_cstride;
    const u64* ka;
    const u64* const* y;
    size_t y_cstride;
    const u64* kb;
};
int run_ctct_merged(const ckks_ctx* c, u32 level, const u64* const* a, size_t a_cstride, const u64* const* b, size_t b_cstride,
                    const u64* addend, size_t add_bstride, const u64* d_rlk, u64* const* outs, u32 n, Arena ar, hipStream_t st,
                    const LinAddend* lin = nullptr) {
    const size_t N = c->N, L1 = level + 1;
    u64* d0 = ar.take(n * L1 * N);
    u64* d1 = ar.take(n * L1 * N);
    u64* d2 = ar.take(n * L1 * N);
    KsWs ws;
    if (!carve_ks(c, level, n, n, ar, ws)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for ct-ct multiply");
    const bool mac = ntt_has_modup(c);  // the inner product inside the forward transforms' second pass
    if (lin && (!mac || addend)) return set_err(c, CKKS_ERR_INVALID_ARG, "internal: linear addend without the fused inner product");
    if (mac && addend) return set_err(c, CKKS_ERR_INVALID_ARG, "internal: with the fused inner product the addend is given as a linear combination");
    const u64 *d2s[CT_BATCH], *add0[CT_BATCH], *add1[CT_BATCH];
    u64* vs[CT_BATCH];
    FinalItem items[CT_BATCH];
    if (mac) {
        // no tensor-product kernel either: d2 = a1 (.) b1 is formed as the inverse transform loads it, d0, d1 and the own-limb
        // term as the inner product's last terms, all from the operands themselves
        const u64 *a1[CT_BATCH], *b1[CT_BATCH], *keys[CT_BATCH];
        for (u32 i = 0; i < n; i++) {
            a1[i] = a[i] + a_cstride;
            b1[i] = b[i] + b_cstride;
            vs[i] = ws.v + i * ws.v_b;
            keys[i] = d_rlk;
            items[i] = FinalItem{nullptr, nullptr, nullptr, outs[i], 1, 0};
        }
        int rc = run_modup(c, level, a1, n, ws, st, true, b1);
        if (rc) return rc;
        MacProduct prod = {a, a1, b, b1};
        if (lin) {
            prod.lin_x = lin->x;
            prod.x_cstride = lin->x_cstride;
            prod.ka = lin->ka;
            prod.lin_y = lin->y;
            prod.y_cstride = lin->y_cstride;
            prod.kb = lin->kb;
        }
        HIP_TRY(launch_ntt_lo_mac(c, level, dsrc(c, ws, 0), keys, vs, n, st, &prod));
        return run_moddown(c, level, ws, n, items, st, true);
    }
    HIP_TRY(launch_tensor(c, level, ptr_list(a, n), a_cstride, ptr_list(b, n), b_cstride, d0, d1, d2, n, addend, add_bstride, st));
    for (u32 i = 0; i < n; i++) {
        d2s[i] = d2 + i * L1 * N;
        add0[i] = d0 + i * L1 * N;
        add1[i] = d1 + i * L1 * N;
        vs[i] = ws.v + i * ws.v_b;
        items[i] = FinalItem{nullptr, nullptr, nullptr, outs[i], 1, 0};
    }
    int rc = run_modup(c, level, d2s, n, ws, st);
    if (rc) return rc;
    HIP_TRY(launch_key_inner_ext(c, level, dsrc(c, ws, 0), d_rlk, 1, add0, add1, nullptr, vs, n, st));
    return run_moddown(c, level, ws, n, items, st, true);
}

size_t ws_poly_act(const ckks_ctx* c, u32 level, u32 n) {
    const size_t N = c->N;
    return blk(2 * (size_t)n * level * N) + 2 * blk(2 * (size_t)n * (level - 1) * N) + blk(2 * (size_t)n * (level - 2) * N) +
           blk(2 * (size_t)n * (level + 1) * N) + ws_ctct(c, level, n) + ws_rescale(c, level, n);
}

// The convolution with one division by P per output channel: every aligned copy stays on the extended
// basis Q_level P (inner product + P * sigma_g(c0), times the tap's mask), the sum over (input channel,
// tap) is taken there, and only the C_out sums go through ModDown and the rescale.  gs: Galois
// elements of the nine taps (1 = no rotation); masks [9][E][N], w_res [C_out][C_in][9][E].
// per-lane scratch of the deferred convolution: the key-switch buffers, a batch of un-rescaled outputs, the rescale's scratch
size_t ws_conv_lane(const ckks_ctx* c, u32 level) {
    return ws_ks(c, level, CT_BATCH, CT_BATCH) + blk((size_t)CT_BATCH * 2 * (level + 1) * c->N) + ws_rescale(c, level, CT_BATCH);
}
u32 conv_lanes(const ckks_ctx* c, const he_conv_desc* d) {  // two batches in flight when there is more than one
    return (c->side_stream() && (d->c_in > CT_BATCH || d->c_out > CT_BATCH)) ? 2 : 1;
}

int conv_deferred(const ckks_ctx* c, const he_conv_desc* d, const u32* gs, const uint64_t* const* h_d_in,
                  const ckks_key* const* rot_keys, const u64* masks, const u64* w_res, uint64_t* const* h_d_out, void* d_ws,
                  size_t ws_bytes, hipStream_t st0) {
    const u32 level = d->level, E = c->ext_limbs(level);
    const bool merged = d->alignment == HE_CONV_DEFERRED_MERGED;  // ModDown and rescale of the sums as one division
    const size_t N = c->N, L1 = level + 1, ct_elems = 2 * L1 * N, x_elems = 2 * (size_t)E * N;
    Arena ar(d_ws, ws_bytes);
    u64* xs = ar.take((size_t)d->c_in * 9 * x_elems);
    u64* acc = ar.take((size_t)d->c_out * x_elems);
    u64* wscratch = ar.take(weighted_sum_scratch_elems(c, E, d->c_in * 9, d->c_out));
    u64* kscratch = ar.take(key_inner_taps_scratch_elems(c, level, 8));
    // Batches of input channels (alignment) and of output channels (division) are independent: with room for two sets of
    // scratch every other batch runs on the library's side stream, between a fork and a join on the caller's stream.
    const size_t lane_bytes = ws_conv_lane(c, level);
    const u32 n_lanes = (conv_lanes(c, d) == 2 && ar.ok() && ar.used + 2 * lane_bytes <= ar.cap) ? 2 : 1;
    struct Lane {
        KsWs ws;
        u64* tmp;
        Arena rest;
        hipStream_t st;
    };
    Lane lanes[2] = {{KsWs{}, nullptr, Arena(nullptr, 0), st0}, {KsWs{}, nullptr, Arena(nullptr, 0), c->side}};
    bool ok = ar.ok();
    for (u32 l = 0; l < n_lanes && ok; l++) {
        ok = carve_ks(c, level, CT_BATCH, CT_BATCH, ar, lanes[l].ws);
        lanes[l].tmp = ar.take((size_t)CT_BATCH * ct_elems);
        u64* r = ar.take(ws_rescale(c, level, CT_BATCH) / sizeof(u64));
        lanes[l].rest = Arena(r, ws_rescale(c, level, CT_BATCH));
        ok = ok && ar.ok();
    }
    if (!ok) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the convolution");
    // the aligned copies are stored term-innermost when the fused inner product can write them that way
    const bool fused_taps = c->live_digits(level) <= 4;
    const XLayout xl = (fused_taps && N % 64 == 0) ? XLayout::tiled((size_t)d->c_in * 9, N) : XLayout::classic(E, N);
    bool forked = false;
    auto fork = [&]() -> int {
        if (n_lanes < 2 || forked) return CKKS_OK;
        HIP_TRY(hipEventRecord(c->ev_fork, st0));
        HIP_TRY(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        forked = true;
        return CKKS_OK;
    };
    auto join = [&](int rc) -> int {  // also on the error paths: the caller's stream never runs ahead of the side stream
        if (!forked) return rc;
        forked = false;
        hipError_t e = hipEventRecord(c->ev_join, c->side);
        if (e == hipSuccess) e = hipStreamWaitEvent(st0, c->ev_join, 0);
        return (e != hipSuccess && rc == CKKS_OK) ? set_hip_err(c, e) : rc;
    };
    auto align_batch = [&](u32 c0, const Lane& L) -> int {
        const KsWs& ws = L.ws;
        hipStream_t st = L.st;
        const u32 n = d->c_in - c0 < CT_BATCH ? d->c_in - c0 : CT_BATCH;
        const u64 *in[CT_BATCH], *c1s[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            in[b] = (const u64*)h_d_in[c0 + b];
            c1s[b] = in[b] + L1 * N;
        }
        int rc = run_modup(c, level, c1s, n, ws, st);
        if (rc) return rc;
        // taps without a rotation (the centre) are a product with the mask; all the others go through one launch
        const u64 *tkeys[8], *tmasks[8], *centre_mask = nullptr;
        u32 tg[8], ttap[8], n_taps = 0, centre_tap = 0, n_centre = 0;
        for (u32 t = 0; t < 9; t++) n_centre += gs[t] == 1 ? 1 : 0;
        for (u32 t = 0; t < 9; t++) {
            const u64* mask = masks + (size_t)t * E * N;
            if (gs[t] == 1) {
                if (fused_taps && n_centre == 1) {  // the tap without a rotation rides on the fused launch
                    centre_mask = mask;
                    centre_tap = t;
                } else {
                    for (u32 b = 0; b < n; b++) HIP_TRY(launch_centre_ext(c, level, mask, in[b], xs, xl, (c0 + b) * 9 + t, st));
                }
                continue;
            }
            tkeys[n_taps] = rot_keys[t]->d_key;
            tmasks[n_taps] = mask;
            tg[n_taps] = gs[t];
            ttap[n_taps++] = t;
        }
        if (fused_taps) {
            HIP_TRY(launch_key_inner_taps(c, level, dsrc(c, ws, 0), tkeys, tg, tmasks, ttap, n_taps, in, xs, xl, c0 * 9, 9, n, kscratch,
                                          c0 == 0, st, centre_mask, centre_tap));  // the masked keys are made once, by the first batch
        } else {  // many digits: one launch per tap (classic layout: every term is a [2][E][N] array)
            for (u32 i = 0; i < n_taps; i++) {
                u64* outs[CT_BATCH];
                for (u32 b = 0; b < n; b++) outs[b] = xs + ((size_t)(c0 + b) * 9 + ttap[i]) * x_elems;
                HIP_TRY(launch_key_inner_ext(c, level, dsrc(c, ws, 0), tkeys[i], tg[i], in, nullptr, tmasks[i], outs, n, st));
            }
        }
        return CKKS_OK;
    };
    int rc;
    for (u32 c0 = 0, k = 0; c0 < d->c_in; c0 += CT_BATCH, k++) {
        // the first batch also prepares the masked keys on the caller's stream; the fork comes after it
        if ((rc = align_batch(c0, lanes[k == 0 ? 0 : (n_lanes == 2 ? k & 1 : 0)]))) return join(rc);
        if (k == 0 && c0 + CT_BATCH < d->c_in && (rc = fork())) return rc;
    }
    if ((rc = join(CKKS_OK))) return rc;
    HIP_TRY(launch_weighted_sum(c, level, true, xs, xl, d->c_in * 9, w_res, d->c_out, acc, wscratch, d->weight_bits, st0));
    if (d->c_out > CT_BATCH && (rc = fork())) return rc;
    for (u32 o0 = 0, k = 0; o0 < d->c_out; o0 += CT_BATCH, k++) {
        const Lane& L = lanes[forked ? k & 1 : 0];
        const u32 n = d->c_out - o0 < CT_BATCH ? d->c_out - o0 : CT_BATCH;
        KsWs wd = L.ws;
        wd.v = acc + (size_t)o0 * x_elems;  // the sums take the place of a batch of inner products
        wd.v_b = x_elems;
        FinalItem items[CT_BATCH];
        const u64* ins[CT_BATCH];
        u64* outs[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            ins[b] = L.tmp + (size_t)b * ct_elems;
            outs[b] = (u64*)h_d_out[o0 + b];
            items[b] = FinalItem{nullptr, nullptr, nullptr, merged ? outs[b] : L.tmp + (size_t)b * ct_elems, 1, 0};
        }
        if ((rc = run_moddown(c, level, wd, n, items, L.st, merged))) return join(rc);
        if (!merged && (rc = run_rescale(c, level, ins, L1 * N, outs, n, L.rest, L.st))) return join(rc);
    }
    return join(CKKS_OK);
}

// n <= CT_BATCH different ciphertexts srcs[b] ([2][level+1][N]) rotated, outs[b] = Rot(srcs[b]) with keys[b] / gal[b]
// ([2][level+1][N], no overlap).  Neighbouring items with the same key go through one inner-product launch (the key
// streams once for all of them).
// accs (optional): outs[b] = Rot(srcs[b]) + accs[b], the sum formed by the division's last step.
int run_rotate_batch(const ckks_ctx* c, u32 level, u32 n, const u64* const* srcs, const ckks_key* const* keys, const u32* gal,
                     u64* const* outs, const KsWs& ws, hipStream_t st, const u64* const* accs = nullptr) {
    const size_t N = c->N, L1 = level + 1;
    const u64* c1s[CT_BATCH];
    FinalItem items[CT_BATCH];
    for (u32 b = 0; b < n; b++) c1s[b] = srcs[b] + L1 * N;
    int rc = run_modup(c, level, c1s, n, ws, st);
    if (rc) return rc;
    for (u32 b0 = 0; b0 < n;) {
        u32 b1 = b0 + 1;
        while (b1 < n && keys[b1] == keys[b0]) b1++;
        if (b1 - b0 == 1)
            HIP_TRY(launch_key_inner(c, level, dsrc(c, ws, b0), keys[b0]->d_key, gal[b0], ws.v + b0 * ws.v_b, st));
        else
            HIP_TRY(launch_key_inner_multi(c, level, dsrc(c, ws, b0), keys[b0]->d_key, gal[b0], ws.v + b0 * ws.v_b,
                                           ws.v_b, b1 - b0, st));
        b0 = b1;
    }
    for (u32 b = 0; b < n; b++) items[b] = FinalItem{srcs[b], nullptr, nullptr, outs[b], gal[b], 0, accs ? accs[b] : nullptr};
    return run_moddown(c, level, ws, n, items, st);
}

size_t ws_merge(const ckks_ctx* c, u32 level, u32 g) {
    const size_t N = c->N, L1 = level + 1;
    const u32 nb = g - 1 < CT_BATCH ? (g > 1 ? g - 1 : 1) : CT_BATCH;
    return ws_ks(c, level, nb, nb) + 2 * blk((size_t)g * 2 * L1 * N) + blk(2 * L1 * N) + ws_rescale(c, level, 1);
}

// out = Rescale( sum_{i<g} Rot(cts[i] (.) mask, -i*sts) ), g <= KS_MAX_BATCH; keys[i] / gal[i] for i >= 1 (validated by the caller)
int run_merge(const ckks_ctx* c, const u64* const* cts, u32 g, u32 level, const u64* mask, const ckks_key* const* keys, const u32* gal,
              u64* out, Arena ar, hipStream_t st) {
    const size_t N = c->N, L1 = level + 1, ct_elems = 2 * L1 * N;
    const u32 nb = g - 1 < CT_BATCH ? (g > 1 ? g - 1 : 1) : CT_BATCH;
    KsWs ws;
    bool ok = carve_ks(c, level, nb, nb, ar, ws);
    u64* masked = ar.take((size_t)g * ct_elems);   // C_i (.) M
    u64* rotated = ar.take((size_t)g * ct_elems);  // Rot(C_i (.) M, -i*sts), i >= 1
    u64* total = ar.take(ct_elems);
    if (!ok || !ar.ok() || ar.used + ws_rescale(c, level, 1) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the merge");
    for (u32 i = 0; i < g; i++) HIP_TRY(launch_mask_mul(c, level, mask, cts[i], masked + i * ct_elems, st));
    // blocks 1..g-1: every block has its own key; a batch shares the decomposition and ModDown launches
    for (u32 i0 = 1; i0 < g; i0 += nb) {
        const u32 n = g - i0 < nb ? g - i0 : nb;
        const u64* srcs[CT_BATCH];
        u64* outs[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            srcs[b] = masked + (i0 + b) * ct_elems;
            outs[b] = rotated + (i0 + b) * ct_elems;
        }
        int rc = run_rotate_batch(c, level, n, srcs, keys + i0, gal + i0, outs, ws, st);
        if (rc) return rc;
    }
    const u64* terms[KS_MAX_BATCH];
    terms[0] = masked;
    for (u32 i = 1; i < g; i++) terms[i] = rotated + i * ct_elems;
    HIP_TRY(launch_ct_sum(c, level, ptr_list(terms, g), g, total, st));
    const u64* in = total;
    return run_rescale(c, level, &in, L1 * N, &out, 1, ar.rest(), st);
}

// Slot re-layout with two rotations per element, for the n_ct ciphertexts of a channel vector (level `level`):
//   outs[b] = sum_h Rot( Rescale( sum_l masks[h*n_lo+l] (.) Rot(cts[b], lo_l) ), hi_h )        ([2][level][N])
// g_lo / g_hi: Galois elements (1 = no rotation, key ignored); masks: device pointers [level+1][N] or null; every h has
// at least one mask (validated by the caller).  First rotations: one decomposition per ciphertext, every key read once per
// batch of up to CT_BATCH (ciphertext, offset) pairs; second rotations batched the same way over (h, ciphertext).
size_t ws_relayout(const ckks_ctx* c, u32 level, u32 n_ct, u32 n_lo, u32 n_hi) {
    const size_t N = c->N, ctl = 2 * (size_t)(level + 1) * N, ctl1 = 2 * (size_t)level * N;
    const size_t nb = n_ct < CT_BATCH ? n_ct : CT_BATCH;
    return blk(nb * n_lo * ctl) + blk(nb * n_hi * ctl) + 2 * blk(nb * n_hi * ctl1) + ws_ks(c, level, CT_BATCH, CT_BATCH) +
           ws_rescale(c, level, CT_BATCH);
}

int run_relayout(const ckks_ctx* c, u32 level, u32 n_ct, const u64* const* cts, u32 n_lo, const ckks_key* const* lo_keys, const u32* g_lo,
                 u32 n_hi, const ckks_key* const* hi_keys, const u32* g_hi, const u64* const* masks, u64* const* outs, Arena ar,
                 hipStream_t st) {
    const size_t N = c->N, ctl = 2 * (size_t)(level + 1) * N, ctl1 = 2 * (size_t)level * N;
    const u32 nb_max = n_ct < CT_BATCH ? n_ct : CT_BATCH, l1 = level - 1;
    u64* R = ar.take((size_t)nb_max * n_lo * ctl);      // Rot(ct_b, lo_l)
    u64* Vacc = ar.take((size_t)nb_max * n_hi * ctl);   // masked sums before their rescale
    u64* V = ar.take((size_t)nb_max * n_hi * ctl1);     // level-1
    u64* Vrot = ar.take((size_t)nb_max * n_hi * ctl1);
    const size_t ks_bytes = ws_ks(c, level, CT_BATCH, CT_BATCH);
    u64* ks_region = ar.take(ks_bytes / sizeof(u64));
    if (!ar.ok() || ar.used + ws_rescale(c, level, CT_BATCH) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the re-layout");
    KsWs ws;
    auto ks_at = [&](u32 lv) {  // the key-switch buffers are carved again for the lower level
        Arena sub(ks_region, ks_bytes);
        return carve_ks(c, lv, CT_BATCH, CT_BATCH, sub, ws);
    };
    int rc;
    for (u32 c0 = 0; c0 < n_ct; c0 += CT_BATCH) {
        const u32 n = n_ct - c0 < CT_BATCH ? n_ct - c0 : CT_BATCH;
        auto r_at = [&](u32 b, u32 l) { return R + ((size_t)b * n_lo + l) * ctl; };
        // first rotations
        ks_at(level);
        const u64* c1s[CT_BATCH];
        for (u32 b = 0; b < n; b++) c1s[b] = cts[c0 + b] + (size_t)(level + 1) * N;
        if ((rc = run_modup(c, level, c1s, n, ws, st))) return rc;
        const u32 per = CT_BATCH / n;  // offsets per ModDown batch
        for (u32 la = 0; la < n_lo; la += per) {
            FinalItem items[CT_BATCH];
            u32 nk = 0;
            for (u32 l = la; l < n_lo && l < la + per; l++) {
                if (g_lo[l] == 1) {
                    for (u32 b = 0; b < n; b++) HIP_TRY(launch_copy(cts[c0 + b], r_at(b, l), ctl, st));
                    continue;
                }
                if (n == 1)
                    HIP_TRY(launch_key_inner(c, level, dsrc(c, ws, 0), lo_keys[l]->d_key, g_lo[l], ws.v + nk * ws.v_b, st));
                else
                    HIP_TRY(launch_key_inner_multi(c, level, dsrc(c, ws, 0), lo_keys[l]->d_key, g_lo[l], ws.v + nk * ws.v_b, ws.v_b, n, st));
                for (u32 b = 0; b < n; b++) items[nk++] = FinalItem{cts[c0 + b], nullptr, nullptr, r_at(b, l), g_lo[l], 0};
            }
            if (nk && (rc = run_moddown(c, level, ws, nk, items, st))) return rc;
        }
        // masked sums, one per (ciphertext, h), and their rescale
        HIP_TRY(launch_relayout_mac(c, level, false, R, masks, Vacc, n, n_lo, n_hi, st));
        const u32 n_v = n * n_hi;
        for (u32 i0 = 0; i0 < n_v; i0 += CT_BATCH) {
            const u32 m = n_v - i0 < CT_BATCH ? n_v - i0 : CT_BATCH;
            const u64* pv[CT_BATCH];
            u64* ov[CT_BATCH];
            for (u32 i = 0; i < m; i++) {
                pv[i] = Vacc + (size_t)(i0 + i) * ctl;
                ov[i] = V + (size_t)(i0 + i) * ctl1;
            }
            if ((rc = run_rescale(c, level, pv, (size_t)(level + 1) * N, ov, m, ar.rest(), st))) return rc;
        }
        // second rotations, ordered by h so that the ciphertexts of a batch share each key
        ks_at(l1);
        const u64* srcs[CT_BATCH];
        const ckks_key* ks[CT_BATCH];
        u32 gs[CT_BATCH], nk = 0;
        u64* dsts[CT_BATCH];
        for (u32 h = 0; h < n_hi; h++) {
            if (g_hi[h] == 1) continue;
            for (u32 b = 0; b < n; b++) {
                srcs[nk] = V + ((size_t)b * n_hi + h) * ctl1;
                dsts[nk] = Vrot + ((size_t)b * n_hi + h) * ctl1;
                ks[nk] = hi_keys[h];
                gs[nk++] = g_hi[h];
                if (nk == CT_BATCH) {
                    if ((rc = run_rotate_batch(c, l1, nk, srcs, ks, gs, dsts, ws, st))) return rc;
                    nk = 0;
                }
            }
        }
        if (nk && (rc = run_rotate_batch(c, l1, nk, srcs, ks, gs, dsts, ws, st))) return rc;
        // the sums; the running sum is one of the terms of every launch after the first
        for (u32 b = 0; b < n; b++) {
            u64* out = outs[c0 + b];
            for (u32 h = 0; h < n_hi;) {
                const u64* terms[KS_MAX_BATCH];
                u32 nt = 0;
                if (h) terms[nt++] = out;
                for (; h < n_hi && nt < KS_MAX_BATCH; h++) terms[nt++] = (g_hi[h] == 1 ? V : Vrot) + ((size_t)b * n_hi + h) * ctl1;
                HIP_TRY(launch_ct_sum(c, l1, ptr_list(terms, nt), nt, out, st));
            }
        }
    }
    return CKKS_OK;
}

// The same re-layout with the divisions by P deferred past the sums (masks on the extended basis, [level+1+k][N]):
//   X_l = (P sigma(c0) + v0, v1) for the first rotations (inner products only), V_h = (sum_l M[h][l] (.) X_l) / (P q_level),
//   out = ModDown( sum_h X'_h ) with X'_h the pre-division copy of Rot(V_h, hi_h).
size_t ws_relayout_deferred(const ckks_ctx* c, u32 level, u32 n_ct, u32 n_lo, u32 n_hi) {
    const size_t N = c->N, xel = 2 * (size_t)c->ext_limbs(level) * N, xel1 = 2 * (size_t)c->ext_limbs(level - 1) * N, ctl1 = 2 * (size_t)level * N;
    const size_t nb = n_ct < CT_BATCH ? n_ct : CT_BATCH;
    return blk(nb * n_lo * xel) + blk(nb * n_hi * xel) + blk(nb * n_hi * ctl1) + blk(nb * n_hi * xel1) + blk(nb * xel1) +
           ws_ks(c, level, CT_BATCH, CT_BATCH);
}

int run_relayout_deferred(const ckks_ctx* c, u32 level, u32 n_ct, const u64* const* cts, u32 n_lo, const ckks_key* const* lo_keys,
                          const u32* g_lo, u32 n_hi, const ckks_key* const* hi_keys, const u32* g_hi, const u64* const* masks,
                          u64* const* outs, Arena ar, hipStream_t st) {
    const u32 l1 = level - 1, nb_max = n_ct < CT_BATCH ? n_ct : CT_BATCH;
    const size_t N = c->N, xel = 2 * (size_t)c->ext_limbs(level) * N, xel1 = 2 * (size_t)c->ext_limbs(l1) * N, ctl1 = 2 * (size_t)level * N;
    u64* X = ar.take((size_t)nb_max * n_lo * xel);     // first rotations before their division
    u64* Vacc = ar.take((size_t)nb_max * n_hi * xel);  // masked sums on the extended basis
    u64* V = ar.take((size_t)nb_max * n_hi * ctl1);    // divided by P q_level: level-1
    u64* Xh = ar.take((size_t)nb_max * n_hi * xel1);   // second rotations before their division
    u64* W = ar.take((size_t)nb_max * xel1);           // their sums
    KsWs ws;
    const size_t ks_bytes = ws_ks(c, level, CT_BATCH, CT_BATCH);
    u64* ks_region = ar.take(ks_bytes / sizeof(u64));
    // Up to eight first rotations of a batch of ciphertexts in one launch (the digits are read once for the eight, not once
    // per rotation): the keyed offsets in groups of eight.
    const bool fused_lo = c->live_digits(level) <= 4;
    std::vector<u32> keyed;
    for (u32 l = 0; l < n_lo; l++)
        if (g_lo[l] != 1) keyed.push_back(l);
    const u32 n_groups = fused_lo ? (u32)((keyed.size() + 7) / 8) : 0;
    if (!ar.ok()) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the re-layout");
    auto ks_at = [&](u32 lv) {
        Arena sub(ks_region, ks_bytes);
        return carve_ks(c, lv, CT_BATCH, CT_BATCH, sub, ws);
    };
    int rc;
    for (u32 c0 = 0; c0 < n_ct; c0 += CT_BATCH) {
        const u32 n = n_ct - c0 < CT_BATCH ? n_ct - c0 : CT_BATCH;
        ks_at(level);
        const u64 *in[CT_BATCH], *c1s[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            in[b] = cts[c0 + b];
            c1s[b] = in[b] + (size_t)(level + 1) * N;
        }
        if ((rc = run_modup(c, level, c1s, n, ws, st))) return rc;
        for (u32 l = 0; l < n_lo; l++) {
            u64* xo[CT_BATCH];
            for (u32 b = 0; b < n; b++) xo[b] = X + ((size_t)b * n_lo + l) * xel;
            if (g_lo[l] == 1) {
                for (u32 b = 0; b < n; b++) HIP_TRY(launch_scale_p_ext(c, level, in[b], xo[b], st));
            } else if (!fused_lo) {
                HIP_TRY(launch_key_inner_ext(c, level, dsrc(c, ws, 0), lo_keys[l]->d_key, g_lo[l], in, nullptr, nullptr, xo, n, st));
            }
        }
        for (u32 g = 0; g < n_groups; g++) {  // X[b][l] = term b * n_lo + l of a [2][E][N] array per term
            const u64* tkeys[8];
            u32 tg[8], ttap[8], nt = 0;
            for (size_t i = (size_t)g * 8; i < keyed.size() && nt < 8; i++) {
                const u32 l = keyed[i];
                tkeys[nt] = lo_keys[l]->d_key;
                tg[nt] = g_lo[l];
                ttap[nt++] = l;
            }
            HIP_TRY(launch_key_inner_taps(c, level, dsrc(c, ws, 0), tkeys, tg, nullptr, ttap, nt, in, X, XLayout::classic(c->ext_limbs(level), N), 0,
                                          n_lo, n, nullptr, false, st, nullptr, 0, true));
        }
        HIP_TRY(launch_relayout_mac(c, level, true, X, masks, Vacc, n, n_lo, n_hi, st));
        const u32 n_v = n * n_hi;
        for (u32 i0 = 0; i0 < n_v; i0 += CT_BATCH) {  // one division by P q_level per sum
            const u32 m = n_v - i0 < CT_BATCH ? n_v - i0 : CT_BATCH;
            KsWs wd = ws;
            wd.v = Vacc + (size_t)i0 * xel;
            wd.v_b = xel;
            FinalItem items[CT_BATCH];
            for (u32 i = 0; i < m; i++) items[i] = FinalItem{nullptr, nullptr, nullptr, V + (size_t)(i0 + i) * ctl1, 1, 0};
            if ((rc = run_moddown(c, level, wd, m, items, st, true))) return rc;
        }
        // second rotations on the extended basis of level-1, ordered by h so that the ciphertexts of a batch share each key
        ks_at(l1);
        const u64 *src[CT_BATCH], *sc1[CT_BATCH];
        const ckks_key* ks[CT_BATCH];
        u32 gs[CT_BATCH], nk = 0;
        u64* dst[CT_BATCH];
        auto flush = [&]() -> int {
            int r = run_modup(c, l1, sc1, nk, ws, st);
            if (r) return r;
            for (u32 b0 = 0; b0 < nk;) {
                u32 b1 = b0 + 1;
                while (b1 < nk && ks[b1] == ks[b0]) b1++;
                HIP_TRY(launch_key_inner_ext(c, l1, dsrc(c, ws, b0), ks[b0]->d_key, gs[b0], src + b0, nullptr, nullptr,
                                             dst + b0, b1 - b0, st));
                b0 = b1;
            }
            nk = 0;
            return CKKS_OK;
        };
        for (u32 h = 0; h < n_hi; h++)
            for (u32 b = 0; b < n; b++) {
                const u64* v = V + ((size_t)b * n_hi + h) * ctl1;
                u64* xh = Xh + ((size_t)b * n_hi + h) * xel1;
                if (g_hi[h] == 1) {
                    HIP_TRY(launch_scale_p_ext(c, l1, v, xh, st));
                    continue;
                }
                src[nk] = v;
                sc1[nk] = v + (size_t)level * N;
                dst[nk] = xh;
                ks[nk] = hi_keys[h];
                gs[nk++] = g_hi[h];
                if (nk == CT_BATCH && (rc = flush())) return rc;
            }
        if (nk && (rc = flush())) return rc;
        // sums on the extended basis, then one ModDown per ciphertext
        for (u32 b = 0; b < n; b++) {
            u64* w = W + (size_t)b * xel1;
            for (u32 h = 0; h < n_hi;) {
                const u64* terms[KS_MAX_BATCH];
                u32 nt = 0;
                if (h) terms[nt++] = w;
                for (; h < n_hi && nt < KS_MAX_BATCH; h++) terms[nt++] = Xh + ((size_t)b * n_hi + h) * xel1;
                HIP_TRY(launch_ct_sum(c, l1, ptr_list(terms, nt), nt, w, st, true));
            }
        }
        KsWs wd = ws;
        wd.v = W;
        wd.v_b = xel1;
        FinalItem items[CT_BATCH];
        for (u32 b = 0; b < n; b++) items[b] = FinalItem{nullptr, nullptr, nullptr, outs[c0 + b], 1, 0};
        if ((rc = run_moddown(c, l1, wd, n, items, st))) return rc;
    }
    return CKKS_OK;
}

u32 ilog2(u32 v) { u32 r = 0; while ((1u << (r + 1)) <= v) r++; return r; }

}  // namespace

extern "C" {

size_t ckks_workspace_bytes(const ckks_ctx* c, int op, uint32_t level, uint32_t count) {
    if (!c || !level_ok(c, level)) return 0;
    const size_t N = c->N, L1 = level + 1;
    const u32 nb = count < 1 ? 1 : (count > CT_BATCH ? CT_BATCH : count);
    switch (op) {
        case CKKS_OP_KEYSWITCH: return c->dnum ? ws_ks(c, level, 1, 1) : 0;
        case CKKS_OP_ROTATE: {
            if (!c->dnum) return 0;
            // hoisted, more than one batch: a second set of inner-product and conversion buffers (two batches in flight);
            // unhoisted: every rotation of a batch has its own permuted copy and its own digits
            const size_t hoisted = ws_ks(c, level, 1, nb) + blk(L1 * N) +
                                   (count > CT_BATCH && c->side ? blk((size_t)nb * 2 * c->ext_limbs(level) * N) + blk((size_t)nb * 2 * L1 * N) : 0);
            const size_t unhoisted = ws_ks(c, level, nb, nb) + blk((size_t)nb * L1 * N);
            return hoisted > unhoisted ? hoisted : unhoisted;
        }
        case CKKS_OP_RESCALE: return level >= 1 ? ws_rescale(c, level, 1) : 0;
        case CKKS_OP_CTCT_MUL_RELIN: return c->dnum ? ws_ctct(c, level, 1) : 0;
        // more than one batch of channels: two batches in flight (one on the library's side stream), each with its own scratch
        case CKKS_OP_POLY_ACT: return (c->dnum && level >= 4) ? ws_poly_act(c, level, nb) * (count > CT_BATCH && c->side ? 2 : 1) : 0;  // sized for overlap on
        default: return 0;
    }
}

size_t he_conv_workspace_bytes(const ckks_ctx* c, const he_conv_desc* d) {
    if (!c || !d || !c->dnum || !level_ok(c, d->level) || d->level < 1) return 0;
    const size_t N = c->N, L1 = d->level + 1;
    if (d->alignment == HE_CONV_DEFERRED_MODDOWN || d->alignment == HE_CONV_DEFERRED_MERGED) {
        const size_t E = c->ext_limbs(d->level);
        const u32 lanes = (c->side && (d->c_in > CT_BATCH || d->c_out > CT_BATCH)) ? 2 : 1;  // sized for overlap on
        return lanes * ws_conv_lane(c, d->level) + blk((size_t)d->c_in * 9 * 2 * E * N) + blk((size_t)d->c_out * 2 * E * N) +
               blk(weighted_sum_scratch_elems(c, (u32)E, d->c_in * 9, d->c_out)) + blk(key_inner_taps_scratch_elems(c, d->level, 8));
    }
    return ws_ks(c, d->level, CT_BATCH, CT_BATCH) + blk((size_t)d->c_in * 9 * 2 * L1 * N) + blk((size_t)d->c_out * 2 * L1 * N) +
           blk(weighted_sum_scratch_elems(c, (u32)L1, d->c_in * 9, d->c_out)) + ws_rescale(c, d->level, CT_BATCH) +
           (d->alignment == HE_CONV_ALIGN_FOUR_KEYS ? 2 * blk((size_t)CT_BATCH * 2 * L1 * N) : 0);
}

int ckks_ctx_set_overlap(ckks_ctx* c, int on) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    c->overlap = on != 0;
    return CKKS_OK;
}

uint32_t ckks_galois_element(const ckks_ctx* c, int32_t offset) {
    if (!c) return 0;
    const long n = (long)(c->N / 2);
    long r = offset % n;
    if (r < 0) r += n;
    const u64 two_n = 2ull * c->N;
    u64 g = 1, base = 5;
    for (; r; r >>= 1) {
        if (r & 1) g = g * base % two_n;
        base = base * base % two_n;
    }
    return (uint32_t)g;
}

static int ntt_entry(const ckks_ctx* c, bool inverse, uint64_t* d_polys, const uint32_t* h_idx, uint32_t n_limbs, uint32_t batch,
                     void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_polys || !h_idx || n_limbs == 0 || batch == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or empty batch");
    if (n_limbs > CKKS_MAX_MODULI) return set_err(c, CKKS_ERR_INVALID_ARG, "at most 64 limbs per polynomial");
    PolyList pl;
    pl.n = n_limbs;
    for (u32 a = 0; a < CKKS_MAX_MODULI; a++) {
        if (a < n_limbs && h_idx[a] >= c->M) return set_err(c, CKKS_ERR_INVALID_ARG, "modulus index out of range");
        pl.spos[a] = pl.dpos[a] = (unsigned char)(a < n_limbs ? a : 0);
        pl.mod[a] = (unsigned char)(a < n_limbs ? h_idx[a] : 0);
    }
    const u32 max_batch = 65535 / n_limbs;  // grid.y limit
    u64* p = (u64*)d_polys;
    for (u32 b0 = 0; b0 < batch; b0 += max_batch) {
        const u32 nb = batch - b0 < max_batch ? batch - b0 : max_batch;
        u64* base = p + (size_t)b0 * n_limbs * c->N;
        HIP_TRY(launch_ntt(c, inverse, base, n_limbs, base, n_limbs, pl, nb, (hipStream_t)stream));
    }
    return CKKS_OK;
}

int ckks_ntt_fwd(const ckks_ctx* c, uint64_t* d_polys, const uint32_t* h_idx, uint32_t n_limbs, uint32_t batch, void* stream) {
    return ntt_entry(c, false, d_polys, h_idx, n_limbs, batch, stream);
}
int ckks_ntt_inv(const ckks_ctx* c, uint64_t* d_polys, const uint32_t* h_idx, uint32_t n_limbs, uint32_t batch, void* stream) {
    return ntt_entry(c, true, d_polys, h_idx, n_limbs, batch, stream);
}

int ckks_key_load(const ckks_ctx* c, const uint64_t* d_key, uint32_t galois_elt, ckks_key** out) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_key || !out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (galois_elt != 0 && ((galois_elt & 1) == 0 || galois_elt >= 2 * c->N)) return set_err(c, CKKS_ERR_INVALID_ARG, "Galois element must be odd and below 2N");
    ckks_key* k = new (std::nothrow) ckks_key;
    if (!k) return set_err(c, CKKS_ERR_INVALID_ARG, "out of host memory");
    k->d_key = (const u64*)d_key;
    k->galois_elt = galois_elt;
    *out = k;
    return CKKS_OK;
}
void ckks_key_free(ckks_key* k) { delete k; }

int ckks_key_expand_a(const ckks_ctx* c, uint64_t a_seed, uint64_t* d_key, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_key) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    HIP_TRY(launch_key_expand_a(c, a_seed, (u64*)d_key, (hipStream_t)stream));
    return CKKS_OK;
}

int ckks_keyset_stage(const ckks_ctx* c, const uint64_t* const* h_b, const uint64_t* h_a_seeds, uint64_t* const* h_d_keys,
                      uint32_t n_keys, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!h_b || !h_a_seeds || !h_d_keys) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    for (u32 i = 0; i < n_keys; i++)
        if (!h_b[i] || !h_d_keys[i]) return set_err(c, CKKS_ERR_INVALID_ARG, "null key pointer");
    const size_t half = (size_t)c->M * c->N * sizeof(u64);  // one digit's b (or a) part
    hipStream_t st = (hipStream_t)stream;
    for (u32 i = 0; i < n_keys; i++) {
        // the b halves: dnum rows of `half` bytes, densely packed on the host, every other row of the device key
        HIP_TRY(hipMemcpy2DAsync(h_d_keys[i], 2 * half, h_b[i], half, half, c->dnum, hipMemcpyHostToDevice, st));
        HIP_TRY(launch_key_expand_a(c, h_a_seeds[i], (u64*)h_d_keys[i], st));
    }
    return CKKS_OK;
}

int ckks_keyswitch(const ckks_ctx* c, const uint64_t* d_c, uint32_t level, const ckks_key* key, uint64_t* d_out, void* d_ws,
                   size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_c || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!key) return set_err(c, CKKS_ERR_NO_KEY, "no key");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    Arena ar(d_ws, ws_bytes);
    KsWs ws;
    if (!carve_ks(c, level, 1, 1, ar, ws)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for key switch");
    hipStream_t st = (hipStream_t)stream;
    const u64* src = (const u64*)d_c;
    const bool mac = ntt_has_modup(c);
    int rc = run_modup(c, level, &src, 1, ws, st, mac);
    if (rc) return rc;
    if (mac) {
        const u64* k = key->d_key;
        HIP_TRY(launch_ntt_lo_mac(c, level, dsrc(c, ws, 0), &k, &ws.v, 1, st));
    } else {
        HIP_TRY(launch_key_inner(c, level, dsrc(c, ws, 0), key->d_key, 1, ws.v, st));
    }
    const FinalItem item = {nullptr, nullptr, nullptr, (u64*)d_out, 1, 0};
    return run_moddown(c, level, ws, 1, &item, st);
}

int ckks_rotate_hoisted(const ckks_ctx* c, const uint64_t* d_ct, uint32_t level, const int32_t* h_offsets, uint32_t n_rot,
                        const ckks_key* const* keys, uint64_t* const* h_d_outs, int hoisted, void* d_ws, size_t ws_bytes,
                        void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_ct || !h_offsets || !h_d_outs || n_rot == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or no rotations");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    const size_t N = c->N, L1 = level + 1;
    // validate everything before the first launch
    u32 n_keyed = 0;
    for (u32 t = 0; t < n_rot; t++) {
        if (!h_d_outs[t]) return set_err(c, CKKS_ERR_INVALID_ARG, "null output pointer");
        const u32 g = ckks_galois_element(c, h_offsets[t]);
        if (g == 1) continue;
        n_keyed++;
        if (!keys || !keys[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key missing");
        if (keys[t]->galois_elt != g) return set_err(c, CKKS_ERR_NO_KEY, "rotation key was made for another offset");
    }
    // rotations go through the kernels in batches of up to CT_BATCH: hoisted ones share the digits and batch their ModDown;
    // unhoisted ones each have their own permuted polynomial and digits and batch everything but the inner product (one key
    // each), in batches as large as the workspace holds (one at a time in the smallest workspace that is accepted)
    u32 rb = n_keyed < CT_BATCH ? (n_keyed ? n_keyed : 1) : CT_BATCH;
    Arena ar(d_ws, ws_bytes);
    KsWs ws = {};
    u64* pc1 = nullptr;
    if (n_keyed) {
        if (hoisted) {
            if (!carve_ks(c, level, 1, rb, ar, ws)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rotation");
        } else {
            for (;; rb--) {
                Arena probe(d_ws, ws_bytes);
                KsWs w;
                const bool fits = carve_ks(c, level, rb, rb, probe, w) && (probe.take((size_t)rb * L1 * N), probe.ok());
                if (fits) break;
                if (rb == 1) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rotation");
            }
            carve_ks(c, level, rb, rb, ar, ws);
            pc1 = ar.take((size_t)rb * L1 * N);
        }
    }
    hipStream_t st = (hipStream_t)stream;
    // More than one batch of hoisted rotations: with room for a second set of inner-product and conversion buffers, every
    // other batch runs on the context's second stream (its traffic-bound inner products next to the other batch's ModDown).
    KsWs lane_ws[2] = {ws, ws};
    bool two_lanes = false;
    if (hoisted && n_keyed > rb && c->side_stream()) {
        Arena extra = ar;
        lane_ws[1].v = extra.take(rb * ws.v_b);
        lane_ws[1].w = extra.take(rb * ws.w_b);
        two_lanes = extra.ok();
    }
    const u64* ct = (const u64*)d_ct;
    const u64* c0 = ct;
    const u64* c1 = ct + L1 * N;
    if (n_keyed && hoisted) {
        int rc = run_modup(c, level, &c1, 1, ws, st);
        if (rc) return rc;
        for (u32 l = 0; l < 2; l++) lane_ws[l].own[0] = ws.own[0];  // both lanes read the same digits
    }
    if (two_lanes) {
        HIP_TRY(hipEventRecord(c->ev_fork, st));
        HIP_TRY(hipStreamWaitEvent(c->side, c->ev_fork, 0));
    }
    auto join = [&](int rc) -> int {  // also on the error paths
        if (!two_lanes) return rc;
        hipError_t e = hipEventRecord(c->ev_join, c->side);
        if (e == hipSuccess) e = hipStreamWaitEvent(st, c->ev_join, 0);
        return (e != hipSuccess && rc == CKKS_OK) ? set_hip_err(c, e) : rc;
    };
    FinalItem items[CT_BATCH];
    const ckks_key* pend_key[CT_BATCH];
    u32 nb = 0, lane = 0;
    // the pending unhoisted rotations: sigma_g(c1) of each, one decomposition and one ModDown for the batch
    auto flush_unhoisted = [&]() -> int {
        const u64* srcs[CT_BATCH];
        for (u32 b = 0; b < nb; b++) {
            u64* dst = pc1 + (size_t)b * L1 * N;
            HIP_TRY(launch_automorph(c, (u32)L1, c1, items[b].g, dst, st));
            srcs[b] = dst;
        }
        const bool mac = ntt_has_modup(c);
        int rc = run_modup(c, level, srcs, nb, ws, st, mac);
        if (rc) return rc;
        // the digits already belong to sigma_g(c1): no gather in the inner product, only on c0
        if (mac) {  // every item with its own key, inside the forward transforms' second pass
            const u64* ks[CT_BATCH];
            u64* vs[CT_BATCH];
            for (u32 b = 0; b < nb; b++) {
                ks[b] = pend_key[b]->d_key;
                vs[b] = ws.v + b * ws.v_b;
            }
            HIP_TRY(launch_ntt_lo_mac(c, level, dsrc(c, ws, 0), ks, vs, nb, st));
        } else {
            for (u32 b = 0; b < nb; b++) HIP_TRY(launch_key_inner(c, level, dsrc(c, ws, b), pend_key[b]->d_key, 1, ws.v + b * ws.v_b, st));
        }
        rc = run_moddown(c, level, ws, nb, items, st);
        nb = 0;
        return rc;
    };
    const bool fused_hoist = hoisted && c->live_digits(level) <= 4;
    auto flush_hoisted = [&]() -> int {
        const KsWs& lw = lane_ws[lane];
        hipStream_t ls = lane ? c->side : st;
        const u64* tkeys[8];
        u32 tg[8], ttap[8];
        for (u32 b = 0; b < nb; b++) {
            tkeys[b] = pend_key[b]->d_key;
            tg[b] = items[b].g;
            ttap[b] = b;
            items[b].g = 1;  // the division's last step adds nothing: c0 is inside the sum already
        }
        if (hipError_t e = launch_key_inner_taps(c, level, dsrc(c, lw, 0), tkeys, tg, nullptr, ttap, nb, &ct, lw.v,
                                                 XLayout::classic(c->ext_limbs(level), N), 0, 0, 1, nullptr, false, ls, nullptr, 0, true);
            e != hipSuccess)
            return set_hip_err(c, e);
        int rc = run_moddown(c, level, lw, nb, items, ls);
        nb = 0;
        if (two_lanes) lane ^= 1;
        return rc;
    };
    for (u32 t = 0; t < n_rot; t++) {
        const u32 g = ckks_galois_element(c, h_offsets[t]);
        u64* out = (u64*)h_d_outs[t];
        if (g == 1) {
            if (hipError_t e = launch_copy(ct, out, 2 * L1 * N, st); e != hipSuccess) return join(set_hip_err(c, e));
            continue;
        }
        if (hoisted && fused_hoist) {
            // same digits, one key per rotation: the rotations of a batch share one launch that reads the digits once and
            // leaves P sigma_g(c0) + inner product on the extended basis (its ModDown is the rotation, c0 included)
            pend_key[nb] = keys[t];
            items[nb] = FinalItem{nullptr, nullptr, nullptr, out, g, 0};
            if (++nb == rb) {
                if (int rc = flush_hoisted()) return join(rc);
            }
        } else if (hoisted) {
            // many digits: one launch per rotation; the digits are read through sigma_g
            const KsWs& lw = lane_ws[lane];
            hipStream_t ls = lane ? c->side : st;
            if (hipError_t e = launch_key_inner(c, level, dsrc(c, lw, 0), keys[t]->d_key, g, lw.v + nb * lw.v_b, ls); e != hipSuccess)
                return join(set_hip_err(c, e));
            items[nb] = FinalItem{c0, nullptr, nullptr, out, g, 0};
            if (++nb == rb) {
                int rc = run_moddown(c, level, lw, nb, items, ls);
                if (rc) return join(rc);
                nb = 0;
                if (two_lanes) lane ^= 1;
            }
        } else {
            items[nb] = FinalItem{c0, nullptr, nullptr, out, g, 0};
            pend_key[nb] = keys[t];
            if (++nb == rb)
                if (int rc = flush_unhoisted()) return rc;
        }
    }
    if (nb && !hoisted) {
        if (int rc = flush_unhoisted()) return rc;
    } else if (nb && fused_hoist) {
        if (int rc = flush_hoisted()) return join(rc);
    } else if (nb) {
        int rc = run_moddown(c, level, lane_ws[lane], nb, items, lane ? c->side : st);
        if (rc) return join(rc);
    }
    return join(CKKS_OK);
}

int ckks_ptct_mac(const ckks_ctx* c, const uint64_t* const* h_d_pts, const uint64_t* const* h_d_cts, uint32_t n_terms,
                  uint32_t level, uint64_t* d_acc, int accumulate, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!h_d_pts || !h_d_cts || !d_acc || n_terms == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or no terms");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    for (u32 k = 0; k < n_terms; k++)
        if (!h_d_pts[k] || !h_d_cts[k]) return set_err(c, CKKS_ERR_INVALID_ARG, "null operand pointer");
    HIP_TRY(launch_ptct_mac(c, level, (const u64* const*)h_d_pts, (const u64* const*)h_d_cts, n_terms, (u64*)d_acc, accumulate,
                            (hipStream_t)stream));
    return CKKS_OK;
}

int ckks_rescale(const ckks_ctx* c, const uint64_t* d_ct, uint32_t level, uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_ct || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!level_ok(c, level) || level < 1) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "rescale needs 1 <= level < num_q");
    const u64* ct = (const u64*)d_ct;
    u64* out = (u64*)d_out;
    return run_rescale(c, level, &ct, (size_t)(level + 1) * c->N, &out, 1, Arena(d_ws, ws_bytes), (hipStream_t)stream);
}

int ckks_ctct_mul_relin(const ckks_ctx* c, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, const ckks_key* rlk,
                        uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_a || !d_b || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!rlk) return set_err(c, CKKS_ERR_NO_KEY, "no relinearisation key");
    if (rlk->galois_elt != 0) return set_err(c, CKKS_ERR_NO_KEY, "key is a rotation key, not the relinearisation key");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    const size_t cs = (size_t)(level + 1) * c->N;
    const u64* a = (const u64*)d_a;
    const u64* b = (const u64*)d_b;
    u64* out = (u64*)d_out;
    return run_ctct(c, level, &a, cs, &b, cs, rlk->d_key, &out, 1, Arena(d_ws, ws_bytes), (hipStream_t)stream);
}

int he_conv_check_weights(const ckks_ctx* c, const he_conv_desc* d, const uint64_t* d_w_res, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d || !d_w_res) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (d->c_in == 0 || d->c_out == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "empty convolution shape");
    if (!level_ok(c, d->level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    if (d->alignment > HE_CONV_DEFERRED_MERGED) return set_err(c, CKKS_ERR_INVALID_ARG, "unknown alignment");
    if (d->weight_bits == 0) return CKKS_OK;  // nothing promised
    const bool ext = d->alignment == HE_CONV_DEFERRED_MODDOWN || d->alignment == HE_CONV_DEFERRED_MERGED;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(launch_weight_check(c, d->level, ext, (const u64*)d_w_res, (size_t)d->c_out * d->c_in * 9, d->weight_bits, c->d_check, st));
    u32 bad = 0;
    HIP_TRY(hipMemcpyAsync(&bad, c->d_check, sizeof(bad), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (bad) {
        c->err = std::to_string(bad) + " weight residues are not integers below 2^(weight_bits-1) = 2^" + std::to_string(d->weight_bits - 1) +
                 " in magnitude: he_conv_batched would return wrong residues with this weight_bits";
        return CKKS_ERR_INVALID_ARG;
    }
    return CKKS_OK;
}

int he_conv_batched(const ckks_ctx* c, const he_conv_desc* d, const uint64_t* const* h_d_in, const ckks_key* const* rot_keys,
                    const uint64_t* d_tap_masks, const uint64_t* d_w_res, uint64_t* const* h_d_out, void* d_ws, size_t ws_bytes,
                    void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d || !h_d_in || !rot_keys || !d_tap_masks || !d_w_res || !h_d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (d->c_in == 0 || d->c_out == 0 || d->height == 0 || d->width == 0 || d->batch == 0)
        return set_err(c, CKKS_ERR_INVALID_ARG, "empty convolution shape");
    if (!level_ok(c, d->level) || d->level < 1) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "convolution needs 1 <= level < num_q");
    if ((u64)d->height * d->width * d->batch > c->N / 2) return set_err(c, CKKS_ERR_INVALID_ARG, "H*W*batch exceeds the N/2 slots");
    if (d->alignment > HE_CONV_DEFERRED_MERGED) return set_err(c, CKKS_ERR_INVALID_ARG, "unknown alignment");
    const bool four = d->alignment == HE_CONV_ALIGN_FOUR_KEYS;
    const u32 level = d->level;
    const size_t N = c->N, L1 = level + 1, ct_elems = 2 * L1 * N;
    u32 gs[9];
    {
        u32 t = 0;
        for (int dy = -1; dy <= 1; dy++)
            for (int dx = -1; dx <= 1; dx++, t++) {
                gs[t] = ckks_galois_element(c, dy * (int32_t)d->width + dx);
                if (gs[t] == 1) continue;
                if (four && (t & 1) == 0) continue;  // the corner taps are reached in two steps: no key of their own
                if (!rot_keys[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key missing for a tap");
                if (rot_keys[t]->galois_elt != gs[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key does not match its tap offset");
            }
    }
    for (u32 i = 0; i < d->c_in; i++) if (!h_d_in[i]) return set_err(c, CKKS_ERR_INVALID_ARG, "null input ciphertext");
    for (u32 o = 0; o < d->c_out; o++) if (!h_d_out[o]) return set_err(c, CKKS_ERR_INVALID_ARG, "null output ciphertext");

    if (d->alignment == HE_CONV_DEFERRED_MODDOWN || d->alignment == HE_CONV_DEFERRED_MERGED)
        return conv_deferred(c, d, gs, h_d_in, rot_keys, (const u64*)d_tap_masks, (const u64*)d_w_res, h_d_out, d_ws, ws_bytes,
                             (hipStream_t)stream);
    Arena ar(d_ws, ws_bytes);
    KsWs ws;
    bool ok = carve_ks(c, level, CT_BATCH, CT_BATCH, ar, ws);
    u64* xs = ar.take((size_t)d->c_in * 9 * ct_elems);
    u64* acc = ar.take((size_t)d->c_out * ct_elems);
    u64* wscratch = ar.take(weighted_sum_scratch_elems(c, (u32)L1, d->c_in * 9, d->c_out));
    u64* side[2] = {nullptr, nullptr};  // C^-1 and C^+1 of the current batch (four-key alignment)
    if (four) {
        side[0] = ar.take((size_t)CT_BATCH * ct_elems);
        side[1] = ar.take((size_t)CT_BATCH * ct_elems);
    }
    if (!ok || !ar.ok() || ar.used + ws_rescale(c, level, CT_BATCH) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the convolution");
    hipStream_t st = (hipStream_t)stream;

    // input alignment: nine aligned copies of every input channel, each times its tap mask.  Channels
    // go in batches: one shared pass of the decomposition kernels, then per tap one inner product that
    // streams the tap's key once for the whole batch and one batched ModDown.
    auto mask_of = [&](u32 t) { return (const u64*)d_tap_masks + (size_t)t * L1 * N; };
    auto slot = [&](u32 ch, u32 t) { return xs + ((size_t)ch * 9 + t) * ct_elems; };
    // rotate the batch `base` (digits already in ws) by the offset of tap `kt`; outs[b] gets mask `m`
    auto rotate_batch = [&](const u64* const* base, u32 n, u32 kt, u64* const* outs, const u64* m) -> int {
        HIP_TRY(launch_key_inner_multi(c, level, dsrc(c, ws, 0), rot_keys[kt]->d_key, gs[kt], ws.v, ws.v_b, n, st));
        FinalItem items[CT_BATCH];
        for (u32 b = 0; b < n; b++) items[b] = FinalItem{base[b], nullptr, m, outs[b], gs[kt], 0};
        return run_moddown(c, level, ws, n, items, st);
    };
    for (u32 c0 = 0; c0 < d->c_in; c0 += CT_BATCH) {
        const u32 n = d->c_in - c0 < CT_BATCH ? d->c_in - c0 : CT_BATCH;
        const u64 *in[CT_BATCH], *c1s[CT_BATCH];
        u64* outs[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            in[b] = (const u64*)h_d_in[c0 + b];
            c1s[b] = in[b] + L1 * N;
        }
        int rc = run_modup(c, level, c1s, n, ws, st);
        if (rc) return rc;
        if (!four) {
            for (u32 t = 0; t < 9; t++) {
                if (gs[t] == 1) {
                    for (u32 b = 0; b < n; b++) HIP_TRY(launch_mask_mul(c, level, mask_of(t), in[b], slot(c0 + b, t), st));
                    continue;
                }
                for (u32 b = 0; b < n; b++) outs[b] = slot(c0 + b, t);
                if ((rc = rotate_batch(in, n, t, outs, mask_of(t)))) return rc;
            }
            continue;
        }
        // four-key alignment, first stage: the input rotated by -1, +1 (kept unmasked for the second
        // stage) and by -W, +W (final), all from the one decomposition of the input
        for (u32 sd = 0; sd < 2; sd++) {
            const u32 kt = sd == 0 ? 3 : 5;
            for (u32 b = 0; b < n; b++) outs[b] = side[sd] + (size_t)b * ct_elems;
            if (gs[kt] == 1) {
                for (u32 b = 0; b < n; b++) HIP_TRY(launch_copy(in[b], outs[b], ct_elems, st));
            } else if ((rc = rotate_batch(in, n, kt, outs, nullptr))) return rc;
        }
        for (u32 kt = 1; kt <= 7; kt += 6) {
            for (u32 b = 0; b < n; b++) outs[b] = slot(c0 + b, kt);
            if (gs[kt] == 1) {
                for (u32 b = 0; b < n; b++) HIP_TRY(launch_mask_mul(c, level, mask_of(kt), in[b], outs[b], st));
            } else if ((rc = rotate_batch(in, n, kt, outs, mask_of(kt)))) return rc;
        }
        for (u32 b = 0; b < n; b++) {
            HIP_TRY(launch_mask_mul(c, level, mask_of(4), in[b], slot(c0 + b, 4), st));
            HIP_TRY(launch_mask_mul(c, level, mask_of(3), side[0] + (size_t)b * ct_elems, slot(c0 + b, 3), st));
            HIP_TRY(launch_mask_mul(c, level, mask_of(5), side[1] + (size_t)b * ct_elems, slot(c0 + b, 5), st));
        }
        // second stage: C^-1 and C^+1 rotated by -W and +W (their own decompositions)
        for (u32 sd = 0; sd < 2; sd++) {
            const u64* base[CT_BATCH];
            for (u32 b = 0; b < n; b++) {
                base[b] = side[sd] + (size_t)b * ct_elems;
                c1s[b] = base[b] + L1 * N;
            }
            if ((rc = run_modup(c, level, c1s, n, ws, st))) return rc;
            for (u32 kt = 1; kt <= 7; kt += 6) {
                const u32 t = (kt == 1 ? 0 : 6) + 2 * sd;  // corner taps 0, 2 (row -1) and 6, 8 (row +1)
                for (u32 b = 0; b < n; b++) outs[b] = slot(c0 + b, t);
                if (gs[kt] == 1) {
                    for (u32 b = 0; b < n; b++) HIP_TRY(launch_mask_mul(c, level, mask_of(t), base[b], outs[b], st));
                } else if ((rc = rotate_batch(base, n, kt, outs, mask_of(t)))) return rc;
            }
        }
    }
    // convolution evaluation: integer-weighted sum over (input channel, tap) for every output channel
    HIP_TRY(launch_weighted_sum(c, level, false, xs, XLayout::classic(L1, N), d->c_in * 9, (const u64*)d_w_res, d->c_out, acc, wscratch, d->weight_bits, st));
    for (u32 o0 = 0; o0 < d->c_out; o0 += CT_BATCH) {
        const u32 n = d->c_out - o0 < CT_BATCH ? d->c_out - o0 : CT_BATCH;
        const u64* ins[CT_BATCH];
        u64* outs[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            ins[b] = acc + (size_t)(o0 + b) * ct_elems;
            outs[b] = (u64*)h_d_out[o0 + b];
        }
        int rc = run_rescale(c, level, ins, L1 * N, outs, n, ar.rest(), st);
        if (rc) return rc;
    }
    return CKKS_OK;
}

size_t he_accumulator_workspace_bytes(const ckks_ctx* c, uint32_t level, uint32_t g) {
    if (!c || !c->dnum || !level_ok(c, level) || level < 1 || g == 0 || g > KS_MAX_BATCH) return 0;
    return ws_merge(c, level, g);
}

int he_accumulator_merge(const ckks_ctx* c, const uint64_t* const* h_d_cts, uint32_t g, uint32_t level, uint32_t sts,
                         const uint64_t* d_mask, const ckks_key* const* keys, uint64_t* d_out, void* d_ws, size_t ws_bytes,
                         void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!h_d_cts || !d_mask || !d_out || g == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or no ciphertexts");
    if (g > KS_MAX_BATCH) return set_err(c, CKKS_ERR_INVALID_ARG, "at most 16 ciphertexts per merge");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, level) || level < 1) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "merge needs 1 <= level < num_q");
    if (sts == 0 || (u64)g * sts > c->N / 2) return set_err(c, CKKS_ERR_INVALID_ARG, "g * sts exceeds the N/2 slots");
    u32 gal[KS_MAX_BATCH];
    for (u32 i = 0; i < g; i++) {
        if (!h_d_cts[i]) return set_err(c, CKKS_ERR_INVALID_ARG, "null ciphertext pointer");
        gal[i] = ckks_galois_element(c, -(int32_t)(i * sts));
        if (i == 0) continue;
        if (!keys || !keys[i]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key missing for a block");
        if (keys[i]->galois_elt != gal[i]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key does not match the block's offset");
    }
    return run_merge(c, (const u64* const*)h_d_cts, g, level, (const u64*)d_mask, keys, gal, (u64*)d_out, Arena(d_ws, ws_bytes),
                     (hipStream_t)stream);
}

// ---- slot re-layout with two rotations per element (down-sampling compaction, FC output reconstruction) ----
size_t he_relayout_workspace_bytes(const ckks_ctx* c, uint32_t level, uint32_t n_ct, uint32_t n_lo, uint32_t n_hi, uint32_t schedule) {
    if (!c || !c->dnum || !level_ok(c, level) || level < 1 || n_ct == 0 || n_lo == 0 || n_hi == 0 || schedule > HE_RELAYOUT_DEFERRED) return 0;
    return schedule == HE_RELAYOUT_DEFERRED ? ws_relayout_deferred(c, level, n_ct, n_lo, n_hi) : ws_relayout(c, level, n_ct, n_lo, n_hi);
}

int he_relayout_two_rotations(const ckks_ctx* c, const uint64_t* const* h_d_cts, uint32_t n_ct, uint32_t level, const int32_t* h_lo,
                              uint32_t n_lo, const ckks_key* const* lo_keys, const int32_t* h_hi, uint32_t n_hi,
                              const ckks_key* const* hi_keys, const uint64_t* const* h_d_masks, uint32_t schedule,
                              uint64_t* const* h_d_outs, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!h_d_cts || !h_lo || !h_hi || !h_d_masks || !h_d_outs || n_ct == 0 || n_lo == 0 || n_hi == 0)
        return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or an empty list");
    if (schedule > HE_RELAYOUT_DEFERRED) return set_err(c, CKKS_ERR_INVALID_ARG, "unknown schedule");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, level) || level < 1) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "the re-layout needs 1 <= level < num_q");
    if ((u64)n_lo * n_hi > (u64)c->N) return set_err(c, CKKS_ERR_INVALID_ARG, "more (lo, hi) pairs than coefficients");
    for (u32 b = 0; b < n_ct; b++)
        if (!h_d_cts[b] || !h_d_outs[b]) return set_err(c, CKKS_ERR_INVALID_ARG, "null ciphertext pointer");
    std::vector<u32> g_lo(n_lo), g_hi(n_hi);
    for (u32 l = 0; l < n_lo; l++) {
        g_lo[l] = ckks_galois_element(c, h_lo[l]);
        if (g_lo[l] != 1 && (!lo_keys || !lo_keys[l] || lo_keys[l]->galois_elt != g_lo[l]))
            return set_err(c, CKKS_ERR_NO_KEY, "key of a first rotation missing or made for another offset");
    }
    for (u32 h = 0; h < n_hi; h++) {
        g_hi[h] = ckks_galois_element(c, h_hi[h]);
        if (g_hi[h] != 1 && (!hi_keys || !hi_keys[h] || hi_keys[h]->galois_elt != g_hi[h]))
            return set_err(c, CKKS_ERR_NO_KEY, "key of a second rotation missing or made for another offset");
        bool any = false;
        for (u32 l = 0; l < n_lo; l++) any = any || h_d_masks[(size_t)h * n_lo + l];
        if (!any) return set_err(c, CKKS_ERR_INVALID_ARG, "a second rotation has no mask at all");
    }
    return (schedule == HE_RELAYOUT_DEFERRED ? run_relayout_deferred : run_relayout)(
        c, level, n_ct, (const u64* const*)h_d_cts, n_lo, lo_keys, g_lo.data(), n_hi, hi_keys, g_hi.data(), (const u64* const*)h_d_masks,
        (u64* const*)h_d_outs, Arena(d_ws, ws_bytes), (hipStream_t)stream);
}

// ---- batched fully connected layer ------------------------------------------------------------------
static u32 fc_base(const he_fc_desc* d) {
    if (d->base) return d->base;
    u32 b = 1;
    while (b * b < d->batch) b++;
    return b;
}

static size_t max3(size_t a, size_t b, size_t c3) { return a > b ? (a > c3 ? a : c3) : (b > c3 ? b : c3); }

size_t he_fc_workspace_bytes(const ckks_ctx* c, const he_fc_desc* d) {
    if (!c || !d || !c->dnum || !level_ok(c, d->level) || d->level < 3 || d->d_out == 0 || d->d_out > KS_MAX_BATCH || d->batch == 0) return 0;
    const size_t N = c->N;
    const u32 level = d->level, base = fc_base(d), n_lo = base < d->batch ? base : d->batch, n_hi = (d->batch + base - 1) / base;
    const size_t ct0 = 2 * (size_t)(level + 1) * N, ct1 = 2 * (size_t)level * N, ct2 = 2 * (size_t)(level - 1) * N;
    return blk(CT_BATCH * ct0) + blk(d->d_out * ct1) + blk(CT_BATCH * ct1) + blk(ct2) + ws_ks(c, level - 1, CT_BATCH, CT_BATCH) +
           max3(ws_merge(c, level - 1, d->d_out), ws_rescale(c, level, CT_BATCH), ws_relayout(c, level - 2, 1, n_lo, n_hi));
}

int he_fc_batched(const ckks_ctx* c, const he_fc_desc* d, const uint64_t* d_in, const uint64_t* d_w_enc, const ckks_key* const* sum_keys,
                  const ckks_key* const* merge_keys, const uint64_t* d_merge_mask, const uint64_t* d_place_masks,
                  const ckks_key* const* lo_keys, const ckks_key* const* hi_keys, const uint64_t* d_bias, uint64_t* d_out, void* d_ws,
                  size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d || !d_in || !d_w_enc || !d_merge_mask || !d_place_masks || !d_bias || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, d->level) || d->level < 3) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "the layer needs 3 <= level < num_q");
    if (d->d_in == 0 || (d->d_in & (d->d_in - 1)) || d->d_out == 0 || d->d_out > d->d_in || d->batch == 0)
        return set_err(c, CKKS_ERR_INVALID_ARG, "d_in must be a power of two and 1 <= d_out <= d_in");
    if (d->d_out > KS_MAX_BATCH) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "at most 16 outputs per call");
    if ((u64)d->batch * d->d_in > c->N / 2) return set_err(c, CKKS_ERR_INVALID_ARG, "batch * d_in exceeds the N/2 slots");
    const u32 level = d->level, l1 = level - 1, l2 = level - 2, l3 = level - 3;
    const u32 base = fc_base(d), n_lo = base < d->batch ? base : d->batch, n_hi = (d->batch + base - 1) / base;
    const u32 delta = d->d_in - d->d_out, n_sum = ilog2(d->d_in);
    // Galois elements and keys of every rotation, checked before the first launch
    u32 g_sum[32], g_merge[KS_MAX_BATCH];
    for (u32 s = 0; s < n_sum; s++) {
        g_sum[s] = ckks_galois_element(c, (int32_t)(1u << s));
        if (!sum_keys || !sum_keys[s] || sum_keys[s]->galois_elt != g_sum[s]) return set_err(c, CKKS_ERR_NO_KEY, "key of an inner-sum rotation missing or wrong");
    }
    for (u32 i = 0; i < d->d_out; i++) {
        g_merge[i] = ckks_galois_element(c, -(int32_t)i);
        if (i && (!merge_keys || !merge_keys[i] || merge_keys[i]->galois_elt != g_merge[i]))
            return set_err(c, CKKS_ERR_NO_KEY, "key of a merge rotation missing or wrong");
    }
    std::vector<u32> g_lo(n_lo), g_hi(n_hi);
    for (u32 l = 0; l < n_lo; l++) {
        g_lo[l] = ckks_galois_element(c, (int32_t)(l * delta));
        if (g_lo[l] != 1 && (!lo_keys || !lo_keys[l] || lo_keys[l]->galois_elt != g_lo[l]))
            return set_err(c, CKKS_ERR_NO_KEY, "key of a layout rotation (mod_idx) missing or wrong");
    }
    for (u32 h = 0; h < n_hi; h++) {
        g_hi[h] = ckks_galois_element(c, (int32_t)(h * base * delta));
        if (g_hi[h] != 1 && (!hi_keys || !hi_keys[h] || hi_keys[h]->galois_elt != g_hi[h]))
            return set_err(c, CKKS_ERR_NO_KEY, "key of a layout rotation (base_idx) missing or wrong");
    }
    const size_t N = c->N;
    const size_t ct0 = 2 * (size_t)(level + 1) * N, ct1 = 2 * (size_t)(l1 + 1) * N, ct2 = 2 * (size_t)(l2 + 1) * N, ct3 = 2 * (size_t)(l3 + 1) * N;
    Arena ar(d_ws, ws_bytes);
    u64* prod = ar.take(CT_BATCH * ct0);        // C_in (.) w_i before its rescale
    u64* S = ar.take(d->d_out * ct1);           // running inner sums, level-1
    u64* Srot = ar.take(CT_BATCH * ct1);        // their rotations
    u64* U = ar.take(ct2);                      // merged, level-2
    KsWs ws;
    bool ok = carve_ks(c, l1, CT_BATCH, CT_BATCH, ar, ws);
    if (!ok || !ar.ok() ||
        ar.used + max3(ws_merge(c, l1, d->d_out), ws_rescale(c, level, CT_BATCH), ws_relayout(c, l2, 1, n_lo, n_hi)) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the layer");
    hipStream_t st = (hipStream_t)stream;
    const u64* in = (const u64*)d_in;
    int rc;
    // 1. per-output products, rescale, inner sums over d_in slots (all outputs of a batch share each rotation key)
    for (u32 i0 = 0; i0 < d->d_out; i0 += CT_BATCH) {
        const u32 n = d->d_out - i0 < CT_BATCH ? d->d_out - i0 : CT_BATCH;
        const u64 *pp[CT_BATCH], *ps[CT_BATCH];
        u64 *os[CT_BATCH], *orot[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            HIP_TRY(launch_mask_mul(c, level, (const u64*)d_w_enc + (size_t)(i0 + b) * (level + 1) * N, in, prod + b * ct0, st));
            pp[b] = prod + b * ct0;
            ps[b] = os[b] = S + (i0 + b) * ct1;
            orot[b] = Srot + b * ct1;
        }
        if ((rc = run_rescale(c, level, pp, (size_t)(level + 1) * N, os, n, ar.rest(), st))) return rc;
        // T <- T + Rot(T, 2^s): the sum rides on the rotation's last kernel, the running sums alternate between two buffers
        const u64* cur[CT_BATCH];
        u64* nxt[CT_BATCH];
        for (u32 b = 0; b < n; b++) cur[b] = ps[b];
        for (u32 s = 0; s < n_sum; s++) {
            const ckks_key* ks[CT_BATCH];
            u32 gs[CT_BATCH];
            for (u32 b = 0; b < n; b++) {
                ks[b] = sum_keys[s];
                gs[b] = g_sum[s];
                nxt[b] = (s & 1) ? os[b] : orot[b];
            }
            if ((rc = run_rotate_batch(c, l1, n, cur, ks, gs, nxt, ws, st, cur))) return rc;
            for (u32 b = 0; b < n; b++) cur[b] = nxt[b];
        }
        if (n_sum & 1)  // an odd number of steps ends in the second buffer
            for (u32 b = 0; b < n; b++) HIP_TRY(launch_copy(orot[b], os[b], ct1, st));
    }
    // 2. merge over the outputs: element (j, i) to slot j*d_in + i
    {
        const u64* cts[KS_MAX_BATCH];
        for (u32 i = 0; i < d->d_out; i++) cts[i] = S + i * ct1;
        if ((rc = run_merge(c, cts, d->d_out, l1, (const u64*)d_merge_mask, merge_keys, g_merge, U, ar.rest(), st))) return rc;
    }
    // 3. layout: block j moves left by mod_idx = (j % base)*delta, then by base_idx = (j / base)*base*delta
    u64* out = (u64*)d_out;
    {
        std::vector<const u64*> masks((size_t)n_hi * n_lo, nullptr);
        for (u32 j = 0; j < d->batch; j++) masks[(size_t)(j / base) * n_lo + j % base] = (const u64*)d_place_masks + (size_t)j * (l2 + 1) * N;
        const u64* u_in = U;
        if ((rc = run_relayout(c, l2, 1, &u_in, n_lo, lo_keys, g_lo.data(), n_hi, hi_keys, g_hi.data(), masks.data(), &out, ar.rest(), st)))
            return rc;
    }
    // 4. bias on component 0
    HIP_TRY(launch_add_plain(c, l3, (const u64*)d_bias, out, st));
    return CKKS_OK;
}

int he_poly_act_deg7(const ckks_ctx* c, const uint64_t* const* h_d_x, uint32_t n_ct, uint32_t level, const int64_t* h_k,
                     const ckks_key* rlk, int merged_division, uint64_t* const* h_d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!h_d_x || !h_k || !h_d_out || n_ct == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer or no ciphertexts");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!rlk) return set_err(c, CKKS_ERR_NO_KEY, "no relinearisation key");
    if (rlk->galois_elt != 0) return set_err(c, CKKS_ERR_NO_KEY, "key is a rotation key, not the relinearisation key");
    if (!level_ok(c, level) || level < 4) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "activation needs 4 <= level < num_q");
    for (u32 i = 0; i < n_ct; i++)
        if (!h_d_x[i] || !h_d_out[i]) return set_err(c, CKKS_ERR_INVALID_ARG, "null ciphertext pointer");
    const size_t N = c->N;
    const u32 nb_max = n_ct < CT_BATCH ? n_ct : CT_BATCH;
    const u32 l1 = level - 1, l2 = level - 2, l3 = level - 3;
    const size_t xs = (size_t)(level + 1) * N;  // component stride of x
    const size_t x2s = (size_t)(l1 + 1) * N, x3s = (size_t)(l2 + 1) * N, Bs = (size_t)(l3 + 1) * N;
    // Batches of channels are independent: with room for two sets of scratch, every other batch goes to the library's side
    // stream (fork after the caller's earlier work, join before the call returns to the caller's stream).
    const size_t lane_bytes = ws_poly_act(c, level, nb_max);
    const u32 n_lanes = (n_ct > CT_BATCH && c->side_stream() && ws_bytes >= 2 * lane_bytes) ? 2 : 1;
    if (ws_bytes < lane_bytes || !d_ws) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the activation");
    hipStream_t st0 = (hipStream_t)stream;
    auto residues = [&](int64_t k, u32 lv, u64* out) {
        for (u32 i = 0; i <= lv; i++) {
            const u64 q = c->mod[i];
            out[i] = k >= 0 ? (u64)k % q : (q - ((u64)(-k) % q)) % q;
        }
    };
    u64 ka[CKKS_MAX_MODULI], kb[CKKS_MAX_MODULI];
    if (n_lanes == 2) {
        HIP_TRY(hipEventRecord(c->ev_fork, st0));
        HIP_TRY(hipStreamWaitEvent(c->side, c->ev_fork, 0));
    }
    auto join = [&](int rc) -> int {  // also on the error paths: the caller's stream never runs ahead of the side stream
        if (n_lanes == 2) {
            hipError_t e = hipEventRecord(c->ev_join, c->side);
            if (e == hipSuccess) e = hipStreamWaitEvent(st0, c->ev_join, 0);
            if (e != hipSuccess && rc == CKKS_OK) {
                c->err = std::string("joining the side stream: ") + hipGetErrorString(e);
                return CKKS_ERR_HIP;
            }
        }
        return rc;
    };

    for (u32 i0 = 0, batch_no = 0; i0 < n_ct; i0 += CT_BATCH, batch_no++) {
        const u32 n = n_ct - i0 < CT_BATCH ? n_ct - i0 : CT_BATCH;
        const u32 lane = n_lanes == 2 ? (batch_no & 1) : 0;
        hipStream_t st = lane ? c->side : st0;
        Arena ar((char*)d_ws + (size_t)lane * lane_bytes, lane_bytes);
        u64* x2 = ar.take(nb_max * 2 * x2s);        // level-1
        u64* x3 = ar.take(nb_max * 2 * x3s);        // level-2
        u64* x4 = ar.take(nb_max * 2 * x3s);        // level-2
        u64* B = ar.take(nb_max * 2 * Bs);          // level-3
        u64* tmp = ar.take(nb_max * 2 * xs);        // un-rescaled products
        if (!ar.ok()) return join(set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the activation"));
        // pointer lists of this batch: inputs, and the per-item slices of the intermediates
        const u64 *px[CT_BATCH], *px2[CT_BATCH], *px3[CT_BATCH], *px4[CT_BATCH], *pB[CT_BATCH], *ptmp[CT_BATCH];
        u64 *ox2[CT_BATCH], *ox3[CT_BATCH], *ox4[CT_BATCH], *oB[CT_BATCH], *otmp[CT_BATCH], *oout[CT_BATCH];
        for (u32 b = 0; b < n; b++) {
            px[b] = (const u64*)h_d_x[i0 + b];
            px2[b] = ox2[b] = x2 + b * 2 * x2s;
            px3[b] = ox3[b] = x3 + b * 2 * x3s;
            px4[b] = ox4[b] = x4 + b * 2 * x3s;
            pB[b] = oB[b] = B + b * 2 * Bs;
            oout[b] = (u64*)h_d_out[i0 + b];
        }
        auto tmp_at = [&](size_t cstride) {  // un-rescaled results, compact at the level that produced them
            for (u32 b = 0; b < n; b++) ptmp[b] = otmp[b] = tmp + b * 2 * cstride;
        };
        int rc;
        if (merged_division) {  // every relinearise-then-rescale pair as one division by P*q_level
            if ((rc = run_ctct_merged(c, level, px, xs, px, xs, nullptr, 0, rlk->d_key, ox2, n, ar.rest(), st))) return join(rc);
            if ((rc = run_ctct_merged(c, l1, px2, x2s, px, xs, nullptr, 0, rlk->d_key, ox3, n, ar.rest(), st))) return join(rc);
            if ((rc = run_ctct_merged(c, l1, px2, x2s, px2, x2s, nullptr, 0, rlk->d_key, ox4, n, ar.rest(), st))) return join(rc);
            residues(h_k[2], l2, ka);
            residues(h_k[3], l2, kb);
            if (ntt_has_modup(c)) {  // B = Rescale(k5 * x + k7 * x3) without storing the linear combination
                if ((rc = run_rescale_lin(c, l2, px, xs, ka, px3, x3s, kb, oB, n, ar.rest(), st))) return join(rc);
            } else {
                tmp_at(x3s);
                if (hipError_t he_ = (launch_lincomb2(c, l2, ptr_list(px, n), xs, ka, ptr_list(px3, n), x3s, kb, nullptr, 0, tmp, 2 * x3s, n, st)); he_ != hipSuccess) return join(set_hip_err(c, he_));
                if ((rc = run_rescale(c, l2, ptmp, x3s, oB, n, ar.rest(), st))) return join(rc);
            }
            // y = Rescale(x4 * B + (k1 * x + k3 * x3)): the linear part rides along as the product's addend
            residues(h_k[0], l3, ka);
            residues(h_k[1], l3, kb);
            if (ntt_has_modup(c)) {  // the linear part is formed inside the product's fused inner product
                const LinAddend lin = {px, xs, ka, px3, x3s, kb};
                if ((rc = run_ctct_merged(c, l3, px4, x3s, pB, Bs, nullptr, 0, rlk->d_key, oout, n, ar.rest(), st, &lin))) return join(rc);
                continue;
            }
            if (hipError_t he_ = (launch_lincomb2(c, l3, ptr_list(px, n), xs, ka, ptr_list(px3, n), x3s, kb, nullptr, 0, tmp, 2 * Bs, n, st)); he_ != hipSuccess) return join(set_hip_err(c, he_));
            if ((rc = run_ctct_merged(c, l3, px4, x3s, pB, Bs, tmp, 2 * Bs, rlk->d_key, oout, n, ar.rest(), st))) return join(rc);
            continue;
        }
        // x2 = Rescale(x * x)                                  level -> level-1
        tmp_at(xs);
        if ((rc = run_ctct(c, level, px, xs, px, xs, rlk->d_key, otmp, n, ar.rest(), st))) return join(rc);
        if ((rc = run_rescale(c, level, ptmp, xs, ox2, n, ar.rest(), st))) return join(rc);
        // x3 = Rescale(x2 * x), x4 = Rescale(x2 * x2)           level-1 -> level-2
        tmp_at(x2s);
        if ((rc = run_ctct(c, l1, px2, x2s, px, xs, rlk->d_key, otmp, n, ar.rest(), st))) return join(rc);
        if ((rc = run_rescale(c, l1, ptmp, x2s, ox3, n, ar.rest(), st))) return join(rc);
        if ((rc = run_ctct(c, l1, px2, x2s, px2, x2s, rlk->d_key, otmp, n, ar.rest(), st))) return join(rc);
        if ((rc = run_rescale(c, l1, ptmp, x2s, ox4, n, ar.rest(), st))) return join(rc);
        // B = Rescale(k5 * x + k7 * x3)                         level-2 -> level-3
        residues(h_k[2], l2, ka);
        residues(h_k[3], l2, kb);
        tmp_at(x3s);
        if (hipError_t he_ = (launch_lincomb2(c, l2, ptr_list(px, n), xs, ka, ptr_list(px3, n), x3s, kb, nullptr, 0, tmp, 2 * x3s, n, st)); he_ != hipSuccess) return join(set_hip_err(c, he_));
        if ((rc = run_rescale(c, l2, ptmp, x3s, oB, n, ar.rest(), st))) return join(rc);
        // y = Rescale((k1 * x + k3 * x3) + x4 * B)              level-3 -> level-4
        u64* prod = x2;  // x2 is no longer needed; n * [2][l3+1][N] fits in it
        u64* oprod[CT_BATCH];
        for (u32 b = 0; b < n; b++) oprod[b] = prod + b * 2 * Bs;
        if ((rc = run_ctct(c, l3, px4, x3s, pB, Bs, rlk->d_key, oprod, n, ar.rest(), st))) return join(rc);
        residues(h_k[0], l3, ka);
        residues(h_k[1], l3, kb);
        tmp_at(Bs);
        if (hipError_t he_ = (launch_lincomb2(c, l3, ptr_list(px, n), xs, ka, ptr_list(px3, n), x3s, kb, prod, 2 * Bs, tmp, 2 * Bs, n, st)); he_ != hipSuccess) return join(set_hip_err(c, he_));
        if ((rc = run_rescale(c, l3, ptmp, Bs, oout, n, ar.rest(), st))) return join(rc);
    }
    return join(CKKS_OK);
}

// ---- optional per-kernel timing -------------------------------------------------------------------
static const char* const kKernelNames[K_COUNT] = {
    "ntt_fwd_hi", "ntt_fwd_lo", "ntt_inv_lo", "ntt_inv_hi", "modup_conv", "key_inner", "moddown_conv", "moddown_final",
    "automorph", "copy", "ptct_mac", "rescale_conv", "rescale_final", "tensor", "mask_mul", "weighted_sum", "lincomb2"};

uint32_t ckks_prof_kernel_count(void) { return K_COUNT; }
const char* ckks_prof_kernel_name(uint32_t id) { return id < K_COUNT ? kKernelNames[id] : ""; }

int ckks_prof_begin(ckks_ctx* c, uint32_t kernel_mask, uint32_t max_launches) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (c->prof) return set_err(c, CKKS_ERR_INVALID_ARG, "profiling already on");
    if (max_launches == 0) return set_err(c, CKKS_ERR_INVALID_ARG, "max_launches must be positive");
    ProfState* p = new (std::nothrow) ProfState;
    if (!p) return set_err(c, CKKS_ERR_INVALID_ARG, "out of host memory");
    p->mask = kernel_mask;
    p->events.resize(2 * (size_t)max_launches);
    p->kernel_of_pair.resize(max_launches);
    for (size_t i = 0; i < p->events.size(); i++) {
        hipError_t e = hipEventCreate(&p->events[i]);
        if (e != hipSuccess) {
            for (size_t j = 0; j < i; j++) (void)hipEventDestroy(p->events[j]);
            delete p;
            c->err = std::string("hipEventCreate: ") + hipGetErrorString(e);
            return CKKS_ERR_HIP;
        }
    }
    c->prof = p;
    return CKKS_OK;
}

int ckks_prof_end(ckks_ctx* c, double* h_ms, uint64_t* h_launches, double* h_bytes, double* h_ops, uint64_t* h_dropped) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    ProfState* p = c->prof;
    if (!p) return set_err(c, CKKS_ERR_INVALID_ARG, "profiling is not on");
    c->prof = nullptr;
    int rc = CKKS_OK;
    for (u32 k = 0; k < K_COUNT; k++) {
        if (h_ms) h_ms[k] = 0.0;
        if (h_launches) h_launches[k] = 0;
        if (h_bytes) h_bytes[k] = p->bytes[k];
        if (h_ops) h_ops[k] = p->ops[k];
    }
    for (size_t i = 0; i < p->used_pairs && rc == CKKS_OK; i++) {
        hipError_t e = hipEventSynchronize(p->events[2 * i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, p->events[2 * i], p->events[2 * i + 1]);
        if (e != hipSuccess) {
            c->err = std::string("profiling events: ") + hipGetErrorString(e);
            rc = CKKS_ERR_HIP;
            break;
        }
        if (h_ms) h_ms[p->kernel_of_pair[i]] += ms;
        if (h_launches) h_launches[p->kernel_of_pair[i]]++;
    }
    if (h_dropped) *h_dropped = p->dropped;
    for (hipEvent_t ev : p->events) (void)hipEventDestroy(ev);
    delete p;
    return rc;
}

}  // extern "C"
