// The C boundary: argument checks, workspace carving and the order of kernel launches of every
// exported operation.  No arithmetic happens on the host; no call here allocates or synchronises.
#include <cstdio>
#include <new>

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

// ---- workspace sizes ---------------------------------------------------------------------------
// rb = how many key switches share one pass of the ModDown kernels (1..KS_MAX_BATCH)
size_t ws_keyswitch(const ckks_ctx* c, u32 level, u32 rb = 1) {
    const size_t N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    return blk(L1 * N) + blk(beta * E * N) + blk(rb * 2 * E * N) + blk(rb * 2 * L1 * N);
}
size_t ws_rescale(const ckks_ctx* c, u32 level) { return blk(2 * (size_t)c->N) + blk(2 * (size_t)level * c->N); }
size_t ws_ctct(const ckks_ctx* c, u32 level) { return 3 * blk((size_t)(level + 1) * c->N) + ws_keyswitch(c, level); }

struct KsBuffers {
    u64 *y, *digits, *v, *w;
};
bool carve_ks(const ckks_ctx* c, u32 level, Arena& ar, KsBuffers& b, u32 rb = 1) {
    const size_t N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    b.y = ar.take(L1 * N);
    b.digits = ar.take(beta * E * N);
    b.v = ar.take(rb * 2 * E * N);
    b.w = ar.take(rb * 2 * L1 * N);
    return ar.ok();
}

// Decompose + ModUp of one polynomial d_c [level+1][N] (NTT form) into b.digits [beta][E][N] (NTT form).
int run_modup(const ckks_ctx* c, u32 level, const u64* d_c, const KsBuffers& b, hipStream_t st) {
    const u32 N = c->N, L1 = level + 1, E = c->ext_limbs(level), beta = c->live_digits(level);
    // all live limbs to coefficient form at once
    HIP_TRY(launch_ntt(c, true, d_c, L1, b.y, L1, range_list(0, L1, 0), 1, st));
    for (u32 j = 0; j < beta; j++) {
        const u32 lo = c->digit_lo(j), hi = c->digit_hi(j, level);
        u64* digit = b.digits + (size_t)j * E * N;
        HIP_TRY(launch_modup_conv(c, level, j, b.y + (size_t)lo * N, d_c, digit, st));
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
        HIP_TRY(launch_ntt(c, false, digit, E, digit, E, pl, 1, st));
    }
    return CKKS_OK;
}

// n <= KS_MAX_BATCH key switches of the same extended digits: inner product with each key (digits read
// through sigma_g of the item), then one pass of every ModDown kernel over the whole batch.  items[r]
// says what is added to / multiplied into the r-th result and where it goes ([2][level+1][N]).
int run_inner_moddown(const ckks_ctx* c, u32 level, const KsBuffers& b, u32 n, const u64* const* d_keys, const FinalItem* items,
                      hipStream_t st) {
    const u32 L1 = level + 1, E = c->ext_limbs(level), k = c->num_p;
    const size_t N = c->N;
    for (u32 r = 0; r < n; r++) HIP_TRY(launch_key_inner(c, level, b.digits, d_keys[r], items[r].g, b.v + (size_t)r * 2 * E * N, st));
    // P-part of every component to coefficient form, in place
    HIP_TRY(launch_ntt(c, true, b.v, E, b.v, E, range_list(L1, k, c->num_q), 2 * n, st));
    HIP_TRY(launch_moddown_conv(c, level, b.v, b.w, 2 * n, st));
    HIP_TRY(launch_ntt(c, false, b.w, L1, b.w, L1, range_list(0, L1, 0), 2 * n, st));
    HIP_TRY(launch_moddown_final(c, level, b.v, b.w, items, n, st));
    return CKKS_OK;
}

int run_rescale(const ckks_ctx* c, u32 level, const u64* ct, size_t ct_cstride, u64* out, Arena& ar, hipStream_t st) {
    const size_t N = c->N;
    u64* r = ar.take(2 * N);
    u64* w = ar.take(2 * (size_t)level * N);
    if (!ar.ok()) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rescale");
    // dropped limb of both components -> coefficient form
    PolyList pl = range_list(0, 1, level);
    HIP_TRY(launch_ntt(c, true, ct + (size_t)level * N, ct_cstride / N, r, 1, pl, 2, st));
    HIP_TRY(launch_rescale_conv(c, level, r, w, st));
    HIP_TRY(launch_ntt(c, false, w, level, w, level, range_list(0, level, 0), 2, st));
    HIP_TRY(launch_rescale_final(c, level, ct, ct_cstride, w, out, st));
    return CKKS_OK;
}

// (a*b relinearised) with operands possibly living at a higher level (component strides given)
int run_ctct(const ckks_ctx* c, u32 level, const u64* a, size_t a_cstride, const u64* b, size_t b_cstride, const u64* d_rlk,
             u64* out, Arena& ar, hipStream_t st) {
    const size_t N = c->N, L1 = level + 1;
    u64* d0 = ar.take(L1 * N);
    u64* d1 = ar.take(L1 * N);
    u64* d2 = ar.take(L1 * N);
    KsBuffers kb;
    if (!carve_ks(c, level, ar, kb)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for ct-ct multiply");
    HIP_TRY(launch_tensor(c, level, a, a_cstride, b, b_cstride, d0, d1, d2, st));
    int rc = run_modup(c, level, d2, kb, st);
    if (rc) return rc;
    const FinalItem item = {d0, d1, nullptr, out, 1, 0};
    return run_inner_moddown(c, level, kb, 1, &d_rlk, &item, st);
}

bool level_ok(const ckks_ctx* c, u32 level) { return level < c->num_q; }

}  // namespace

extern "C" {

size_t ckks_workspace_bytes(const ckks_ctx* c, int op, uint32_t level, uint32_t count) {
    if (!c || !level_ok(c, level)) return 0;
    const size_t N = c->N, L1 = level + 1;
    switch (op) {
        case CKKS_OP_KEYSWITCH: return c->dnum ? ws_keyswitch(c, level) : 0;
        case CKKS_OP_ROTATE: {
            const u32 rb = count < 1 ? 1 : (count > KS_MAX_BATCH ? KS_MAX_BATCH : count);
            return c->dnum ? ws_keyswitch(c, level, rb) + blk(L1 * N) : 0;
        }
        case CKKS_OP_RESCALE: return level >= 1 ? ws_rescale(c, level) : 0;
        case CKKS_OP_CTCT_MUL_RELIN: return c->dnum ? ws_ctct(c, level) : 0;
        case CKKS_OP_POLY_ACT: {
            if (!c->dnum || level < 4) return 0;
            // x2 [level], x3, x4 [level-1], B [level-2], product/pre-rescale scratch [level+1], plus one
            // ct-ct multiply and one rescale at the top level
            size_t s = blk(2 * (size_t)level * N) + 2 * blk(2 * (size_t)(level - 1) * N) + blk(2 * (size_t)(level - 2) * N) +
                       blk(2 * L1 * N);
            return s + ws_ctct(c, level) + ws_rescale(c, level);
        }
        default: (void)count; return 0;
    }
}

size_t he_conv_workspace_bytes(const ckks_ctx* c, const he_conv_desc* d) {
    if (!c || !d || !c->dnum || !level_ok(c, d->level) || d->level < 1) return 0;
    const size_t N = c->N, L1 = d->level + 1;
    return ws_keyswitch(c, d->level, KS_MAX_BATCH) + blk((size_t)d->c_in * 9 * 2 * L1 * N) + blk((size_t)d->c_out * 2 * L1 * N) +
           blk(weighted_sum_scratch_elems(c, d->level, d->c_in * 9, d->c_out)) + ws_rescale(c, d->level);
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

int ckks_keyswitch(const ckks_ctx* c, const uint64_t* d_c, uint32_t level, const ckks_key* key, uint64_t* d_out, void* d_ws,
                   size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_c || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!key) return set_err(c, CKKS_ERR_NO_KEY, "no key");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    Arena ar(d_ws, ws_bytes);
    KsBuffers b;
    if (!carve_ks(c, level, ar, b)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for key switch");
    hipStream_t st = (hipStream_t)stream;
    int rc = run_modup(c, level, (const u64*)d_c, b, st);
    if (rc) return rc;
    const FinalItem item = {nullptr, nullptr, nullptr, (u64*)d_out, 1, 0};
    return run_inner_moddown(c, level, b, 1, &key->d_key, &item, st);
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
    bool any = false;
    for (u32 t = 0; t < n_rot; t++) {
        if (!h_d_outs[t]) return set_err(c, CKKS_ERR_INVALID_ARG, "null output pointer");
        const u32 g = ckks_galois_element(c, h_offsets[t]);
        if (g == 1) continue;
        any = true;
        if (!keys || !keys[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key missing");
        if (keys[t]->galois_elt != g) return set_err(c, CKKS_ERR_NO_KEY, "rotation key was made for another offset");
    }
    // hoisted rotations go through the ModDown kernels in batches of up to KS_MAX_BATCH
    u32 n_keyed = 0;
    for (u32 t = 0; t < n_rot; t++) n_keyed += ckks_galois_element(c, h_offsets[t]) != 1;
    const u32 rb = hoisted ? (n_keyed < KS_MAX_BATCH ? (n_keyed ? n_keyed : 1) : KS_MAX_BATCH) : 1;
    Arena ar(d_ws, ws_bytes);
    KsBuffers b = {nullptr, nullptr, nullptr, nullptr};
    u64* pc1 = nullptr;
    if (any) {
        if (!carve_ks(c, level, ar, b, rb)) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rotation");
        if (!hoisted) {
            pc1 = ar.take(L1 * N);
            if (!ar.ok()) return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for rotation");
        }
    }
    hipStream_t st = (hipStream_t)stream;
    const u64* ct = (const u64*)d_ct;
    const u64* c0 = ct;
    const u64* c1 = ct + L1 * N;
    if (any && hoisted) {
        int rc = run_modup(c, level, c1, b, st);
        if (rc) return rc;
    }
    FinalItem items[KS_MAX_BATCH];
    const u64* bkeys[KS_MAX_BATCH];
    u32 nb = 0;
    for (u32 t = 0; t < n_rot; t++) {
        const u32 g = ckks_galois_element(c, h_offsets[t]);
        u64* out = (u64*)h_d_outs[t];
        if (g == 1) {
            HIP_TRY(launch_copy(ct, out, 2 * L1 * N, st));
            continue;
        }
        if (hoisted) {
            items[nb] = FinalItem{c0, nullptr, nullptr, out, g, 0};
            bkeys[nb] = keys[t]->d_key;
            if (++nb == rb) {
                int rc = run_inner_moddown(c, level, b, nb, bkeys, items, st);
                if (rc) return rc;
                nb = 0;
            }
        } else {
            HIP_TRY(launch_automorph(c, (u32)L1, c1, g, pc1, st));
            int rc = run_modup(c, level, pc1, b, st);
            if (rc) return rc;
            // the digits already belong to sigma_g(c1): no gather in the inner product, only on c0
            const u32 E = c->ext_limbs(level), k = c->num_p;
            HIP_TRY(launch_key_inner(c, level, b.digits, keys[t]->d_key, 1, b.v, st));
            HIP_TRY(launch_ntt(c, true, b.v, E, b.v, E, range_list((u32)L1, k, c->num_q), 2, st));
            HIP_TRY(launch_moddown_conv(c, level, b.v, b.w, 2, st));
            HIP_TRY(launch_ntt(c, false, b.w, L1, b.w, L1, range_list(0, (u32)L1, 0), 2, st));
            const FinalItem item = {c0, nullptr, nullptr, out, g, 0};
            HIP_TRY(launch_moddown_final(c, level, b.v, b.w, &item, 1, st));
        }
    }
    if (nb) {
        int rc = run_inner_moddown(c, level, b, nb, bkeys, items, st);
        if (rc) return rc;
    }
    return CKKS_OK;
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
    Arena ar(d_ws, ws_bytes);
    return run_rescale(c, level, (const u64*)d_ct, (size_t)(level + 1) * c->N, (u64*)d_out, ar, (hipStream_t)stream);
}

int ckks_ctct_mul_relin(const ckks_ctx* c, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, const ckks_key* rlk,
                        uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_a || !d_b || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!rlk) return set_err(c, CKKS_ERR_NO_KEY, "no relinearisation key");
    if (rlk->galois_elt != 0) return set_err(c, CKKS_ERR_NO_KEY, "key is a rotation key, not the relinearisation key");
    if (!level_ok(c, level)) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "level out of range");
    Arena ar(d_ws, ws_bytes);
    const size_t cs = (size_t)(level + 1) * c->N;
    return run_ctct(c, level, (const u64*)d_a, cs, (const u64*)d_b, cs, rlk->d_key, (u64*)d_out, ar, (hipStream_t)stream);
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
    const u32 level = d->level;
    const size_t N = c->N, L1 = level + 1, ct_elems = 2 * L1 * N;
    int32_t offs[9];
    u32 gs[9];
    {
        u32 t = 0;
        for (int dy = -1; dy <= 1; dy++)
            for (int dx = -1; dx <= 1; dx++, t++) {
                offs[t] = dy * (int32_t)d->width + dx;
                gs[t] = ckks_galois_element(c, offs[t]);
                if (gs[t] == 1) continue;
                if (!rot_keys[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key missing for a tap");
                if (rot_keys[t]->galois_elt != gs[t]) return set_err(c, CKKS_ERR_NO_KEY, "rotation key does not match its tap offset");
            }
    }
    for (u32 i = 0; i < d->c_in; i++) if (!h_d_in[i]) return set_err(c, CKKS_ERR_INVALID_ARG, "null input ciphertext");
    for (u32 o = 0; o < d->c_out; o++) if (!h_d_out[o]) return set_err(c, CKKS_ERR_INVALID_ARG, "null output ciphertext");

    Arena ar(d_ws, ws_bytes);
    KsBuffers b;
    bool ok = carve_ks(c, level, ar, b, KS_MAX_BATCH);
    u64* xs = ar.take((size_t)d->c_in * 9 * ct_elems);
    u64* acc = ar.take((size_t)d->c_out * ct_elems);
    u64* wscratch = ar.take(weighted_sum_scratch_elems(c, level, d->c_in * 9, d->c_out));
    if (!ok || !ar.ok() || ar.used + ws_rescale(c, level) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the convolution");
    hipStream_t st = (hipStream_t)stream;

    // input alignment: nine aligned copies of every input channel, each times its tap mask; the eight
    // rotations of a channel share the decomposition and go through the ModDown kernels as one batch
    for (u32 ci = 0; ci < d->c_in; ci++) {
        const u64* ct = (const u64*)h_d_in[ci];
        int rc = run_modup(c, level, ct + L1 * N, b, st);
        if (rc) return rc;
        FinalItem items[KS_MAX_BATCH];
        const u64* bkeys[KS_MAX_BATCH];
        u32 nb = 0;
        for (u32 t = 0; t < 9; t++) {
            const u64* mask = (const u64*)d_tap_masks + (size_t)t * L1 * N;
            u64* x = xs + ((size_t)ci * 9 + t) * ct_elems;
            if (gs[t] == 1) {
                HIP_TRY(launch_mask_mul(c, level, mask, ct, x, st));
                continue;
            }
            items[nb] = FinalItem{ct, nullptr, mask, x, gs[t], 0};
            bkeys[nb] = rot_keys[t]->d_key;
            if (++nb == KS_MAX_BATCH) {
                if ((rc = run_inner_moddown(c, level, b, nb, bkeys, items, st))) return rc;
                nb = 0;
            }
        }
        if (nb && (rc = run_inner_moddown(c, level, b, nb, bkeys, items, st))) return rc;
    }
    // convolution evaluation: integer-weighted sum over (input channel, tap) for every output channel
    HIP_TRY(launch_weighted_sum(c, level, xs, d->c_in * 9, (const u64*)d_w_res, d->c_out, acc, wscratch, st));
    for (u32 o = 0; o < d->c_out; o++) {
        Arena tmp(ar.base + ar.used, ar.cap - ar.used);
        int rc = run_rescale(c, level, acc + (size_t)o * ct_elems, L1 * N, (u64*)h_d_out[o], tmp, st);
        if (rc) return rc;
    }
    return CKKS_OK;
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

int he_poly_act_deg7(const ckks_ctx* c, const uint64_t* d_x, uint32_t level, const int64_t* h_k, const ckks_key* rlk,
                     uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    if (!d_x || !h_k || !d_out) return set_err(c, CKKS_ERR_INVALID_ARG, "null pointer");
    if (!c->dnum) return set_err(c, CKKS_ERR_UNSUPPORTED_PARAMS, "context has no key-switching digits");
    if (!rlk) return set_err(c, CKKS_ERR_NO_KEY, "no relinearisation key");
    if (rlk->galois_elt != 0) return set_err(c, CKKS_ERR_NO_KEY, "key is a rotation key, not the relinearisation key");
    if (!level_ok(c, level) || level < 4) return set_err(c, CKKS_ERR_LEVEL_MISMATCH, "activation needs 4 <= level < num_q");
    const size_t N = c->N;
    Arena ar(d_ws, ws_bytes);
    u64* x2 = ar.take(2 * (size_t)level * N);         // level-1
    u64* x3 = ar.take(2 * (size_t)(level - 1) * N);   // level-2
    u64* x4 = ar.take(2 * (size_t)(level - 1) * N);   // level-2
    u64* B = ar.take(2 * (size_t)(level - 2) * N);    // level-3
    u64* tmp = ar.take(2 * (size_t)(level + 1) * N);  // un-rescaled products
    if (!ar.ok() || ar.used + ws_ctct(c, level) + ws_rescale(c, level) > ar.cap)
        return set_err(c, CKKS_ERR_WORKSPACE_TOO_SMALL, "workspace too small for the activation");
    hipStream_t st = (hipStream_t)stream;
    const u64* x = (const u64*)d_x;
    const size_t xs = (size_t)(level + 1) * N;  // component stride of x
    auto scratch = [&]() { return Arena(ar.base + ar.used, ar.cap - ar.used); };
    auto residues = [&](int64_t k, u32 lv, u64* out) {
        for (u32 i = 0; i <= lv; i++) {
            const u64 q = c->mod[i];
            out[i] = k >= 0 ? (u64)k % q : (q - ((u64)(-k) % q)) % q;
        }
    };
    int rc;
    // x2 = Rescale(x * x)                                  level -> level-1
    { Arena s = scratch(); if ((rc = run_ctct(c, level, x, xs, x, xs, rlk->d_key, tmp, s, st))) return rc; }
    { Arena s = scratch(); if ((rc = run_rescale(c, level, tmp, xs, x2, s, st))) return rc; }
    const u32 l1 = level - 1, l2 = level - 2, l3 = level - 3;
    const size_t x2s = (size_t)(l1 + 1) * N, x3s = (size_t)(l2 + 1) * N;
    // x3 = Rescale(x2 * x), x4 = Rescale(x2 * x2)           level-1 -> level-2
    { Arena s = scratch(); if ((rc = run_ctct(c, l1, x2, x2s, x, xs, rlk->d_key, tmp, s, st))) return rc; }
    { Arena s = scratch(); if ((rc = run_rescale(c, l1, tmp, x2s, x3, s, st))) return rc; }
    { Arena s = scratch(); if ((rc = run_ctct(c, l1, x2, x2s, x2, x2s, rlk->d_key, tmp, s, st))) return rc; }
    { Arena s = scratch(); if ((rc = run_rescale(c, l1, tmp, x2s, x4, s, st))) return rc; }
    // B = Rescale(k5 * x + k7 * x3)                         level-2 -> level-3
    u64 ka[CKKS_MAX_MODULI], kb[CKKS_MAX_MODULI];
    residues(h_k[2], l2, ka);
    residues(h_k[3], l2, kb);
    HIP_TRY(launch_lincomb2(c, l2, x, xs, ka, x3, x3s, kb, nullptr, tmp, st));
    { Arena s = scratch(); if ((rc = run_rescale(c, l2, tmp, x3s, B, s, st))) return rc; }
    // y = Rescale((k1 * x + k3 * x3) + x4 * B)              level-3 -> level-4
    const size_t Bs = (size_t)(l3 + 1) * N;
    u64* prod = x2;  // x2 is no longer needed; [2][l3+1][N] fits in it
    { Arena s = scratch(); if ((rc = run_ctct(c, l3, x4, x3s, B, Bs, rlk->d_key, prod, s, st))) return rc; }
    residues(h_k[0], l3, ka);
    residues(h_k[1], l3, kb);
    HIP_TRY(launch_lincomb2(c, l3, x, xs, ka, x3, x3s, kb, prod, tmp, st));
    { Arena s = scratch(); if ((rc = run_rescale(c, l3, tmp, Bs, (u64*)d_out, s, st))) return rc; }
    return CKKS_OK;
}

}  // extern "C"
