// Internal: the immutable context (host mirror + device tables) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "../../include/ckks.h"
#include "f64mod.h"
#include "modarith.h"

#define CKKS_MAX_MODULI 64
#define CKKS_TILE_LOG 11  // one workgroup transforms 2^11 points held in LDS

// Which limb-polys a batched kernel touches: entry a of the list reads the poly at position
// spos[a] of the source block and writes position dpos[a] of the destination block, modulo
// moduli[mod[a]].  Passed by value.
struct PolyList {
    u32 n;
    unsigned char spos[CKKS_MAX_MODULI];
    unsigned char dpos[CKKS_MAX_MODULI];
    unsigned char mod[CKKS_MAX_MODULI];
};

// a constant multiplier and its Shoup companion floor(w * 2^64 / q), loaded as one 16-byte word
struct __attribute__((aligned(16))) TwPair {
    u64 w, s;
};

// the same for the double-precision butterflies: TwF (f64mod.h), the twiddle as a double and twiddle / q rounded to nearest
// per-modulus constants of the double-precision butterflies
#define POW256_ROW 42  // 13 x 3 parts, 2^17 mod q, (2^17 mod q) / q, one word of padding

struct ModConstF {
    double q, qinv;        // the modulus and 1/q rounded to nearest
    double ninv, ninv_q;   // N^-1 mod q and (N^-1 mod q) / q
};

// kernel classes, for the optional per-kernel timing (ckks_prof_begin / ckks_prof_end)
enum KernelId {
    K_NTT_FWD_HI = 0, K_NTT_FWD_LO, K_NTT_INV_LO, K_NTT_INV_HI, K_MODUP_CONV, K_KEY_INNER, K_MODDOWN_CONV, K_MODDOWN_FINAL,
    K_AUTOMORPH, K_COPY, K_PTCT_MAC, K_RESCALE_CONV, K_RESCALE_FINAL, K_TENSOR, K_MASK_MUL, K_WEIGHTED_SUM, K_LINCOMB2, K_COUNT
};

struct ProfState {
    std::vector<hipEvent_t> events;  // pairs (start, stop)
    std::vector<int> kernel_of_pair;
    size_t used_pairs = 0, dropped = 0;
    u32 mask = 0;
    double bytes[K_COUNT] = {0};  // algorithmic HBM bytes of the recorded launches
    double ops[K_COUNT] = {0};    // modular multiplications (butterflies, multiply-adds) of the recorded launches
};

// Batched kernels take up to KS_MAX_BATCH items; item b's operand starts at p[b].
#define KS_MAX_BATCH 16   // pointer-list capacity; ciphertext batches are at most CT_BATCH = 8 (two components each)
#define CT_BATCH 8
struct PtrList8 {
    const u64* p[KS_MAX_BATCH];
};
struct OutList8 {
    u64* p[KS_MAX_BATCH];
};

// Where element (term k, component comp, limb e, point x) of the operands of the layer's multiply-accumulate
// lives:  base + k*s_k + comp*s_comp + e*s_e + (x >> 6)*s_xt + (x & 63).  Two layouts:
//   classic  [k][comp][limb][N]: every term is a ciphertext-shaped array (s_k = 2*nl*N, s_comp = nl*N, s_e = N, s_xt = 64)
//   tiled    [limb][comp][N/64][k][64]: all terms of one (limb, component, 64 points) are one contiguous run, which
//            is what one workgroup of the matrix-core kernel consumes and what one wavefront of the fused inner
//            product scatters into (s_k = 64, s_xt = 64*K, s_comp = N*K, s_e = 2*N*K); needs N % 64 == 0
struct XLayout {
    size_t s_k, s_comp, s_e, s_xt;
    __host__ __device__ size_t at(size_t k, u32 comp, u32 e, u32 x) const { return k * s_k + comp * s_comp + e * s_e + (size_t)(x >> 6) * s_xt + (x & 63); }
    static XLayout classic(size_t nl, size_t N) { return XLayout{2 * nl * N, nl * N, N, 64}; }
    static XLayout tiled(size_t K, size_t N) { return XLayout{64, N * K, 2 * N * K, 64 * K}; }
};

// One key switch of a batch, as its last kernel sees it (see moddown_final_kernel).
struct FinalItem {
    const u64* add0;
    const u64* add1;
    const u64* mask;
    u64* out;
    u32 g;
    u32 pad;
    const u64* acc;  // optional: a ciphertext shaped like `out`, added to it as it is (no gather, after the mask): out = ... + acc
};
// Where the inner-product kernels find the extended digits of batch item b: digit j, position e of the extended basis is
// row (j*E + e) of digits + b*bstride, except for the digit's OWN limbs (e <= level, e / alpha == j), which ModUp does not
// copy: they are the limbs of the decomposed polynomial itself, own.p[b] ([level+1][N], evaluation form).
struct DigitSrc {
    const u64* digits;
    size_t bstride;
    PtrList8 own;
    u32 alpha, pad;
};
struct FinalBatch {
    FinalItem it[KS_MAX_BATCH];
};
// The last step of a division by dropped moduli (ModDown, or ModDown merged with the rescale), applied by the forward
// transform itself as it stores its results w (batch item 2r + comp, limb i) instead of writing them:
//   out_r[comp][i] = ((v[2r+comp][i] - w) * cinv[i] + addend) * mask      (addend, mask as in FinalItem)
struct FwdEpilogue {
    const u64* v;         // [batch][E][N]
    const u64* cinv;      // the multiplier per limb, its Shoup companion at cinv[num_q + i]
    const ModConst* mci;  // integer constants per modulus
    u32 E, n_out, num_q;
    u32 use_vl;           // v is given per ciphertext instead: item 2r + comp reads vl.p[r] + comp * v_cstride (the rescale)
    PtrList8 vl;
    size_t v_cstride;
    // use_vl == 2 (double-precision arithmetic): v = ka * vl + kb * vl2, a linear combination of two ciphertexts with one
    // scalar residue per limb, formed as it is read
    PtrList8 vl2;
    size_t v2_cstride;
    u64 ka[CKKS_MAX_MODULI], kb[CKKS_MAX_MODULI];
    FinalBatch B;
};

struct ckks_key {
    const u64* d_key;
    u32 galois_elt;
};

struct ckks_ctx {
    u32 log_n, N, num_q, num_p, dnum, alpha, M;
    u32 log_lo, log_hi;  // N = 2^log_hi blocks-of-stride x 2^log_lo contiguous
    bool small_q;        // every modulus is below 2^50: carry-free 25-bit-split accumulation applies
    u32 lazy_terms;      // how many products of two residues may be summed in 128 bits before a reduction
    std::vector<u64> mod, psi;
    std::vector<ModConst> mc;

    // device tables
    ModConst* d_mc = nullptr;         // [M]
    TwPair* d_tw = nullptr;           // [M][N]  psi^bitrev(i) with its Shoup companion   (integer butterflies)
    TwPair* d_itw = nullptr;          // [M][N]  psi^-bitrev(i) with its Shoup companion
    bool ntt_f64 = false;             // moduli below 2^50 and N >= 2^11: double-precision butterflies, tables below instead
    TwF* d_twf = nullptr;             // [M][N]  psi^bitrev(i) and psi^bitrev(i) / q as doubles
    TwF* d_itwf = nullptr;
    double* d_twf_val = nullptr;      // [M][N]  psi^bitrev(i) alone: what the lo passes read (half the bytes of d_twf)
    double* d_itwf_val = nullptr;
    ModConstF* d_mcf = nullptr;       // [M]
    double* d_pow256 = nullptr;       // [M][POW256_ROW]: 2^(8s) mod q, s < 13, in parts of 17, 17 and 16 bits, then 2^17 mod q and its quotient by q (moduli below 2^50 only)
    u64* d_modup = nullptr;           // per level, per digit: see modup_digit_stride()
    u64* d_moddown = nullptr;         // phat_inv[k_pad], phat_inv_sh[k_pad], phat_q[num_q][k_pad], pinv[num_q], pinv_sh[num_q], negp[num_q]
    u64* d_moddown_rs = nullptr;      // per level l >= 1, the same layout (k_pad -> k2_pad) for the dropped set {q_l, p_0..p_{k-1}}:
                                      // ModDown and rescale as one division by P*q_l; see moddown_rs_table()
    u32* d_check = nullptr;           // one word: the violation count of he_conv_check_weights
    u64* d_rescale = nullptr;         // [num_q][num_q][3]: (q_l^-1 mod q_i, its Shoup companion, q_l mod q_i)
    // The conversion constants once more as doubles (w, w / q_target), for the double-precision base conversions that
    // contexts with ntt_f64 use: same row layout as the integer tables, one TwF per entry.
    TwF* d_modup_f = nullptr;         // [level][digit][M positions e][alpha_pad]
    TwF* d_modup_prep_f = nullptr;    // [level][num_q]: N^-1 (Q_j/q_i)^-1 mod q_i, what the inverse transform in front of ModUp scales by
    TwF* d_moddown_f = nullptr;       // [num_q][k_pad]
    TwF* d_moddown_rs_f = nullptr;    // [level][num_q][k2_pad]
    TwF* d_rescale_prep_f = nullptr;     // [M], by modulus: N^-1 mod q_m (the inverse transform in front of a fused rescale)
    TwF* d_rescale_conv_f = nullptr;     // [num_q][4]: (1, 1 / q_i), 0, 0, 0: the "conversion" of the one dropped limb
    u64* d_rescale_ep = nullptr;         // [level][2][num_q]: q_level^-1 mod q_i and its Shoup companion, as FwdEpilogue.cinv
    TwF* d_moddown_prep_f = nullptr;     // [M], by modulus: N^-1 (P/p_a)^-1 mod p_a at the special primes (zero elsewhere)
    TwF* d_moddown_rs_prep_f = nullptr;  // [level][M], by modulus: N^-1 (P q_l / m)^-1 mod m for m in {q_l, p_0..p_{k-1}}
    const TwF* modup_table_f(u32 level, u32 j) const { return d_modup_f + ((size_t)level * dnum + j) * M * alpha_pad; }
    const TwF* moddown_rs_table_f(u32 level) const { return d_moddown_rs_f + (size_t)level * num_q * k2_pad; }

    // A second stream of the library's own (default priority) with the two events of a fork/join: operations made of
    // independent channel batches put every other batch on it, so that kernels bound by arithmetic overlap with
    // kernels bound by memory traffic.  The caller sees all work ordered in its own stream.  Calls that use it must
    // not be issued on one context from several host threads at once.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool overlap = true;  // ckks_ctx_set_overlap: off = everything on the caller's stream
    hipStream_t side_stream() const { return overlap ? side : nullptr; }

    int device = 0;  // the HIP device the tables live on (the one that was current at creation)

    mutable std::string err;
    mutable ProfState* prof = nullptr;  // non-null between ckks_prof_begin and ckks_prof_end

    u32 ext_limbs(u32 level) const { return level + 1 + num_p; }
    u32 live_digits(u32 level) const { return (level + alpha) / alpha; }
    u32 digit_lo(u32 j) const { return j * alpha; }
    u32 digit_hi(u32 j, u32 level) const { u32 h = (j + 1) * alpha; return h < level + 1 ? h : level + 1; }
    u32 ext_modulus(u32 level, u32 e) const { return e <= level ? e : num_q + (e - level - 1); }
    // ModUp table of one digit: inv[alpha_pad], inv_sh[alpha_pad], conv[M][alpha_pad], negq[M] (conv and negq
    // indexed by the position e in the extended basis of that level; negq = -Q_j mod t).  The alpha
    // constants of one target limb are adjacent so that a wavefront fetches them with one wide scalar load.
    // Rows are padded to alpha_pad / k_pad entries (4, 8 or 16; zeros beyond the real ones).
    u32 alpha_pad, k_pad, k2_pad;  // k2_pad: padded num_p + 1
    // rounded up to 16 words so that every level's rows keep the 128-byte alignment the wide scalar loads assume
    size_t moddown_rs_stride() const { return (2 * (size_t)k2_pad + (size_t)k2_pad * num_q + 3 * num_q + 15) / 16 * 16; }
    const u64* moddown_rs_table(u32 level) const { return d_moddown_rs + level * moddown_rs_stride(); }
    size_t modup_negq_off() const { return (size_t)alpha_pad * (2 + M); }
    size_t modup_digit_stride() const { return modup_negq_off() + ((M + 15) / 16) * 16; }
    size_t modup_level_stride() const { return modup_digit_stride() * dnum; }
    const u64* modup_table(u32 level, u32 j) const { return d_modup + level * modup_level_stride() + j * modup_digit_stride(); }
};

// Records a (start, stop) event pair around one kernel launch while profiling is on.
struct ProfScope {
    const ckks_ctx* c;
    hipStream_t st;
    long pair;
    // bytes: what the launch must read and write at least once; ops: its modular multiplications
    ProfScope(const ckks_ctx* ctx, int kernel, hipStream_t s, double bytes, double ops) : c(ctx), st(s), pair(-1) {
        ProfState* p = c->prof;
        if (!p || !((p->mask >> kernel) & 1u)) return;
        if (2 * (p->used_pairs + 1) > p->events.size()) { p->dropped++; return; }
        pair = (long)p->used_pairs++;
        p->kernel_of_pair[pair] = kernel;
        p->bytes[kernel] += bytes;
        p->ops[kernel] += ops;
        (void)hipEventRecord(p->events[2 * pair], st);
    }
    ~ProfScope() {
        if (pair >= 0) (void)hipEventRecord(c->prof->events[2 * pair + 1], st);
    }
};

// noalloc.hip: the device address of the library's built-in scratch array on the current device (looked up on first use)
hipError_t noalloc_scratch_current_device(int* device, void** ptr);

// ---- kernel launchers (each enqueues on `st` and returns the launch status) -------------------
// ntt.hip: batch x pl.n limb-polys; item b reads src + b*src_bstride*N (or src_ptrs[b] when given: host
// array of `batch` <= KS_MAX_BATCH device pointers) and writes dst + b*dst_bstride*N
hipError_t launch_ntt(const ckks_ctx* c, bool inverse, const u64* src, size_t src_bstride, u64* dst,
                      size_t dst_bstride, const PolyList& pl, u32 batch, hipStream_t st, const u64* const* src_ptrs = nullptr,
                      const FwdEpilogue* epilogue = nullptr, const TwF* inv_scale = nullptr, const u64* const* mul_ptrs = nullptr,
                      const u64* lin_k = nullptr);
// mul_ptrs (inverse, with src_ptrs, double-precision arithmetic): batch item b is src_ptrs[b] (.) mul_ptrs[b], formed on load;
// with lin_k = {ka, kb} (one limb only) it is ka * src_ptrs[b] + kb * mul_ptrs[b] instead.
// ModUp fused into transforms (contexts with ntt_f64 and the two-pass transform): the inverse transform of the polynomial
// scales the limb with modulus index m by inv_scale[m] instead of 1/N and stores the CENTRED residue as a double (launch_ntt with inv_scale);
// launch_ntt_modup then evaluates the basis conversion of digit j, y [batch][level+1][N] doubles -> the pl.n target limbs
// pl.dpos[] of dst (batch stride dst_bstride limb-polys), inside the first pass of their forward transforms.
inline bool ntt_has_modup(const ckks_ctx* c) { return c->ntt_f64 && c->log_n > CKKS_TILE_LOG && c->d_modup_prep_f != nullptr; }
// The same for ModDown's conversion: y are the 2*batch extended polynomials ([E][N] each, the dropped limbs left as scaled
// centred doubles by launch_ntt with the moddown prep table), dst the converted dropped part ([n_out][N] per polynomial,
// NTT form), epilogue what the second pass does with it.  merged: the dropped set is {q_level, p_0..p_{k-1}}.
hipError_t launch_ntt_moddown(const ckks_ctx* c, u32 level, bool merged, const double* y, u64* dst, u32 batch, hipStream_t st,
                              const FwdEpilogue* epilogue);
// The same for the rescale: y [batch][N] is the dropped limb `level` of every component (centred doubles, from launch_ntt
// with d_rescale_prep_f), dst [batch][level][N] scratch, epilogue the subtraction and the multiplication by q_level^-1.
hipError_t launch_ntt_rescale(const ckks_ctx* c, u32 level, const double* y, u64* dst, u32 batch, hipStream_t st,
                              const FwdEpilogue* epilogue);
// hi_only: stop after the converting hi pass; launch_ntt_lo_mac then runs the lo passes of all digits and multiplies the
// results by the switching keys (keys[b]: [dnum][2][M][N], one per batch item) as they come out, adding P * add0s[b] /
// add1s[b] (optional, [level+1][N]) on the q-limbs: outs[b] [2][E][N] is the finished inner product on the extended basis.
hipError_t launch_ntt_modup(const ckks_ctx* c, u32 level, u32 j, const double* y, size_t y_bstride, u64* dst, size_t dst_bstride,
                            const PolyList& pl, u32 batch, hipStream_t st, bool hi_only = false);
// prod: the decomposed polynomial is the d2 = a1 (.) b1 of n ciphertext products and was never stored (the inverse
// transform took it as a product, launch_ntt with mul_ptrs): the term of the digits' own limbs and the addends
// d0 = a0 (.) b0, d1 = a0 (.) b1 + a1 (.) b0 are formed from the operands (host arrays of n device pointers,
// [level+1][N] each).
// lin (optional): the product's addend is the linear combination ka * x + kb * y of two more ciphertexts (component
// strides x_cstride, y_cstride; ka, kb: one residue per q-limb), formed on the fly as well.
struct MacProduct {
    const u64* const* a0;
    const u64* const* a1;
    const u64* const* b0;
    const u64* const* b1;
    const u64* const* lin_x = nullptr;
    const u64* const* lin_y = nullptr;
    size_t x_cstride = 0, y_cstride = 0;
    const u64* ka = nullptr;
    const u64* kb = nullptr;
};
hipError_t launch_ntt_lo_mac(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* const* keys, u64* const* outs, u32 n,
                             hipStream_t st, const MacProduct* prod = nullptr);
// whether launch_ntt can apply an epilogue in this ring (it needs the two-pass transform)
inline bool ntt_has_epilogue(const ckks_ctx* c) { return c->log_n > CKKS_TILE_LOG; }
// keyswitch.hip
hipError_t launch_modup_conv(const ckks_ctx* c, u32 level, u32 j, const u64* y, size_t y_bstride, const PtrList8& c_in, u64* digit,
                             size_t digit_bstride, u32 n, hipStream_t st);
hipError_t launch_key_inner(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g, u64* v, hipStream_t st);
hipError_t launch_key_inner_multi(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g,
                                  u64* v, size_t v_bstride, u32 n, hipStream_t st);
// add0s / add1s: per item, polynomials [level+1][N] whose P-fold is added to component 0 / 1 (either list, or entries, may be null)
hipError_t launch_key_inner_ext(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* key, u32 g,
                                const u64* const* add0s, const u64* const* add1s, const u64* mask, u64* const* outs, u32 n,
                                hipStream_t st);
// result of (item b, tap i) = term k0 + b*k_bstride + taps[i] of `xs` in layout xl; c0s[b] = the whole ciphertext
// [2][level+1][N]; centre_mask (optional, [E][N]): the tap without a rotation, written as term centre_tap
hipError_t launch_key_inner_taps(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* const* keys,
                                 const u32* gs, const u64* const* masks, const u32* taps, u32 n_taps, const u64* const* c0s,
                                 u64* xs, XLayout xl, u32 k0, u32 k_bstride, u32 n, u64* scratch, bool prepare, hipStream_t st,
                                 const u64* centre_mask = nullptr, u32 centre_tap = 0, bool direct_keys = false);
size_t key_inner_taps_scratch_elems(const ckks_ctx* c, u32 level, u32 n_taps);
// merged: the dropped limbs are q_level and the special primes (division by P*q_level, results on limbs 0..level-1)
hipError_t launch_moddown_conv(const ckks_ctx* c, u32 level, bool merged, const u64* v, u64* w, u32 batch, hipStream_t st);
hipError_t launch_moddown_final(const ckks_ctx* c, u32 level, bool merged, const u64* v, const u64* w, const FinalItem* items, u32 n,
                                hipStream_t st);
// pointwise.hip
hipError_t launch_automorph(const ckks_ctx* c, u32 n_polys, const u64* in, u32 g, u64* out, hipStream_t st);
hipError_t launch_copy(const u64* in, u64* out, size_t n, hipStream_t st);
hipError_t launch_ptct_mac(const ckks_ctx* c, u32 level, const u64* const* pts, const u64* const* cts, u32 n_terms, u64* acc,
                           int accumulate, hipStream_t st, bool extended = false);
hipError_t launch_relayout_mac(const ckks_ctx* c, u32 level, bool extended, const u64* xs, const u64* const* masks, u64* acc, u32 n,
                               u32 n_lo, u32 n_hi, hipStream_t st);
hipError_t launch_scale_p_ext(const ckks_ctx* c, u32 level, const u64* ct, u64* out, hipStream_t st);
hipError_t launch_rescale_conv(const ckks_ctx* c, u32 level, const u64* r, u64* w, u32 batch, hipStream_t st);
hipError_t launch_rescale_final(const ckks_ctx* c, u32 level, const PtrList8& ct, size_t ct_cstride, const u64* w, const OutList8& out,
                                u32 n, hipStream_t st);
hipError_t launch_tensor(const ckks_ctx* c, u32 level, const PtrList8& a, size_t a_cstride, const PtrList8& b, size_t b_cstride,
                         u64* d0, u64* d1, u64* d2, u32 n, const u64* add, size_t add_bstride, hipStream_t st);
hipError_t launch_mask_mul(const ckks_ctx* c, u32 level, const u64* mask, const u64* ct, u64* out, hipStream_t st);
hipError_t launch_key_expand_a(const ckks_ctx* c, u64 seed, u64* key, hipStream_t st);
hipError_t launch_add_plain(const ckks_ctx* c, u32 level, const u64* pt, u64* ct, hipStream_t st);
hipError_t launch_ct_sum(const ckks_ctx* c, u32 level, const PtrList8& items, u32 n, u64* out, hipStream_t st, bool extended = false);
hipError_t launch_centre_ext(const ckks_ctx* c, u32 level, const u64* mask, const u64* ct, u64* xs, XLayout xl, u32 k, hipStream_t st);
hipError_t launch_weight_check(const ckks_ctx* c, u32 level, bool extended, const u64* w_res, size_t n_w, u32 weight_bits, u32* d_count,
                               hipStream_t st);
size_t weighted_sum_scratch_elems(const ckks_ctx* c, u32 n_limbs, u32 n_terms, u32 c_out);
// weight_bits: the caller's bound |w| < 2^(weight_bits - 1) on the integers behind w_res (0 = none)
hipError_t launch_weighted_sum(const ckks_ctx* c, u32 level, bool extended, const u64* xs, XLayout xl, u32 n_terms, const u64* w_res,
                               u32 c_out, u64* acc, u64* scratch, u32 weight_bits, hipStream_t st);
// wsum_mfma.hip
bool wsum_mfma_applies(const ckks_ctx* c, u32 n_terms);
size_t wsum_mfma_scratch_elems(u32 n_limbs, u32 n_terms, u32 c_out);
hipError_t launch_wsum_mfma(const ckks_ctx* c, u32 level, u32 nl, const u64* xs, XLayout xl, u32 n_terms, const u64* w_res, u32 c_out,
                            u64* acc, u64* scratch, u32 weight_bits, hipStream_t st);
hipError_t launch_lincomb2(const ckks_ctx* c, u32 level, const PtrList8& a, size_t a_cstride, const u64* ka, const PtrList8& b,
                           size_t b_cstride, const u64* kb, const u64* add, size_t add_bstride, u64* out, size_t out_bstride, u32 n,
                           hipStream_t st);
