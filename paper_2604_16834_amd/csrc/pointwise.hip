// Pointwise (per evaluation point) kernels on limb-major ciphertexts for gfx950: automorphism
// gather, plaintext-ciphertext multiply-accumulate (Methodology, "Convolution Evaluation", Eq. 11
// and the rotation-free channel sum), the two elementwise steps of rescaling, the tensor product
// of a ciphertext multiplication and small linear combinations for the polynomial activation
// ("Other Layers").  All of them stream HBM once; coefficients x are the fastest index so every
// wavefront touches contiguous 512-byte runs.
#include "ctx.h"
#include "galois.h"

#define PW_THREADS 256

// out[p][k] = in[p][pi_g(k)] for n_polys limb-polys (the same gather for every modulus)
__global__ __launch_bounds__(PW_THREADS) void automorph_kernel(const u64* __restrict__ in, u64* __restrict__ out, u32 log_n, u32 g) {
    const u32 N = 1u << log_n;
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const size_t base = (size_t)blockIdx.y * N;
    out[base + x] = in[base + galois_gather_index(x, g, log_n)];
}

hipError_t launch_automorph(const ckks_ctx* c, u32 n_polys, const u64* in, u32 g, u64* out, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, n_polys);
    { ProfScope ps__(c, K_AUTOMORPH, st, 16.0 * c->N * n_polys, 0.0); hipLaunchKernelGGL(automorph_kernel, grid, dim3(PW_THREADS), 0, st, in, out, c->log_n, g); }
    return hipGetLastError();
}

__global__ __launch_bounds__(PW_THREADS) void copy_kernel(const u64* __restrict__ in, u64* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * PW_THREADS;
    for (; i < n; i += stride) out[i] = in[i];
}

hipError_t launch_copy(const u64* in, u64* out, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + PW_THREADS - 1) / PW_THREADS;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(copy_kernel, dim3((u32)blocks), dim3(PW_THREADS), 0, st, in, out, n);
    return hipGetLastError();
}

// ---- plaintext x ciphertext multiply-accumulate -------------------------------------------------
#define MAC_TERMS_PER_LAUNCH 16
struct MacTerms {
    const u64* pt[MAC_TERMS_PER_LAUNCH];
    const u64* ct[MAC_TERMS_PER_LAUNCH];
    u32 n;
};

// limbs = level+1 (ciphertext limbs) or level+1+k (extended basis Q_level P: positions above `level` are the special primes)
__global__ __launch_bounds__(PW_THREADS) void ptct_mac_kernel(MacTerms T, u64* __restrict__ acc, const ModConst* __restrict__ mc,
                                                              u32 N, u32 level, u32 limbs, u32 num_q, int accumulate) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, comp = blockIdx.z;
    const ModConst m = mc[i <= level ? i : num_q + (i - level - 1)];
    const size_t po = (size_t)i * N + x, co = ((size_t)comp * limbs + i) * N + x;
    U128 s = {0, 0};
    if (accumulate) s.lo = acc[co];
    for (u32 k = 0; k < T.n; k++) acc_wide(s, T.pt[k][po], T.ct[k][co]);
    acc[co] = barrett_reduce(s, m);
}

hipError_t launch_ptct_mac(const ckks_ctx* c, u32 level, const u64* const* pts, const u64* const* cts, u32 n_terms, u64* acc,
                           int accumulate, hipStream_t st, bool extended) {
    const u32 limbs = extended ? c->ext_limbs(level) : level + 1;
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, limbs, 2);
    for (u32 k0 = 0; k0 < n_terms; k0 += MAC_TERMS_PER_LAUNCH) {
        MacTerms T;
        T.n = n_terms - k0 < MAC_TERMS_PER_LAUNCH ? n_terms - k0 : MAC_TERMS_PER_LAUNCH;
        for (u32 k = 0; k < MAC_TERMS_PER_LAUNCH; k++) {
            T.pt[k] = k < T.n ? pts[k0 + k] : nullptr;
            T.ct[k] = k < T.n ? cts[k0 + k] : nullptr;
        }
        ProfScope ps__(c, K_PTCT_MAC, st, 8.0 * c->N * limbs * (3.0 * T.n + 2.0 + ((accumulate || k0 > 0) ? 2.0 : 0.0)), 2.0 * c->N * limbs * T.n);
        hipLaunchKernelGGL(ptct_mac_kernel, grid, dim3(PW_THREADS), 0, st, T, acc, c->d_mc, c->N, level, limbs, c->num_q, accumulate || k0 > 0);
    }
    return hipGetLastError();
}

// ---- the masked sums of a re-layout, all of them in one pass over the rotated copies --------------------------
//   acc[b][h] = sum_l mask[h][l] (.) x[b][l]      b < n ciphertexts, h < n_hi, l < n_lo
// x[b][l] = xs + (b*n_lo + l)*stride, acc[b][h] = acc + (b*n_hi + h)*stride, each [2][limbs][N].  A thread owns one
// (coefficient, limb) of RL_CB ciphertexts and keeps the sums of up to RL_NH values of h, so every rotated copy is
// read once per group of RL_NH sums (a launch per (h, l) pair list read it once per sum) and every mask word once per
// RL_CB ciphertexts.  Absent pairs are null pointers.
#define RL_NH 4
#define RL_CB 4
#define RL_NL 32
struct RelayoutMasks {
    const u64* m[RL_NH][RL_NL];
};

__global__ __launch_bounds__(PW_THREADS) void relayout_mac_kernel(const u64* __restrict__ xs, RelayoutMasks M, u64* __restrict__ acc,
                                                                  const ModConst* __restrict__ mc, u32 N, u32 level, u32 limbs, u32 num_q,
                                                                  size_t stride, u32 n, u32 n_lo, u32 n_hi, u32 l0, u32 nl, u32 h0,
                                                                  u32 nh, int accumulate) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, b0 = blockIdx.z * RL_CB;
    const ModConst m = mc[i <= level ? i : num_q + (i - level - 1)];
    const size_t po = (size_t)i * N + x;
    U128 s[RL_NH][RL_CB][2];
#pragma unroll
    for (u32 h = 0; h < RL_NH; h++)
#pragma unroll
        for (u32 b = 0; b < RL_CB; b++)
#pragma unroll
            for (u32 comp = 0; comp < 2; comp++) {
                s[h][b][comp] = {0, 0};
                if (accumulate && h < nh && b0 + b < n)
                    s[h][b][comp].lo = acc[((size_t)(b0 + b) * n_hi + h0 + h) * stride + ((size_t)comp * limbs + i) * N + x];
            }
    for (u32 l = 0; l < nl; l++) {
        u64 xv[RL_CB][2];
#pragma unroll
        for (u32 b = 0; b < RL_CB; b++)
#pragma unroll
            for (u32 comp = 0; comp < 2; comp++)
                xv[b][comp] = b0 + b < n ? xs[((size_t)(b0 + b) * n_lo + l0 + l) * stride + ((size_t)comp * limbs + i) * N + x] : 0;
#pragma unroll
        for (u32 h = 0; h < RL_NH; h++) {
            const u64* mp = M.m[h][l];
            if (h >= nh || !mp) continue;  // uniform over the workgroup
            const u64 mv = mp[po];
#pragma unroll
            for (u32 b = 0; b < RL_CB; b++)
#pragma unroll
                for (u32 comp = 0; comp < 2; comp++) acc_wide(s[h][b][comp], mv, xv[b][comp]);
        }
    }
#pragma unroll
    for (u32 h = 0; h < RL_NH; h++)
#pragma unroll
        for (u32 b = 0; b < RL_CB; b++)
#pragma unroll
            for (u32 comp = 0; comp < 2; comp++)
                if (h < nh && b0 + b < n)
                    acc[((size_t)(b0 + b) * n_hi + h0 + h) * stride + ((size_t)comp * limbs + i) * N + x] = barrett_reduce(s[h][b][comp], m);
}

// masks: host array of n_hi*n_lo device pointers ([limbs][N] each, or null)
hipError_t launch_relayout_mac(const ckks_ctx* c, u32 level, bool extended, const u64* xs, const u64* const* masks, u64* acc, u32 n,
                               u32 n_lo, u32 n_hi, hipStream_t st) {
    const u32 limbs = extended ? c->ext_limbs(level) : level + 1;
    const size_t stride = 2 * (size_t)limbs * c->N;
    const u32 nl_max = c->lazy_terms < RL_NL ? (c->lazy_terms ? c->lazy_terms : 1) : RL_NL;  // products summed before a reduction
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, limbs, (n + RL_CB - 1) / RL_CB);
    for (u32 h0 = 0; h0 < n_hi; h0 += RL_NH) {
        const u32 nh = n_hi - h0 < RL_NH ? n_hi - h0 : RL_NH;
        for (u32 l0 = 0; l0 < n_lo; l0 += nl_max) {
            const u32 nl = n_lo - l0 < nl_max ? n_lo - l0 : nl_max;
            RelayoutMasks M;
            double n_masks = 0.0;
            for (u32 h = 0; h < RL_NH; h++)
                for (u32 l = 0; l < RL_NL; l++) {
                    M.m[h][l] = (h < nh && l < nl) ? masks[(size_t)(h0 + h) * n_lo + l0 + l] : nullptr;
                    n_masks += M.m[h][l] ? 1.0 : 0.0;
                }
            ProfScope ps__(c, K_PTCT_MAC, st, 8.0 * c->N * limbs * (2.0 * n * nl + n_masks * ((n + RL_CB - 1) / RL_CB) + 2.0 * n * nh * (l0 ? 2.0 : 1.0)),
                           2.0 * c->N * limbs * n * n_masks);
            hipLaunchKernelGGL(relayout_mac_kernel, grid, dim3(PW_THREADS), 0, st, xs, M, acc, c->d_mc, c->N, level, limbs, c->num_q, stride, n,
                               n_lo, n_hi, l0, nl, h0, nh, l0 > 0 ? 1 : 0);
        }
    }
    return hipGetLastError();
}

// ---- rescale (batched over ciphertext components) -----------------------------------------------
// r [batch][N]: dropped limbs in coefficient form.  w[b][i][x] = centred r[b][x] mod q_i.
__global__ __launch_bounds__(PW_THREADS) void rescale_conv_kernel(const u64* __restrict__ r, u64* __restrict__ w,
                                                                  const u64* __restrict__ tab, const ModConst* __restrict__ mc,
                                                                  u32 N, u32 level, u32 num_q) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, b = blockIdx.z;
    const ModConst m = mc[i];
    const u64 ql = mc[level].q;
    const u64 rv = r[(size_t)b * N + x];
    u64 v = reduce_word(rv, m);
    if (rv > ql / 2) v = sub_mod(v, tab[((size_t)level * num_q + i) * 3 + 2], m.q);  // r - q_l
    w[((size_t)b * level + i) * N + x] = v;
}

hipError_t launch_rescale_conv(const ckks_ctx* c, u32 level, const u64* r, u64* w, u32 batch, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level, batch);
    ProfScope ps__(c, K_RESCALE_CONV, st, 8.0 * batch * c->N * (1.0 + level), 0.0);
    hipLaunchKernelGGL(rescale_conv_kernel, grid, dim3(PW_THREADS), 0, st, r, w, c->d_rescale, c->d_mc, c->N, level, c->num_q);
    return hipGetLastError();
}

// out_b[comp][i] = (ct_b[comp][i] - w[2b+comp][i]) * q_l^-1, i < level; ct_b = ct.p[b] with component stride ct_cstride
__global__ __launch_bounds__(PW_THREADS) void rescale_final_kernel(PtrList8 ct, size_t ct_cstride, const u64* __restrict__ w,
                                                                   OutList8 out, const u64* __restrict__ tab,
                                                                   const ModConst* __restrict__ mc, u32 N, u32 level, u32 num_q) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, z = blockIdx.z, b = z >> 1, comp = z & 1;
    const u64 q = mc[i].q;
    const u64* t = tab + ((size_t)level * num_q + i) * 3;
    u64 d = sub_mod(ct.p[b][comp * ct_cstride + (size_t)i * N + x], w[((size_t)z * level + i) * N + x], q);
    out.p[b][((size_t)comp * level + i) * N + x] = mul_shoup(d, t[0], t[1], q);
}

hipError_t launch_rescale_final(const ckks_ctx* c, u32 level, const PtrList8& ct, size_t ct_cstride, const u64* w, const OutList8& out,
                                u32 n, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level, 2 * n);
    ProfScope ps__(c, K_RESCALE_FINAL, st, 48.0 * n * c->N * level, 2.0 * n * c->N * level);
    hipLaunchKernelGGL(rescale_final_kernel, grid, dim3(PW_THREADS), 0, st, ct, ct_cstride, w, out, c->d_rescale, c->d_mc, c->N, level,
                       c->num_q);
    return hipGetLastError();
}

// ---- tensor product of ciphertext pairs -----------------------------------------------------------
// item b: d0 = a0 b0 (+ add0), d1 = a0 b1 + a1 b0 (+ add1), d2 = a1 b1 on limbs 0..level; operands a.p[b], b.p[b] may sit
// at a higher level (component strides in elements); d0/d1/d2 are [n][level+1][N]; add (optional): item z at
// add + z*add_bstride, [2][level+1][N]
__global__ __launch_bounds__(PW_THREADS) void tensor_kernel(PtrList8 a, size_t a_cstride, PtrList8 b, size_t b_cstride,
                                                            u64* __restrict__ d0, u64* __restrict__ d1, u64* __restrict__ d2,
                                                            const u64* __restrict__ add, size_t add_bstride,
                                                            const ModConst* __restrict__ mc, u32 N, u32 level) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, z = blockIdx.z;
    const ModConst m = mc[i];
    const size_t o = (size_t)i * N + x;
    const u64* pa = a.p[z];
    const u64* pb = b.p[z];
    const u64 a0 = pa[o], a1 = pa[a_cstride + o], b0 = pb[o], b1 = pb[b_cstride + o];
    const size_t oo = ((size_t)z * (level + 1) + i) * N + x;
    u64 r0 = mulmod_barrett(a0, b0, m);
    U128 s = mul_wide(a0, b1);
    acc_wide(s, a1, b0);
    u64 r1 = barrett_reduce(s, m);
    if (add) {
        const u64* ad = add + z * add_bstride;
        r0 = add_mod(r0, ad[o], m.q);
        r1 = add_mod(r1, ad[(size_t)(level + 1) * N + o], m.q);
    }
    d0[oo] = r0;
    d1[oo] = r1;
    d2[oo] = mulmod_barrett(a1, b1, m);
}

hipError_t launch_tensor(const ckks_ctx* c, u32 level, const PtrList8& a, size_t a_cstride, const PtrList8& b, size_t b_cstride,
                         u64* d0, u64* d1, u64* d2, u32 n, const u64* add, size_t add_bstride, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level + 1, n);
    ProfScope ps__(c, K_TENSOR, st, (56.0 + (add ? 16.0 : 0.0)) * n * c->N * (level + 1.0), 4.0 * n * c->N * (level + 1.0));
    hipLaunchKernelGGL(tensor_kernel, grid, dim3(PW_THREADS), 0, st, a, a_cstride, b, b_cstride, d0, d1, d2, add, add_bstride, c->d_mc,
                       c->N, level);
    return hipGetLastError();
}

// ---- convolution operands -----------------------------------------------------------------------
// out[comp][i] = mask[i] * ct[comp][i]: an aligned ciphertext times the tap's encoded validity mask
__global__ __launch_bounds__(PW_THREADS) void mask_mul_kernel(const u64* __restrict__ mask, const u64* __restrict__ ct,
                                                              u64* __restrict__ out, const ModConst* __restrict__ mc, u32 N, u32 level) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, comp = blockIdx.z;
    const size_t co = ((size_t)comp * (level + 1) + i) * N + x;
    out[co] = mulmod_barrett(mask[(size_t)i * N + x], ct[co], mc[i]);
}

hipError_t launch_mask_mul(const ckks_ctx* c, u32 level, const u64* mask, const u64* ct, u64* out, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level + 1, 2);
    { ProfScope ps__(c, K_MASK_MUL, st, 40.0 * c->N * (level + 1.0), 2.0 * c->N * (level + 1.0)); hipLaunchKernelGGL(mask_mul_kernel, grid, dim3(PW_THREADS), 0, st, mask, ct, out, c->d_mc, c->N, level); }
    return hipGetLastError();
}

// The centre tap of a convolution that divides by P after its sum: out[comp][e] = mask[e] * [P]_{q_e} * ct[comp][e]
// on the live q-limbs, zero on the special primes (result = term k of xs in layout xl, mask [E][N], ct [2][level+1][N]).
__global__ __launch_bounds__(PW_THREADS) void centre_ext_kernel(const u64* __restrict__ mask, const u64* __restrict__ ct,
                                                                u64* __restrict__ xs, XLayout xl, u32 k, const u64* __restrict__ negp,
                                                                const ModConst* __restrict__ mc, u32 N, u32 level, u32 E) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y, comp = blockIdx.z;
    u64 r = 0;
    if (e <= level) {
        const ModConst m = mc[e];
        const u64 pm = mulmod_barrett(m.q - negp[e], mask[(size_t)e * N + x], m);
        r = mulmod_barrett(pm, ct[((size_t)comp * (level + 1) + e) * N + x], m);
    }
    xs[xl.at(k, comp, e, x)] = r;
}

hipError_t launch_centre_ext(const ckks_ctx* c, u32 level, const u64* mask, const u64* ct, u64* xs, XLayout xl, u32 k, hipStream_t st) {
    const u32 E = c->ext_limbs(level);
    const u64* negp = c->d_moddown + 2 * c->k_pad + (size_t)c->k_pad * c->num_q + 2 * c->num_q;
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, E, 2);
    ProfScope ps__(c, K_MASK_MUL, st, 8.0 * c->N * (3.0 * (level + 1.0) + 2.0 * E), 4.0 * c->N * (level + 1.0));
    hipLaunchKernelGGL(centre_ext_kernel, grid, dim3(PW_THREADS), 0, st, mask, ct, xs, xl, k, negp, c->d_mc, c->N, level, E);
    return hipGetLastError();
}

// acc[o][comp][i][x] = sum_k w_res[o][k][i] * xs[k][comp][i][x]  mod q_i: the sum over (input
// channel, tap) of Eq. 11 with the integer weight factored out of the plaintext.  This is the kernel
// for moduli above 2^50 (the matrix-core kernel in wsum_mfma.hip takes the others): each thread keeps
// WS_OUT_TILE output channels' 128-bit sums so that every xs element is loaded once per tile.
#define WS_OUT_TILE 4
__global__ __launch_bounds__(PW_THREADS) void weighted_sum_kernel(const u64* __restrict__ xs, XLayout xl, const u64* __restrict__ w_res,
                                                                  u64* __restrict__ acc, const ModConst* __restrict__ mc, u32 N,
                                                                  u32 level, u32 L1, u32 num_q, u32 n_terms, u32 c_out, u32 lazy_terms) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y % L1, comp = blockIdx.y / L1;
    const u32 o0 = blockIdx.z * WS_OUT_TILE;
    const ModConst m = mc[i <= level ? i : num_q + (i - level - 1)];
    const size_t ct_stride = (size_t)2 * L1 * N;
    const size_t off = ((size_t)comp * L1 + i) * N + x;
    U128 s[WS_OUT_TILE];
#pragma unroll
    for (u32 t = 0; t < WS_OUT_TILE; t++) s[t] = {0, 0};
    u32 pending = 0;
    for (u32 k = 0; k < n_terms; k++) {
        const u64 v = xs[xl.at(k, comp, i, x)];
#pragma unroll
        for (u32 t = 0; t < WS_OUT_TILE; t++)
            if (o0 + t < c_out) acc_wide(s[t], v, w_res[((size_t)(o0 + t) * n_terms + k) * L1 + i]);
        if (++pending == lazy_terms) {
            pending = 0;
#pragma unroll
            for (u32 t = 0; t < WS_OUT_TILE; t++) { s[t].lo = barrett_reduce(s[t], m); s[t].hi = 0; }
        }
    }
#pragma unroll
    for (u32 t = 0; t < WS_OUT_TILE; t++)
        if (o0 + t < c_out) acc[(o0 + t) * ct_stride + off] = barrett_reduce(s[t], m);
}

size_t weighted_sum_scratch_elems(const ckks_ctx* c, u32 n_limbs, u32 n_terms, u32 c_out) {
    if (wsum_mfma_applies(c, n_terms)) return wsum_mfma_scratch_elems(n_limbs, n_terms, c_out);
    return 0;
}

// xs: n_terms operands in layout xl, w_res [c_out][n_terms][nl], acc [c_out][2][nl][N]; nl = level+1 (the live q-limbs) or,
// with `extended`, level+1+num_p (the extended basis: positions above `level` are the special primes).
// scratch: weighted_sum_scratch_elems() words (may be null when that is 0)
hipError_t launch_weighted_sum(const ckks_ctx* c, u32 level, bool extended, const u64* xs, XLayout xl, u32 n_terms, const u64* w_res,
                               u32 c_out, u64* acc, u64* scratch, u32 weight_bits, hipStream_t st) {
    const u32 L1 = extended ? c->ext_limbs(level) : level + 1;
    const double bytes = 16.0 * c->N * L1 * ((double)n_terms + c_out), ops = 2.0 * c->N * L1 * n_terms * c_out;
    if (wsum_mfma_applies(c, n_terms)) {  // moduli below 2^50: exact 8-bit digit products on the matrix cores
        ProfScope ps__(c, K_WEIGHTED_SUM, st, bytes, ops);
        return launch_wsum_mfma(c, level, L1, xs, xl, n_terms, w_res, c_out, acc, scratch, weight_bits, st);
    }
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, 2 * L1, (c_out + WS_OUT_TILE - 1) / WS_OUT_TILE);
    ProfScope ps__(c, K_WEIGHTED_SUM, st, bytes, ops);
    hipLaunchKernelGGL(weighted_sum_kernel, grid, dim3(PW_THREADS), 0, st, xs, xl, w_res, acc, c->d_mc, c->N, level, L1, c->num_q, n_terms,
                       c_out, c->lazy_terms);
    return hipGetLastError();
}

// ---- out = sum of n <= KS_MAX_BATCH ciphertexts [2][level+1][N] (the accumulator's additions) ----------
__global__ __launch_bounds__(PW_THREADS) void ct_sum_kernel(PtrList8 items, u32 n, u64* out,  // out may be one of the items
                                                            const ModConst* __restrict__ mc, u32 N, u32 level, u32 limbs, u32 num_q) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, comp = blockIdx.z;
    const u64 q = mc[i <= level ? i : num_q + (i - level - 1)].q;
    const size_t o = ((size_t)comp * limbs + i) * N + x;
    u64 s = items.p[0][o];
    for (u32 b = 1; b < n; b++) s = add_mod(s, items.p[b][o], q);
    out[o] = s;
}

// extended: the items are [2][level+1+k][N] on the basis Q_level P
hipError_t launch_ct_sum(const ckks_ctx* c, u32 level, const PtrList8& items, u32 n, u64* out, hipStream_t st, bool extended) {
    const u32 limbs = extended ? c->ext_limbs(level) : level + 1;
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, limbs, 2);
    ProfScope ps__(c, K_LINCOMB2, st, 16.0 * c->N * limbs * (n + 1.0), 0.0);
    hipLaunchKernelGGL(ct_sum_kernel, grid, dim3(PW_THREADS), 0, st, items, n, out, c->d_mc, c->N, level, limbs, c->num_q);
    return hipGetLastError();
}

// ---- out = P * ct on the extended basis Q_level P (zero on the special primes): a ciphertext that joins a sum
// which is divided by P afterwards
__global__ __launch_bounds__(PW_THREADS) void scale_p_ext_kernel(const u64* __restrict__ ct, u64* __restrict__ out,
                                                                 const u64* __restrict__ negp, const ModConst* __restrict__ mc, u32 N,
                                                                 u32 level, u32 E) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 e = blockIdx.y, comp = blockIdx.z;
    u64 r = 0;
    if (e <= level) {
        const ModConst m = mc[e];
        r = mulmod_barrett(m.q - negp[e], ct[((size_t)comp * (level + 1) + e) * N + x], m);
    }
    out[((size_t)comp * E + e) * N + x] = r;
}

hipError_t launch_scale_p_ext(const ckks_ctx* c, u32 level, const u64* ct, u64* out, hipStream_t st) {
    const u32 E = c->ext_limbs(level);
    const u64* negp = c->d_moddown + 2 * c->k_pad + (size_t)c->k_pad * c->num_q + 2 * c->num_q;
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, E, 2);
    ProfScope ps__(c, K_MASK_MUL, st, 8.0 * c->N * (2.0 * (level + 1.0) + 2.0 * E), 2.0 * c->N * (level + 1.0));
    hipLaunchKernelGGL(scale_p_ext_kernel, grid, dim3(PW_THREADS), 0, st, ct, out, negp, c->d_mc, c->N, level, E);
    return hipGetLastError();
}

// ---- ct[0][i] += pt[i] on limbs 0..level (a plaintext, e.g. the replicated bias of the FC layer) -----------
__global__ __launch_bounds__(PW_THREADS) void add_plain_kernel(const u64* __restrict__ pt, u64* __restrict__ ct,
                                                               const ModConst* __restrict__ mc, u32 N) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y;
    const size_t o = (size_t)i * N + x;
    ct[o] = add_mod(ct[o], pt[o], mc[i].q);
}

hipError_t launch_add_plain(const ckks_ctx* c, u32 level, const u64* pt, u64* ct, hipStream_t st) {
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level + 1);
    hipLaunchKernelGGL(add_plain_kernel, grid, dim3(PW_THREADS), 0, st, pt, ct, c->d_mc, c->N);
    return hipGetLastError();
}

// ---- out_b = ka * a_b + kb * b_b (+ add_b) on limbs 0..level, integer scalars given by residues ----
struct Scalars {
    u64 ka[CKKS_MAX_MODULI];
    u64 kb[CKKS_MAX_MODULI];
};

__global__ __launch_bounds__(PW_THREADS) void lincomb2_kernel(PtrList8 a, size_t a_cstride, PtrList8 b, size_t b_cstride,
                                                              const u64* __restrict__ add, size_t add_bstride, Scalars K,
                                                              u64* __restrict__ out, size_t out_bstride,
                                                              const ModConst* __restrict__ mc, u32 N, u32 level) {
    const u32 x = blockIdx.x * PW_THREADS + threadIdx.x;
    if (x >= N) return;
    const u32 i = blockIdx.y, z = blockIdx.z, bi = z >> 1, comp = z & 1;
    const ModConst m = mc[i];
    const size_t o = (size_t)i * N + x;
    U128 s = mul_wide(a.p[bi][comp * a_cstride + o], K.ka[i]);
    acc_wide(s, b.p[bi][comp * b_cstride + o], K.kb[i]);
    const size_t oo = ((size_t)comp * (level + 1) + i) * N + x;
    u64 r = barrett_reduce(s, m);
    if (add) r = add_mod(r, add[bi * add_bstride + oo], m.q);
    out[bi * out_bstride + oo] = r;
}

hipError_t launch_lincomb2(const ckks_ctx* c, u32 level, const PtrList8& a, size_t a_cstride, const u64* ka, const PtrList8& b,
                           size_t b_cstride, const u64* kb, const u64* add, size_t add_bstride, u64* out, size_t out_bstride, u32 n,
                           hipStream_t st) {
    Scalars K;
    for (u32 i = 0; i < CKKS_MAX_MODULI; i++) {
        K.ka[i] = i <= level ? ka[i] : 0;
        K.kb[i] = i <= level ? kb[i] : 0;
    }
    dim3 grid((c->N + PW_THREADS - 1) / PW_THREADS, level + 1, 2 * n);
    ProfScope ps__(c, K_LINCOMB2, st, 16.0 * n * c->N * (level + 1.0) * (3.0 + (add ? 1.0 : 0.0)), 4.0 * n * c->N * (level + 1.0));
    hipLaunchKernelGGL(lincomb2_kernel, grid, dim3(PW_THREADS), 0, st, a, a_cstride, b, b_cstride, add, add_bstride, K, out, out_bstride,
                       c->d_mc, c->N, level);
    return hipGetLastError();
}

// ---- the weight-width promise of the convolution (he_conv_desc.weight_bits), tested on the device-resident weights ----------
// w_res [n_w][nl]: counts the residues outside [0, bound) and (q - bound, q), bound = 2^(weight_bits - 1)
__global__ __launch_bounds__(PW_THREADS) void weight_check_kernel(const u64* __restrict__ w_res, const ModConst* __restrict__ mc, size_t n_w,
                                                                  u32 nl, u32 level, u32 num_q, u64 bound, u32* __restrict__ bad) {
    const size_t idx = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    if (idx >= n_w * nl) return;
    const u32 e = (u32)(idx % nl);
    const u64 q = mc[e <= level ? e : num_q + (e - level - 1)].q;
    const u64 v = w_res[idx];
    const bool ok = v < q && (v < bound || q - v < bound);
    if (!ok) atomicAdd(bad, 1u);
}
__global__ void clear_word_kernel(u32* p) { *p = 0; }

hipError_t launch_weight_check(const ckks_ctx* c, u32 level, bool extended, const u64* w_res, size_t n_w, u32 weight_bits, u32* d_count,
                               hipStream_t st) {
    const u32 nl = extended ? c->ext_limbs(level) : level + 1;
    const u64 bound = weight_bits >= 64 ? ~0ull : 1ull << (weight_bits - 1);
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, st, d_count);
    const size_t total = n_w * nl;
    hipLaunchKernelGGL(weight_check_kernel, dim3((unsigned)((total + PW_THREADS - 1) / PW_THREADS)), dim3(PW_THREADS), 0, st, w_res, c->d_mc,
                       n_w, nl, level, c->num_q, bound, d_count);
    return hipGetLastError();
}
