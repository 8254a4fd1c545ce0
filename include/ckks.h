/*
 * ckks.h -- C boundary of the MI355X RNS-CKKS batched-convolution library.
 *
 * The operations are the ones the paper's batched convolution layer is made of (Methodology,
 * "Convolution Layer": Rot, plaintext (.) ciphertext, accumulation; Eq. 8-11) and the RNS-CKKS
 * primitives underneath them, which the paper uses through a library (Background: "Rotations and
 * Key Switching", "RNS Decomposition and NTT Optimization"; Experiments, "HE Security Parameters":
 * digit-decomposed key switching, rescaling), plus the ciphertext product that the polynomial
 * activation needs ("Other Layers"), the batched fully connected layer ("Fully Connected Layer"), and
 * the pipeline's accumulator, down-sampling compaction and key staging ("Optimized Inference
 * Pipeline").  The server side only: key generation, encryption and decryption belong to the client
 * (Threat Model) and are not part of this library.
 *
 * Conventions shared by every call
 *   - Every function returns CKKS_OK (0) or a negative ckks_status; nothing throws or aborts.
 *     ckks_last_error_string() gives the reason of the last failure on that context.
 *   - Pointers named d_* are DEVICE pointers owned by the caller; pointers named h_* and all
 *     structs are HOST memory.  Hot calls never allocate, free or synchronise: work is enqueued on
 *     the caller's stream (a hipStream_t passed as void*, NULL = default stream; two calls may put
 *     part of it on a second stream of the context's, joined before they return: see
 *     ckks_ctx_set_overlap) and scratch space comes from the caller's workspace (d_ws, ws_bytes; size
 *     from the *_workspace_bytes() queries).  The caller keeps every buffer alive until the stream
 *     has drained.
 *   - A polynomial limb is N uint64 residues in [0, q) (canonical on input and on output).
 *     Polynomials are in evaluation (NTT) form: entry k of a limb is the value at
 *     psi^(2*bitrev(k)+1), psi the 2N-th root given for that modulus.  ckks_ntt_fwd maps
 *     natural-order coefficients to this order, ckks_ntt_inv maps back.
 *   - Moduli are indexed q_0..q_L (num_q ciphertext primes) then p_0..p_{k-1} (num_p special primes).
 *     A ciphertext at level l is uint64[2][l+1][N] (component, limb, coefficient), compact.
 *     The scale of a ciphertext is a host-side double the caller tracks; the library is integer only.
 *   - A switching key is uint64[dnum][2][num_q+num_p][N] in NTT form, component 0 = "b" part,
 *     component 1 = "a" part; digit j covers limbs [j*alpha, (j+1)*alpha), alpha = ceil(num_q/dnum).
 *     A key made for the top level serves every lower level.
 *   - Outputs must not overlap inputs or the workspace unless a call says "in place".
 */
#ifndef CKKS_MI355X_H
#define CKKS_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ckks_status {
    CKKS_OK = 0,
    CKKS_ERR_INVALID_ARG = -1,        /* null pointer, zero count, level out of range, ... */
    CKKS_ERR_LEVEL_MISMATCH = -2,     /* operation needs a lower/higher level than given */
    CKKS_ERR_UNSUPPORTED_PARAMS = -3, /* parameter set outside what the kernels handle */
    CKKS_ERR_WORKSPACE_TOO_SMALL = -4,
    CKKS_ERR_NO_KEY = -5,             /* key missing or made for another Galois element */
    CKKS_ERR_HIP = -6                 /* a HIP runtime call failed */
} ckks_status;

typedef struct ckks_ctx ckks_ctx; /* tables immutable after creation; see ckks_ctx_set_overlap for calls from several threads */
typedef struct ckks_key ckks_key;

/* Parameter set.  Supported: 4 <= log_n <= 17; num_q >= 1; num_q + num_p <= 64; every modulus a
 * prime below 2^58 with q = 1 mod 2N; psi[t]^N = -1 mod moduli[t]; dnum = 0 (no key switching,
 * then num_p = 0) or 1 <= dnum <= num_q with num_p >= 1. */
typedef struct ckks_params {
    uint32_t log_n;
    uint32_t num_q;
    uint32_t num_p;
    uint32_t dnum;
    const uint64_t* moduli; /* host, num_q + num_p entries */
    const uint64_t* psi;    /* host, primitive 2N-th root of unity per modulus */
} ckks_params;

/* Builds the context on the current HIP device: twiddle tables, reduction constants, basis-
 * conversion tables for every level, plus a stream and two events (ckks_ctx_set_overlap).  This is the
 * only call that allocates device memory (about 32*N bytes per modulus) and it synchronises the
 * device once. */
int ckks_ctx_create(const ckks_params* params, ckks_ctx** out_ctx);
void ckks_ctx_destroy(ckks_ctx* ctx);
const char* ckks_last_error_string(const ckks_ctx* ctx);

/* Scheduling (not from the paper).  Operations made of independent channel batches (he_conv_batched in the deferred
 * schedules, he_poly_act_deg7) run every other batch on a second stream owned by the context, between a fork after the
 * caller's earlier work and a join before the call's last enqueue on the caller's stream: arithmetic-bound and
 * traffic-bound kernels of different batches overlap.  The caller still sees one ordered stream.  on = 0 keeps all work
 * on the caller's stream (per-kernel timings are then not blurred by overlap); default on.  Results are identical.
 * With overlap on, such calls must not be issued on one context from several host threads at the same time. */
int ckks_ctx_set_overlap(ckks_ctx* ctx, int on);

typedef enum ckks_op {
    CKKS_OP_KEYSWITCH = 0,
    CKKS_OP_ROTATE = 1,        /* count = number of rotations in the call */
    CKKS_OP_RESCALE = 2,
    CKKS_OP_CTCT_MUL_RELIN = 3,
    CKKS_OP_POLY_ACT = 5       /* count = number of ciphertexts; the convolution has its own query */
} ckks_op;

/* Bytes of workspace the given operation needs at `level` (0 on invalid arguments). */
size_t ckks_workspace_bytes(const ckks_ctx* ctx, int op, uint32_t level, uint32_t count);

/* Negacyclic NTT over Z_q[X]/(X^N+1) (Background, "RNS Decomposition and NTT Optimization").
 * In place on batch*n_limbs consecutive limb-polys at d_polys; limb-poly number b*n_limbs+t uses
 * modulus moduli[h_modulus_idx[t]].  fwd: natural-order coefficients -> evaluation form;
 * inv: the exact inverse (includes 1/N). */
int ckks_ntt_fwd(const ckks_ctx* ctx, uint64_t* d_polys, const uint32_t* h_modulus_idx,
                 uint32_t n_limbs, uint32_t batch, void* stream);
int ckks_ntt_inv(const ckks_ctx* ctx, uint64_t* d_polys, const uint32_t* h_modulus_idx,
                 uint32_t n_limbs, uint32_t batch, void* stream);

/* Wraps a caller-owned switching key (no copy).  galois_elt = 5^r mod 2N for the key of a rotation
 * by r slots, 0 for the relinearisation key (s^2 -> s). */
int ckks_key_load(const ckks_ctx* ctx, const uint64_t* d_key, uint32_t galois_elt, ckks_key** out_key);
void ckks_key_free(ckks_key* key);

/* Staged keys ("Optimized Inference Pipeline", Evaluation Keys Reuse: only the keys of the current block group are
 * resident; sets are offloaded and loaded between groups).  The public halves a_j of a switching key are uniform
 * residues, so a staged key is its b_j halves (host, uint64[dnum][num_q+num_p][N], evaluation form) plus a 64-bit
 * seed: a[j][t][x] = the top bitlength(q_t) bits of the first of the outputs 64e, 64e+1, ... (e = (j*M + t)*N + x,
 * M = num_q+num_p) of the SplitMix64 sequence started at the seed that is below q_t (the 64th output reduced mod
 * q_t if none is).  Half the bytes cross the host link.
 * SplitMix64 is a stand-in here: it is not a cryptographic generator and its state is 64 bits, while the security argument
 * for seeded public halves needs an expansion by a pseudo-random function or extendable-output function keyed with at
 * least 128 bits (the paper runs at a 128-bit setting: Experiments, "HE Security Parameters").  The benchmark measures the
 * data movement and the expansion's cost; a deployment replaces the one device function that produces output number
 * `index` of the stream (and the seed type) and keeps everything else.
 * ckks_key_expand_a writes the a halves of d_key (uint64[dnum][2][M][N]); the b halves are left as they are.
 * ckks_keyset_stage enqueues, for each of n_keys keys, the copy of h_b[i] (pinned host memory for the copy to be
 * asynchronous) into the b halves of h_d_keys[i] and the expansion of h_a_seeds[i], all on `stream` (normally a
 * copy stream of the caller's, ordered against the compute stream with the caller's events); no allocation, no
 * synchronisation.  The device buffers are then keys for ckks_key_load. */
int ckks_key_expand_a(const ckks_ctx* ctx, uint64_t a_seed, uint64_t* d_key, void* stream);
int ckks_keyset_stage(const ckks_ctx* ctx, const uint64_t* const* h_b, const uint64_t* h_a_seeds,
                      uint64_t* const* h_d_keys, uint32_t n_keys, void* stream);

/* Galois element of a left rotation by `offset` slots (negative = right): 5^offset mod 2N. */
uint32_t ckks_galois_element(const ckks_ctx* ctx, int32_t offset);

/* Hybrid key switch of one polynomial (Background, "Rotations and Key Switching"):
 * d_c uint64[level+1][N] -> d_out uint64[2][level+1][N] with out0 + out1*s = c*s' + small noise,
 * s' the secret the key was made for.  Steps: per digit iNTT and basis extension to the live
 * q-limbs and the special primes (centred representatives, plain sum without floating-point
 * correction), NTT, inner product with the key, division by P (P-part extended the same way, so
 * the division rounds to nearest up to an error below num_p/2). */
int ckks_keyswitch(const ckks_ctx* ctx, const uint64_t* d_c, uint32_t level, const ckks_key* key,
                   uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream);

/* Rot(ct, r) for n_rot offsets of one ciphertext (Eq. 8-10): slot i of output t holds slot
 * (i + h_offsets[t]) mod N/2 of the input.  keys[t] must carry the Galois element of h_offsets[t];
 * an offset that is 0 mod N/2 is a plain copy and needs no key (keys[t] may be NULL).
 * hoisted = 1: c1 is decomposed and extended once and every rotation permutes the extended digits
 * ("fast rotations"); hoisted = 0: each rotation permutes the ciphertext and key-switches the
 * permuted c1.  Both orders give the same residues (centred digits commute with the automorphism).
 * h_d_outs: host array of n_rot device pointers, each uint64[2][level+1][N].
 * Workspace: ckks_workspace_bytes(ctx, CKKS_OP_ROTATE, level, n_rot) lets up to 8 rotations share every launch
 * but the inner products; a smaller one is accepted down to the size for n_rot = 1 (unhoisted rotations then go
 * in smaller batches, same residues), below that CKKS_ERR_WORKSPACE_TOO_SMALL. */
int ckks_rotate_hoisted(const ckks_ctx* ctx, const uint64_t* d_ct, uint32_t level,
                        const int32_t* h_offsets, uint32_t n_rot, const ckks_key* const* keys,
                        uint64_t* const* h_d_outs, int hoisted, void* d_ws, size_t ws_bytes, void* stream);

/* Plaintext-ciphertext multiply-accumulate (Eq. 11 and the channel sum after it):
 * acc[c][i][x] = (accumulate ? acc[c][i][x] : 0) + sum_k pt_k[i][x] * ct_k[c][i][x]  mod q_i.
 * h_d_pts / h_d_cts: host arrays of n_terms device pointers (uint64[level+1][N] and
 * uint64[2][level+1][N]).  d_acc may not overlap any operand. */
int ckks_ptct_mac(const ckks_ctx* ctx, const uint64_t* const* h_d_pts, const uint64_t* const* h_d_cts,
                  uint32_t n_terms, uint32_t level, uint64_t* d_acc, int accumulate, void* stream);

/* Rescale (Experiments, "HE Security Parameters"): divide by q_level with rounding to nearest and
 * drop that limb.  d_ct uint64[2][level+1][N] -> d_out uint64[2][level][N]; level >= 1.
 * The caller divides the scale by q_level. */
int ckks_rescale(const ckks_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out,
                 void* d_ws, size_t ws_bytes, void* stream);

/* ckks_rescale for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same residues; the scratch (the dropped limb in
 * coefficient form and the forward transforms' first-pass output) is a buffer of CKKS_NOALLOC_SCRATCH_BYTES that is part
 * of the library's image on every GPU it runs on, so the call needs ckks_workspace_bytes(ctx, CKKS_OP_RESCALE, level, 1)
 * <= CKKS_NOALLOC_SCRATCH_BYTES ((level + 1) * 16 * N bytes: N = 2^16 up to level 31, N = 2^17 up to level 15) and returns
 * CKKS_ERR_UNSUPPORTED_PARAMS beyond that.  It calls no allocating routine and does not synchronise.  All calls on one
 * GPU share the buffer: calls whose work overlaps in time on one GPU (different streams, different contexts) race; on
 * one stream they are ordered.  The context's device must be the current one. */
#define CKKS_NOALLOC_SCRATCH_BYTES (32u << 20)
int ckks_rescale_noalloc(const ckks_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out, void* stream);

/* Ciphertext product with relinearisation ("Other Layers": polynomial activation):
 * (d0, d1, d2) = (a0 b0, a0 b1 + a1 b0, a1 b1); out = (d0, d1) + KeySwitch(d2, rlk).  No rescale.
 * rlk must be the relinearisation key (galois_elt 0).  d_a may equal d_b. */
int ckks_ctct_mul_relin(const ckks_ctx* ctx, const uint64_t* d_a, const uint64_t* d_b, uint32_t level,
                        const ckks_key* rlk, uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream);

/* Batched 3x3 convolution layer, stride 1, zero padding 1, on channel-by-channel packed
 * ciphertexts (Eqs. 2-5: ciphertext c holds channel c of all `batch` images, image j in slots
 * [j*H*W, (j+1)*H*W); Eqs. 6-7, 10, 11):
 *   out_o = Rescale( sum_{c < C_in} sum_{tap} pt[o,c,tap] (.) Rot(in_c, dy*W + dx) ),  tap = (dy,dx)
 * in row-major order over {-1,0,1}^2.  The weight plaintexts are given in factored form,
 *   pt[o,c,tap] = w_int[o,c,tap] * M_tap  (mod q_i),
 * M_tap = d_tap_masks[tap] the encoded 0/1 validity mask of the tap (uint64[9][level+1][N], NTT
 * form) and w_int the integer weight, given by its residues d_w_res uint64[C_out][C_in][9][level+1].
 * rot_keys[tap] is the key of offset dy*W+dx (entry 4, the centre, is ignored).  With
 * HE_CONV_ALIGN_DIRECT the eight rotations of each input share one decomposition (hoisted).
 * h_d_in: C_in device pointers uint64[2][level+1][N]; h_d_out: C_out device pointers
 * uint64[2][level][N].  Fails with CKKS_ERR_INVALID_ARG if H*W*batch > N/2 (Eq. 4). */
typedef enum he_conv_alignment {
    HE_CONV_ALIGN_DIRECT = 0,   /* eight rotations of the input by dy*W+dx, eight keys, one decomposition */
    HE_CONV_ALIGN_FOUR_KEYS = 1,/* the paper's input alignment (Eqs. 8-10): C^-1 = Rot(in,-1), C^+1 =
                                   Rot(in,+1), then Rot(.,-W) and Rot(.,+W) of C^-1, in, C^+1; only the keys
                                   of -1, +1, -W, +W (rot_keys entries 3, 5, 1, 7) are read; three
                                   decompositions per input; half the resident key bytes */
    HE_CONV_DEFERRED_MODDOWN = 2,/* eight direct rotations as in DIRECT, but the division by P that ends each
                                   key switch is taken once per OUTPUT channel, after the sum of Eq. 11:
                                     X_tap(in) = (P * sigma_g(c0) + v_0, v_1),  v = <sigma_g(ModUp(c1)), key_g>
                                     out_o = Rescale( ModDown( sum_c sum_tap pt[o,c,tap] (.) X_tap(in_c) ) )
                                   on the extended basis q_0..q_level, p_0..p_{k-1}.  In this mode
                                   d_tap_masks is uint64[9][level+1+num_p][N] and d_w_res is
                                   uint64[C_out][C_in][9][level+1+num_p] (residues modulo the special primes
                                   appended); C_out ModDowns instead of 8*C_in, one rounding per output */
    HE_CONV_DEFERRED_MERGED = 3/* as DEFERRED_MODDOWN, and the ModDown of every sum is merged with its rescale: one
                                   division by P * q_level (dropped limbs q_level, p_0..p_{k-1}), one rounding, 48
                                   fewer limb transforms per output at 24 limbs */
} he_conv_alignment;

typedef struct he_conv_desc {
    uint32_t c_in, c_out, height, width, batch, level;
    uint32_t alignment; /* he_conv_alignment; all give the same slots up to noise, different residues */
    uint32_t weight_bits; /* 0, or a promise that every weight is an integer w with |w| < 2^(weight_bits-1) (d_w_res
                             holds w mod each modulus): weights are a real number times the weight scale, rounded, so
                             they are far narrower than a residue, and the multiply-accumulate then writes them in 3
                             (weight_bits <= 24) or 4 (<= 32) signed 8-bit digits instead of 7.  Same residues out;
                             a weight beyond the promised bound gives wrong residues without an error from
                             he_conv_batched itself: he_conv_check_weights tests the promise. */
} he_conv_desc;

/* Workspace bytes he_conv_batched needs for this shape (0 on invalid arguments): the shared
 * decomposition, 9*C_in masked aligned ciphertexts, C_out accumulators and rescale scratch. */
size_t he_conv_workspace_bytes(const ckks_ctx* ctx, const he_conv_desc* desc);

int he_conv_batched(const ckks_ctx* ctx, const he_conv_desc* desc, const uint64_t* const* h_d_in,
                    const ckks_key* const* rot_keys, const uint64_t* d_tap_masks, const uint64_t* d_w_res,
                    uint64_t* const* h_d_out, void* d_ws, size_t ws_bytes, void* stream);

/* Tests the promise desc->weight_bits on the device-resident weights d_w_res of a layer (same layout and basis as
 * he_conv_batched takes for desc->alignment): every residue must be the reduction of an integer w with
 * |w| < 2^(weight_bits-1), i.e. lie in [0, 2^(weight_bits-1)) or in (q_i - 2^(weight_bits-1), q_i).  Returns CKKS_OK,
 * or CKKS_ERR_INVALID_ARG with the number of offending residues in the error string.  weight_bits = 0 promises
 * nothing and passes.  For set-up time, once per set of weights, not per layer evaluation: it waits for `stream`
 * (one pass over d_w_res, one word read back) and, unlike every other call, must not be issued on one context from
 * several host threads at once. */
int he_conv_check_weights(const ckks_ctx* ctx, const he_conv_desc* desc, const uint64_t* d_w_res, void* stream);

/* The accumulator of the optimised pipeline ("Optimized Inference Pipeline", the merge equation): g
 * down-sampled intermediate ciphertexts whose data occupy slots [0, sts) are cleaned, moved to
 * disjoint slot ranges and added,
 *   out = Rescale( sum_{i<g} Rot(C_i (.) M, -i*sts) ),
 * so that block i lands in slots [i*sts, (i+1)*sts).  d_mask: the encoded cleaning mask M (ones on the
 * first sts slots), uint64[level+1][N], NTT form; keys[i] the key of offset -i*sts for 1 <= i < g
 * (keys[0] ignored).  h_d_cts: g <= 16 device pointers uint64[2][level+1][N]; d_out uint64[2][level][N].
 * Fails with CKKS_ERR_INVALID_ARG if g*sts > N/2.  Workspace from he_accumulator_workspace_bytes(). */
size_t he_accumulator_workspace_bytes(const ckks_ctx* ctx, uint32_t level, uint32_t g);
int he_accumulator_merge(const ckks_ctx* ctx, const uint64_t* const* h_d_cts, uint32_t g, uint32_t level, uint32_t sts,
                         const uint64_t* d_mask, const ckks_key* const* keys, uint64_t* d_out, void* d_ws,
                         size_t ws_bytes, void* stream);

/* Slot re-layout with two rotations per element: the output reconstruction of the FC layer ("Fully Connected
 * Layer": every element moves by base_idx + mod_idx with two rotation keys) as an operation of its own, applied to
 * the n_ct ciphertexts of a channel vector (they share keys and masks):
 *   out_b = sum_h Rot( Rescale( sum_l M[h][l] (.) Rot(ct_b, lo[l]) ), hi[h] )
 * An element that has to move left by lo[l] + hi[h] slots is selected by the mask M[h][l] after its first rotation.
 * It is what compacts the slots after a stride-r layer ("Optimized Inference Pipeline": H' = H/r, W' = W/r,
 * sts' = sts/r^2) in front of he_accumulator_merge: once inside every image (lo = x'(r-1), hi = y'(rW - W')), once
 * over whole images (lo = (j mod base) d, hi = (j div base) base d, d = HW - H'W').
 * h_d_cts[b] uint64[2][level+1][N], level >= 1; h_lo / h_hi: host arrays of slot offsets (0 = no rotation, key
 * ignored); lo_keys[l] / hi_keys[h] made for those offsets; h_d_masks: host array of n_hi*n_lo device pointers,
 * entry h*n_lo + l is a plaintext in NTT form or NULL when no element takes that pair (every h needs one mask at
 * least); h_d_outs[b] uint64[2][level][N], one level lower.  Outputs must not overlap inputs.
 * schedule HE_RELAYOUT_DIRECT: every rotation is completed (divided by P) on its own; masks uint64[level+1][N].
 * schedule HE_RELAYOUT_DEFERRED: the divisions by P come after the sums, as in the convolution's deferred schedules:
 * the first rotations stay on the extended basis Q_level P, each inner sum takes one division by P*q_level, the second
 * rotations are summed on the extended basis of level-1 and divided by P once; masks uint64[level+1+num_p][N] on the
 * extended basis.  A first rotation then costs an inner product only.  Same slots, different residues. */
enum he_relayout_schedule { HE_RELAYOUT_DIRECT = 0, HE_RELAYOUT_DEFERRED = 1 };
size_t he_relayout_workspace_bytes(const ckks_ctx* ctx, uint32_t level, uint32_t n_ct, uint32_t n_lo, uint32_t n_hi,
                                   uint32_t schedule);
int he_relayout_two_rotations(const ckks_ctx* ctx, const uint64_t* const* h_d_cts, uint32_t n_ct, uint32_t level,
                              const int32_t* h_lo, uint32_t n_lo, const ckks_key* const* lo_keys, const int32_t* h_hi,
                              uint32_t n_hi, const ckks_key* const* hi_keys, const uint64_t* const* h_d_masks,
                              uint32_t schedule, uint64_t* const* h_d_outs, void* d_ws, size_t ws_bytes, void* stream);

/* Batched fully connected layer ("Fully Connected Layer": FC evaluation and output reconstruction).  The input
 * ciphertext holds x^(j) (d_in values, d_in a power of two) in slots [j*d_in, (j+1)*d_in) for j < batch
 * (batch*d_in <= N/2); the output, three levels lower, holds W x^(j) + bias in slots [j*d_out, (j+1)*d_out).
 *   1. C_i = Rescale(C_in (.) w_i^enc), S_i = Sum_{d_in}(C_i) by log2(d_in) steps T <- T + Rot(T, 2^s)   (i < d_out)
 *   2. U = Rescale( sum_i Rot(S_i (.) E, -i) )                  element (j, i) at slot j*d_in + i
 *   3. R_l = Rot(U, l*delta), l < base, delta = d_in - d_out    (mod_idx rotations; one decomposition)
 *      V_h = Rescale( sum_l R_l (.) E'_{h*base+l} );  out = sum_h Rot(V_h, h*base*delta)   (base_idx rotations)
 *   4. out_0 += bias^enc
 * Operands (all NTT form): d_w_enc uint64[d_out][level+1][N] (row i of W replicated over the batch blocks),
 * d_merge_mask uint64[level][N] (ones at slots j*d_in), d_place_masks uint64[batch][level-1][N] (block j's d_out
 * slots after its first rotation: ones at [j*d_in - (j % base)*delta, +d_out)), d_bias uint64[level-2][N].
 * Keys: sum_keys[s] for offset 2^s (s < log2 d_in), merge_keys[i] for -i, lo_keys[l] for l*delta, hi_keys[h] for
 * h*base*delta (entries whose offset is 0 mod N/2 are ignored).  base = 0 means ceil(sqrt(batch)).
 * d_in_ct uint64[2][level+1][N], level >= 3; d_out uint64[2][level-2][N]; d_out <= 16 outputs per call. */
typedef struct he_fc_desc {
    uint32_t d_in, d_out, batch, level, base;
} he_fc_desc;
size_t he_fc_workspace_bytes(const ckks_ctx* ctx, const he_fc_desc* desc);
int he_fc_batched(const ckks_ctx* ctx, const he_fc_desc* desc, const uint64_t* d_in_ct, const uint64_t* d_w_enc,
                  const ckks_key* const* sum_keys, const ckks_key* const* merge_keys, const uint64_t* d_merge_mask,
                  const uint64_t* d_place_masks, const ckks_key* const* lo_keys, const ckks_key* const* hi_keys,
                  const uint64_t* d_bias, uint64_t* d_out, void* d_ws, size_t ws_bytes, void* stream);

/* Odd degree-7 polynomial activation on a vector of n_ct channel ciphertexts, four ciphertext
 * products each ("Other Layers": the activation applied independently to every element of the
 * channel vector):  x2 = x*x, x3 = x2*x, x4 = x2*x2 (each rescaled once),
 *   B = Rescale(k[2]*x + k[3]*x3),  y = Rescale((k[0]*x + k[1]*x3) + x4*B).
 * h_k: four signed integers that fold the polynomial coefficients and the scale ratios (the caller
 * tracks scales; the same four for every channel).  h_d_x: n_ct device pointers uint64[2][level+1][N],
 * level >= 4; h_d_out: n_ct device pointers uint64[2][level-3][N].  Channels are processed in
 * batches that share one pass over the relinearisation key; workspace from
 * ckks_workspace_bytes(ctx, CKKS_OP_POLY_ACT, level, n_ct).
 * merged_division != 0: every relinearise-then-rescale pair is one division by P * q_level instead of
 * two (the tensor product's d0, d1, and for y the linear part, enter the extended basis as P times
 * themselves before the division): same levels and scales, one rounding per product, other residues. */
int he_poly_act_deg7(const ckks_ctx* ctx, const uint64_t* const* h_d_x, uint32_t n_ct, uint32_t level,
                     const int64_t* h_k, const ckks_key* rlk, int merged_division, uint64_t* const* h_d_out,
                     void* d_ws, size_t ws_bytes, void* stream);

/* Self-test hook (not part of the paper's method): evaluates on the GPU the routines of the double-precision modular
 * arithmetic that the transforms, basis conversions and fused inner products are made of, for moduli q < 2^50, on
 * caller-given operands, so that a test can judge the device's results with wide integers.
 *   CKKS_F64_MULMOD      out = y*w - q*c, c the integer nearest to y*wq      (d_wq[i] = d_w[i] / q rounded to nearest)
 *   CKKS_F64_MULMOD_ANY  the same with c taken from the rounded product y*w  (d_wq unused)
 *   CKKS_F64_REDUCE      out = y - q*round(y/q)                              (d_w, d_wq unused)
 *   CKKS_F64_CANONICAL   out = y mod q in [0, q), through REDUCE             (d_w, d_wq unused)
 *   CKKS_F64_CENTRE      out = y*w mod q as the centred residue, through MULMOD
 *   CKKS_F64_DOT8, _DOT9 out[i] = sum_a y[i][a] * w[a] mod q as a reduced double: the basis-conversion sum of 8 or 9 terms
 *                        (d_y int64[n][8 or 9], centred residues |y| < 2^49; d_w uint64[8 or 9] in [0, q), taken by their
 *                        centred representatives as the library's tables hold them; d_wq unused)
 * d_y int64[n] (integers, |y| < 2^51 for the products, < 2^53 otherwise), d_w uint64[n] in [0, q), d_out double[n]. */
enum ckks_f64_op { CKKS_F64_MULMOD = 0, CKKS_F64_MULMOD_ANY = 1, CKKS_F64_REDUCE = 2, CKKS_F64_CANONICAL = 3, CKKS_F64_CENTRE = 4,
                   CKKS_F64_DOT8 = 5, CKKS_F64_DOT9 = 6 };
int ckks_f64mod_probe(int op, const int64_t* d_y, const uint64_t* d_w, const double* d_wq, uint64_t q, double* d_out, size_t n,
                      void* stream);

/* Optional per-kernel timing, for benchmarks (not part of the paper's method; callers that measure).
 * Between ckks_prof_begin and ckks_prof_end every launch of a kernel class whose bit is set in
 * kernel_mask is bracketed by a HIP event pair on the stream it is launched on (at most
 * max_launches pairs; later launches are counted as dropped).  ckks_prof_begin creates the events
 * (not a hot call); ckks_prof_end waits for them and writes, per kernel class (arrays of
 * ckks_prof_kernel_count() entries, any of them may be NULL): total milliseconds, launch count, the
 * algorithmic HBM bytes of those launches (every operand read once, every result written once) and
 * their modular multiplications (butterflies / multiply-adds); then it frees the events.
 * One profiling session at a time per context; not thread-safe. */
uint32_t ckks_prof_kernel_count(void);
const char* ckks_prof_kernel_name(uint32_t id);
int ckks_prof_begin(ckks_ctx* ctx, uint32_t kernel_mask, uint32_t max_launches);
int ckks_prof_end(ckks_ctx* ctx, double* h_ms, uint64_t* h_launches, double* h_bytes, double* h_ops, uint64_t* h_dropped);

#ifdef __cplusplus
}
#endif
#endif /* CKKS_MI355X_H */
