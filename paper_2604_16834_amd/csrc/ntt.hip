// Negacyclic NTT / inverse NTT over Z_q[X]/(X^N+1) for gfx950 (Background, "RNS Decomposition and
// NTT Optimization": the transform that makes ring multiplication quasi-linear).
//
// Forward: natural-order coefficients in, out[k] = a(psi^(2*bitrev(k)+1)).  The log2(N) radix-2
// stages are split into two passes; in each pass one 256-thread workgroup transforms a 2^11-point
// tile, every thread holding 8 points in registers:
//   hi pass : the first log_hi = log2(N) - 11 stages pair points 2^11 or more apart.  A tile is all
//             2^log_hi rows (rows are 2^11 elements apart) of a run of adjacent columns, so every
//             row segment is a contiguous, coalesced run.  Radix-8 in registers, one exchange through
//             LDS, then the remaining log_hi - 3 stages in registers.
//   lo pass : the last 11 stages act inside contiguous blocks of 2^11 points: radix 8, 8, 8, 4 in
//             registers with three exchanges through (padded, double-buffered) LDS.
// The bit-reversed output order falls out of this split with no transpose.  The inverse runs the
// mirrored lo pass first, then the mirrored hi pass, and folds the 1/N into its last store.
// Twiddles psi^bitrev(i) sit in one table per modulus, 16 bytes per entry; the index of the twiddle of
// a butterfly group obeys T(next stage) = 2*T + bit, so a thread needs only the index of its group at
// the first stage of a round.
//
// Two butterfly arithmetics, chosen per context (both give the same canonical residues):
//   ArithU64  any modulus below 2^58: 64-bit Shoup multiplication (twiddle + precomputed quotient), lazy
//             values (forward: no correction at all, below 35q < 2^64; inverse: kept in [0, 2q)).
//   ArithF64  every modulus below 2^50: residues are integers held in doubles and the twiddle product is
//             reduced with fused multiply-adds: for |y| < 2^51, h = y*w rounded, l = fma(y, w, -h) its
//             exact error, c = the integer nearest to y*(w/q) (one fma against 1.5*2^52), and
//             fma(-c, q, h) + l = y*w - c*q exactly, of magnitude below 0.75 q: six double-precision
//             operations where the integer path spends more than twenty 32-bit ones, which moves the
//             lo pass from instruction issue to the HBM roof.  Values are brought back to |v| <= q/2 + 1
//             (three operations) after every round of at most three forward stages and after every sum of
//             an inverse butterfly, so every multiplicand stays below 2q < 2^51 and every sum below 2^53:
//             all arithmetic is exact.  Between the two passes the data sit in HBM as doubles.
// Rings below 2^11 use a plain one-tile integer kernel.
#include <type_traits>

#include "ctx.h"
#include "f64mod.h"
#include "galois.h"

#define NTT_THREADS 256
#define NTT_TILE 2048
// Where point p of a tile sits in LDS.  A wavefront's 8-byte accesses are served sixteen lanes at a time, one per pair of
// 4-byte banks, so an access is conflict-free when the low four bits of the sixteen word indices are distinct.  The lo
// pass' four patterns spread the sixteen lanes over index bits {0,1,2,3} (thread-contiguous), {0,1,5,6} (round C),
// and {3,4,5,6} (eight consecutive points per thread); folding bits 4, 5, 6 into bits 1, 2, 3 and bit 6 also into
// bit 0 makes the low four bits a bijection of the lanes in all of them (measured: 6.2 cycles per wave-level 8-byte
// write in every pattern, against 8.1 with one padding word per eight in the two thread-contiguous ones).
#define LDS_PAD(p) ((p) ^ ((((p) >> 4) & 7u) << 1) ^ (((p) >> 6) & 1u))
#define LDS_PADDED_WORDS NTT_TILE

// ---- 64-bit integer arithmetic --------------------------------------------------------------------------
// Forward butterfly with no correction at all: the Shoup product t is in [0, 2q) for ANY 64-bit y, so
// both outputs stay non-negative and grow by at most 2q per stage: below (1 + 2*17) q < 2^64 for every
// supported modulus (q < 2^58) over a whole transform.  One word reduction at the very end.
struct ArithU64 {
    typedef u64 E;
    typedef TwPair TW;
    typedef ModConst MC;
    static __device__ __forceinline__ E load_first(u64 raw, const MC&, bool /*inverse*/) { return raw; }
    static __device__ __forceinline__ E load_mid(u64 raw) { return raw; }
    static __device__ __forceinline__ u64 store_mid(E v) { return v; }
    static __device__ __forceinline__ u64 store_fwd_final(E v, const MC& m) { return reduce_word(v, m); }
    static __device__ __forceinline__ u64 store_inv_final(E v, const MC& m) { return mul_shoup(v, m.n_inv, m.n_inv_sh, m.q); }
    static __device__ __forceinline__ void fwd_bf(E& x, E& y, const TW w, const MC& m) {
        const u64 t = mul_shoup_lazy(y, w.w, w.s, m.q);
        y = x + 2 * m.q - t;
        x = x + t;
    }
    static __device__ __forceinline__ void inv_bf(E& x, E& y, const TW w, const MC& m) {
        const u64 two_q = 2 * m.q;
        u64 s = x + y;
        if (s >= two_q) s -= two_q;
        const u64 d = x + two_q - y;
        x = s;
        y = mul_shoup_lazy(d, w.w, w.s, m.q);
    }
    static __device__ __forceinline__ void fwd_round_end(E*, const MC&) {}
};

// ---- double-precision arithmetic for moduli below 2^50 (the routines themselves: f64mod.h) -----------------------
struct ArithF64 {
    typedef double E;
    typedef TwF TW;
    typedef ModConstF MC;
    static __device__ __forceinline__ double round_mul(double v, double c) { return f64m_round_mul(v, c); }
    // v - q * round(v / q): |result| <= q/2 + 1 for integer |v| < 2^53
    static __device__ __forceinline__ double reduce(double v, const MC& m) { return f64m_reduce(v, m.q, m.qinv); }
    // y * w - q * c, c an integer within 3/4 of y * w / q: exact, magnitude below 0.75 q; needs |y| < 2^51, 0 <= w < q, wq = w / q rounded
    static __device__ __forceinline__ double mulmod(double y, double w, double wq, double q) { return f64m_mulmod(y, w, wq, q); }
    // the same for a multiplier without a precomputed w / q (a key word, a ciphertext residue): |y| < q, 0 <= w < q;
    // exact, magnitude below 0.75 q (0.63 q for |y| <= q/2 + 1)
    static __device__ __forceinline__ double mulmod_any(double y, double w, double q, double qinv) { return f64m_mulmod_any(y, w, q, qinv); }
    static __device__ __forceinline__ double from_u64(u64 raw) { return f64m_from_u64(raw); }
    static __device__ __forceinline__ u64 to_u64(double v) { return f64m_to_u64(v); }
    static __device__ __forceinline__ u64 canonical(double v, const MC& m) { return f64m_canonical(v, m.q); }  // |v| <= q/2 + 1 -> [0, q)
    static __device__ __forceinline__ E load_first(u64 raw, const MC& m, bool) { return reduce(from_u64(raw), m); }
    static __device__ __forceinline__ E load_mid(u64 raw) { return __longlong_as_double((long long)raw); }
    static __device__ __forceinline__ u64 store_mid(E v) { return (u64)__double_as_longlong(v); }
    static __device__ __forceinline__ u64 store_fwd_final(E v, const MC& m) { return canonical(v, m); }  // after fwd_round_end
    static __device__ __forceinline__ u64 store_inv_final(E v, const MC& m) { return canonical(mulmod(v, m.ninv, m.ninv_q, m.q), m); }
    static __device__ __forceinline__ void fwd_bf(E& x, E& y, const TW w, const MC& m) {
        const double t = mulmod(y, w.w, w.wq, m.q);
        y = x - t;
        x = x + t;
    }
    static __device__ __forceinline__ void inv_bf(E& x, E& y, const TW w, const MC& m) {
        const double s = x + y, d = x - y;
        x = reduce(s, m);
        y = mulmod(d, w.w, w.wq, m.q);
    }
    static __device__ __forceinline__ void fwd_round_end(E* v, const MC& m) {
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = reduce(v[j], m);
    }
};

// S radix-2 stages on 2^S "rows" of KC independent columns held in registers, v[row*KC + col];
// row bit S-1 is the largest distance.  T = twiddle index of this group at the first stage.
template <class A, int S, int KC>
__device__ __forceinline__ void fwd_rows(typename A::E* v, const typename A::TW* __restrict__ tw, u32 T, const typename A::MC& m) {
#pragma unroll
    for (int a = 0; a < S; a++) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            const typename A::TW w = tw[(T << a) + (rr >> (S - a))];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) A::fwd_bf(v[rr * KC + kc], v[(rr + half) * KC + kc], w, m);
        }
    }
}

template <class A, int S, int KC>
__device__ __forceinline__ void inv_rows(typename A::E* v, const typename A::TW* __restrict__ tw, u32 T, const typename A::MC& m) {
#pragma unroll
    for (int a = S - 1; a >= 0; a--) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            const typename A::TW w = tw[(T << a) + (rr >> (S - a))];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) A::inv_bf(v[rr * KC + kc], v[(rr + half) * KC + kc], w, m);
        }
    }
}

// Butterflies whose twiddle is the value alone (no twiddle / q): the quotient comes from the rounded product.  Half the
// registers and half the bytes per twiddle; from inputs reduced to q/2 + 1 the three stages of a round add at most 0.63 q,
// 0.79 q and 0.98 q, so multiplicands stay below 2q and sums below 2^53 as with the precomputed quotient.
struct ArithF64W : ArithF64 {
    typedef double TW;
    static __device__ __forceinline__ void fwd_bf(E& x, E& y, const double w, const MC& m) {
        const double t = mulmod_any(y, w, m.q, m.qinv);
        y = x - t;
        x = x + t;
    }
    // the inverse butterfly: the sum is re-centred, the difference (below 2q) times the twiddle is at most q
    static __device__ __forceinline__ void inv_bf(E& x, E& y, const double w, const MC& m) {
        const double s = x + y, d = x - y;
        x = reduce(s, m);
        y = mulmod_any(d, w, m.q, m.qinv);
    }
};
template <int S>
__device__ __forceinline__ void load_tw_w(const double* __restrict__ tw, u32 T, double* tv) {
#pragma unroll
    for (int a = 0; a < S; a++)
#pragma unroll
        for (int j = 0; j < (1 << a); j++) tv[(1 << a) - 1 + j] = tw[(T << a) + j];
}

// what the lo passes hold of a twiddle and how they multiply by it: the value alone in double precision
template <class A>
struct LoTw {
    typedef A AR;
    typedef typename A::TW TW;
};
template <>
struct LoTw<ArithF64> {
    typedef ArithF64W AR;
    typedef double TW;
};

// The same with the round's 2^S - 1 twiddles already in registers (tv[(1 << a) - 1 + j] = tw[(T << a) + j]):
// the lo pass requests the twiddles of the next round before it starts the current one, so their
// latency (they come from L2) hides behind a round of butterflies and an LDS exchange.
template <class A, int S>
__device__ __forceinline__ void load_tw(const typename A::TW* __restrict__ tw, u32 T, typename A::TW* tv) {
#pragma unroll
    for (int a = 0; a < S; a++)
#pragma unroll
        for (int j = 0; j < (1 << a); j++) tv[(1 << a) - 1 + j] = tw[(T << a) + j];
}

template <class A, int S>
__device__ __forceinline__ void fwd_rows_pre(typename A::E* v, const typename A::TW* tv, const typename A::MC& m) {
#pragma unroll
    for (int a = 0; a < S; a++) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            A::fwd_bf(v[rr], v[rr + half], tv[(1 << a) - 1 + (rr >> (S - a))], m);
        }
    }
}

template <class A, int S>
__device__ __forceinline__ void inv_rows_pre(typename A::E* v, const typename A::TW* tv, const typename A::MC& m) {
#pragma unroll
    for (int a = S - 1; a >= 0; a--) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            A::inv_bf(v[rr], v[rr + half], tv[(1 << a) - 1 + (rr >> (S - a))], m);
        }
    }
}

struct NttArgs {
    const u64* src;
    u64* dst;
    size_t src_bstride;  // in limb-polys
    size_t dst_bstride;
    const void* mc;      // [M] ModConst or ModConstF
    const void* tw;      // [M][N] TwPair or TwF
    const double* tw_val;  // [M][N] the twiddles' values alone (lo passes in double precision), or null
    u32 log_n, log_lo, log_hi;
    u32 first;           // this pass reads the caller's canonical residues (else the other pass's intermediate form)
    u32 last;            // this pass writes the final result (canonical; inverse: times 1/N)
    u32 batch;           // batch items (each pl.n limb-polys)
    u32 lo_group;        // slices per group of the lo-pass numbering (0: plain)
    u32 use_src_list;    // batch item b reads src_list.p[b] instead of src + b*src_bstride*N
    PtrList8 src_list;
    PtrList8 mul_list;     // inverse, first pass, product variant: batch item b is src_list.p[b] (.) mul_list.p[b]
    u64 lin_ka, lin_kb;    // use_lin: ... is lin_ka * src_list.p[b] + lin_kb * mul_list.p[b] instead (one limb per item)
    u32 use_lin, pad2;
    const TwF* inv_scale;  // inverse, last pass (double-precision arithmetic): the limb of modulus m is scaled by inv_scale[m]
                           // instead of 1/N and stored as the centred residue in a double (the form ModUp's conversion reads)
};

// Lo-pass workgroups are numbered in groups of `grp` consecutive (limb, block) slices, batch item by
// batch item: the `batch` tiles that use the same twiddle slice get ids that are a multiple of 8
// apart (same XCD) and close in time, so the slice comes from HBM once and from that XCD's L2 for the
// rest of the batch, while each batch item's `grp` tiles are one contiguous run of memory.
struct LoTile {
    u32 b, a, blk;
};
// grid = (grp, batch, slices / grp): linear id = x + grp * (y + batch * z), slice t = z * grp + x, item b = y
// (plain numbering when grp == 0: grid = (batch, slices), b = x, t = y)
__device__ __forceinline__ LoTile lo_tile(u32 log_hi, u32 grp) {
    const u32 t = grp ? blockIdx.z * grp + blockIdx.x : blockIdx.y;
    LoTile r;
    r.b = grp ? blockIdx.y : blockIdx.x;
    r.a = t >> log_hi;
    r.blk = t & ((1u << log_hi) - 1);
    return r;
}

// Entry i of one of a PolyList's byte arrays.  The list is a kernel argument and i is the same for the whole workgroup: read
// as the 32-bit word that holds it, this is a scalar load; a byte load is a vector load whose round trip to memory every
// address of the kernel then waits for.
__device__ __forceinline__ u32 pl_at(const unsigned char* arr, u32 i) {
    const u32 w = reinterpret_cast<const u32*>(arr)[i >> 2];
    return (w >> (8 * (i & 3))) & 0xffu;
}

template <class A>
struct PolyRef {
    const u64* src;
    u64* dst;
    const typename A::TW* tw;
    const double* tw_val;  // this modulus' row of NttArgs::tw_val
    typename A::MC mc;
};

// BYTES: read the list's entries with byte loads all the same (the converting hi pass: with scalar positions its tables of
// constants become scalar loads too, four limbs' worth of them more than the scalar registers hold: measured slower)
template <class A, bool BYTES = false>
__device__ __forceinline__ PolyRef<A> poly_ref(const NttArgs& args, const PolyList& pl, u32 b, u32 a) {
    const u32 m_idx = BYTES ? pl.mod[a] : pl_at(pl.mod, a);
    PolyRef<A> r;
    const u32 sp = BYTES ? pl.spos[a] : pl_at(pl.spos, a), dp = BYTES ? pl.dpos[a] : pl_at(pl.dpos, a);
    r.src = (args.use_src_list ? args.src_list.p[b] : args.src + (((size_t)b * args.src_bstride) << args.log_n)) + ((size_t)sp << args.log_n);
    r.dst = args.dst + (((size_t)b * args.dst_bstride + dp) << args.log_n);
    r.tw = (const typename A::TW*)args.tw + ((size_t)m_idx << args.log_n);
    r.tw_val = args.tw_val ? args.tw_val + ((size_t)m_idx << args.log_n) : nullptr;
    r.mc = ((const typename A::MC*)args.mc)[m_idx];
    return r;
}

template <class A, int S>
__device__ __forceinline__ void load_lo_tw(const PolyRef<A>& P, u32 T, typename LoTw<A>::TW* tv) {
    if constexpr (std::is_same<A, ArithF64>::value) load_tw_w<S>(P.tw_val, T, tv);
    else load_tw<A, S>(P.tw, T, tv);
}

// ================================ lo pass (contiguous 2^11 blocks) ================================
// positions inside the block: pos = d3*256 + d2*32 + d1*4 + d0 (d3,d2,d1 < 8, d0 < 4)
//   round A: thread = pos % 256,           points over d3          (distances 1024, 512, 256)
//   round B: thread = (d3, pos % 32),      points over d2          (distances 128, 64, 32)
//   round C: thread = (d3, d2, d0),        points over d1          (distances 16, 8, 4)
//   round D: thread = pos / 8,             8 consecutive points    (distances 2, 1)
// A workgroup transforms the same (limb, block) slice of IT consecutive batch items one after the other: the
// slice's twiddles (half as many bytes as the tile itself as values alone, as many with their quotients) are fetched once for
// all of them, and the next item's
// points are requested before the current item's butterflies start, so their latency hides behind a whole
// tile of work.  A buffer is rewritten only after a barrier that every reader of its old contents has passed: the
// forward pass has four exchanges per item (the last one turns each thread's 8 consecutive results into stores of
// 512 contiguous bytes per wave) and uses the two buffers in turn; the inverse pass has three, so its buffers swap
// roles from one item to the next.
template <class A>
__device__ __forceinline__ const u64* item_src(const NttArgs& args, const PolyList& pl, u32 b, u32 a) {
    return (args.use_src_list ? args.src_list.p[b] : args.src + (((size_t)b * args.src_bstride) << args.log_n)) + ((size_t)pl_at(pl.spos, a) << args.log_n);
}
__device__ __forceinline__ u64* item_dst(const NttArgs& args, const PolyList& pl, u32 b, u32 a) {
    return args.dst + (((size_t)b * args.dst_bstride + pl_at(pl.dpos, a)) << args.log_n);
}

// EM (with EPI): which of the optional operands of the division's last step the launch has: 0 = look at each item's pointers,
// 1 = every item has its addend and nothing else, 2 = none has any.  In cases 1 and 2 the step is straight-line code and the
// addend is requested with v, a round ahead of its use; behind a condition the compiler keeps each request next to its use, one
// round trip to memory per point.
template <class A, int IT, bool EPI, int EM = 0>
__device__ __forceinline__ void fwd_lo_body(const NttArgs& args, const PolyList& pl, const FwdEpilogue& ep) {
    typedef typename A::E E;
    __shared__ E lds0[LDS_PADDED_WORDS];
    __shared__ E lds1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(args.log_hi, args.lo_group);
    const u32 blk = tile.blk, b0 = tile.b * IT;
    const u32 cnt = args.batch - b0 < (u32)IT ? args.batch - b0 : (u32)IT;
    const PolyRef<A> P = poly_ref<A>(args, pl, b0, tile.a);
    const size_t off = (size_t)blk << 11;
    const u32 TA = (1u << args.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    typedef typename LoTw<A>::TW TW;
    typedef typename LoTw<A>::AR AR;
    E v[8];
    u64 raw[8];
    TW wa[7], wb[7], wc[7], wd[6];
    load_lo_tw<A, 3>(P, TA, wa);
    load_lo_tw<A, 3>(P, 8 * TA + d3, wb);
    {
        const u64* src = P.src + off;
#pragma unroll
        for (int j = 0; j < 8; j++) raw[j] = src[tid + 256 * j];
    }
#pragma unroll
    for (int it = 0; it < IT; it++) {
        if ((u32)it >= cnt) break;
        E* buf0 = lds0;
        E* buf1 = lds1;
        if (args.first) {
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = A::load_first(raw[j], P.mc, false);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = A::load_mid(raw[j]);
        }
        if (it + 1 < IT && (u32)(it + 1) < cnt) {  // the next item's points, a tile ahead
            const u64* src = item_src<A>(args, pl, b0 + it + 1, tile.a) + off;
#pragma unroll
            for (int j = 0; j < 8; j++) raw[j] = src[tid + 256 * j];
        }
        fwd_rows_pre<AR, 3>(v, wa, P.mc);
        A::fwd_round_end(v, P.mc);
        if (it == 0) load_lo_tw<A, 3>(P, 64 * TA + 8 * d3 + d2, wc);
#pragma unroll
        for (int j = 0; j < 8; j++) buf0[LDS_PAD(tid + 256 * j)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(d3 * 256 + 32 * j + x5)];
        fwd_rows_pre<AR, 3>(v, wb, P.mc);
        A::fwd_round_end(v, P.mc);
        if (it == 0) {
            load_lo_tw<A, 2>(P, 512 * TA + 2 * tid, wd);
            load_lo_tw<A, 2>(P, 512 * TA + 2 * tid + 1, wd + 3);
        }
#pragma unroll
        for (int j = 0; j < 8; j++) buf1[LDS_PAD(d3 * 256 + 32 * j + x5)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)];
        fwd_rows_pre<AR, 3>(v, wc, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) buf0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(8 * tid + j)];
        u64 vv[8], vv2[8], av[8];
        if (EPI) {  // what the results are subtracted from: requested now, needed after the last round
            const u32 bv = b0 + it;
            if (EM == 1) {  // and the addend (gathered through the item's automorphism)
                const FinalItem& fa = ep.B.it[bv >> 1];
                const u64* add = ((bv & 1) ? fa.add1 : fa.add0) + ((size_t)pl_at(pl.dpos, tile.a) << args.log_n);
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const u32 x = (u32)off + tid + 256 * j;
                    av[j] = add[fa.g == 1 ? x : galois_gather_index(x, fa.g, args.log_n)];
                }
            }
            const u64* vrow = (ep.use_vl ? ep.vl.p[bv >> 1] + (bv & 1) * ep.v_cstride + ((size_t)pl_at(pl.dpos, tile.a) << args.log_n)
                                         : ep.v + (((size_t)bv * ep.E + pl_at(pl.dpos, tile.a)) << args.log_n)) + off;
#pragma unroll
            for (int j = 0; j < 8; j++) vv[j] = vrow[tid + 256 * j];
            if constexpr (std::is_same<A, ArithF64>::value) {
                if (ep.use_vl == 2) {
                    const u64* vrow2 = ep.vl2.p[bv >> 1] + (bv & 1) * ep.v2_cstride + ((size_t)pl_at(pl.dpos, tile.a) << args.log_n) + off;
#pragma unroll
                    for (int j = 0; j < 8; j++) vv2[j] = vrow2[tid + 256 * j];
                }
            }
        }
        fwd_rows_pre<AR, 2>(v, wd, P.mc);
        fwd_rows_pre<AR, 2>(v + 4, wd + 3, P.mc);
        A::fwd_round_end(v, P.mc);
        // back through LDS so that a wave stores 512 contiguous bytes per instruction
#pragma unroll
        for (int j = 0; j < 8; j++) buf1[LDS_PAD(8 * tid + j)] = v[j];
        __syncthreads();
        if (!EPI) {
            u64* dst = item_dst(args, pl, b0 + it, tile.a) + off;
#pragma unroll
            for (int j = 0; j < 8; j++) dst[tid + 256 * j] = A::store_fwd_final(buf1[LDS_PAD(tid + 256 * j)], P.mc);
        } else {
            // the division's last step on the results w, which are not stored: out = ((v - w) * cinv + addend) * mask
            const u32 i = pl_at(pl.dpos, tile.a), bb = b0 + it, comp = bb & 1;
            const FinalItem fi = ep.B.it[bb >> 1];
            const u64 cv = ep.cinv[i];
            const u64* add = comp ? fi.add1 : fi.add0;
            u64* orow = fi.out + (((size_t)comp * ep.n_out + i) << args.log_n) + off;
            if constexpr (std::is_same<A, ArithF64>::value) {
                // in the transform's own arithmetic: v - w is an integer below 2q in magnitude, its product with the constant is
                // below 0.75 q, one more reduction after the addend; every value below is exact
                const double q = P.mc.q, cvd = A::from_u64(cv), cvq = cvd / q;
                double vd[8];
                if (ep.use_vl == 2) {  // v = ka * x + kb * y
                    const double ka = A::from_u64(ep.ka[i]), kb = A::from_u64(ep.kb[i]);
#pragma unroll
                    for (int j = 0; j < 8; j++)
                        vd[j] = A::reduce(A::mulmod_any(A::from_u64(vv[j]), ka, q, P.mc.qinv) + A::mulmod_any(A::from_u64(vv2[j]), kb, q, P.mc.qinv), P.mc);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; j++) vd[j] = A::from_u64(vv[j]);
                }
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const u32 p = tid + 256 * j;
                    double r = A::mulmod(vd[j] - buf1[LDS_PAD(p)], cvd, cvq, q);
                    if (EM == 1) {
                        r = A::reduce(r + A::from_u64(av[j]), P.mc);
                    } else if (EM == 0) {
                        if (add) {
                            const u32 x = (u32)off + p;
                            const u32 xs = fi.g == 1 ? x : galois_gather_index(x, fi.g, args.log_n);
                            r = A::reduce(r + A::from_u64(add[((size_t)i << args.log_n) + xs]), P.mc);
                        }
                        if (fi.mask) r = A::mulmod_any(r, A::from_u64(fi.mask[((size_t)i << args.log_n) + off + p]), q, P.mc.qinv);
                        if (fi.acc) r = A::reduce(r + A::from_u64(fi.acc[(((size_t)comp * ep.n_out + i) << args.log_n) + off + p]), P.mc);
                    }
                    orow[p] = A::canonical(r, P.mc);
                }
            } else {
                const ModConst mi = ep.mci[pl_at(pl.mod, tile.a)];
                const u64 cvs = ep.cinv[ep.num_q + i];
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const u32 p = tid + 256 * j;
                    const u64 w = A::store_fwd_final(buf1[LDS_PAD(p)], P.mc);
                    u64 r = mul_shoup(sub_mod(vv[j], w, mi.q), cv, cvs, mi.q);
                    if (EM == 1) {
                        r = add_mod(r, av[j], mi.q);
                    } else if (EM == 0) {
                        if (add) {
                            const u32 x = (u32)off + p;
                            const u32 xs = fi.g == 1 ? x : galois_gather_index(x, fi.g, args.log_n);
                            r = add_mod(r, add[((size_t)i << args.log_n) + xs], mi.q);
                        }
                        if (fi.mask) r = mulmod_barrett(r, fi.mask[((size_t)i << args.log_n) + off + p], mi);
                        if (fi.acc) r = add_mod(r, fi.acc[(((size_t)comp * ep.n_out + i) << args.log_n) + off + p], mi.q);
                    }
                    orow[p] = r;
                }
            }
        }
    }
}

// The plain forward lo pass with the workgroup's batch items in a loop: items tile.b, tile.b + (the grid's extent over
// items), ... of the same 2^11-point slice.  The slice's 27 twiddles per thread are 216 bytes (432 with their quotients) against the 128 bytes of
// an item's points and results, so a workgroup that fetches them for two items still moves more twiddles than data through
// the CU's cache; this one fetches them once for all its items and requests an item's points while the previous one is
// transformed.  Same rounds, same LDS exchanges as fwd_lo_body.
template <class A>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_lo_loop_kernel(NttArgs args, PolyList pl) {
    typedef typename A::E E;
    typedef typename LoTw<A>::TW TW;
    typedef typename LoTw<A>::AR AR;
    __shared__ E lds0[LDS_PADDED_WORDS];
    __shared__ E lds1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(args.log_hi, args.lo_group);
    const u32 b_step = args.lo_group ? gridDim.y : gridDim.x;
    const u32 blk = tile.blk;
    const PolyRef<A> P = poly_ref<A>(args, pl, tile.b, tile.a);
    const size_t off = (size_t)blk << 11;
    const u32 TA = (1u << args.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    E v[8];
    u64 raw[8];
    TW wa[7], wb[7], wc[7], wd[6];
    load_lo_tw<A, 3>(P, TA, wa);
    {
        const u64* src = P.src + off;
#pragma unroll
        for (int j = 0; j < 8; j++) raw[j] = src[tid + 256 * j];
    }
    load_lo_tw<A, 3>(P, 8 * TA + d3, wb);
    load_lo_tw<A, 3>(P, 64 * TA + 8 * d3 + d2, wc);
    load_lo_tw<A, 2>(P, 512 * TA + 2 * tid, wd);
    load_lo_tw<A, 2>(P, 512 * TA + 2 * tid + 1, wd + 3);
    for (u32 b = tile.b; b < args.batch; b += b_step) {
        if (args.first) {
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = A::load_first(raw[j], P.mc, false);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = A::load_mid(raw[j]);
        }
        if (b + b_step < args.batch) {  // the next item's points, a tile ahead
            const u64* src = item_src<A>(args, pl, b + b_step, tile.a) + off;
#pragma unroll
            for (int j = 0; j < 8; j++) raw[j] = src[tid + 256 * j];
        }
        fwd_rows_pre<AR, 3>(v, wa, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) lds0[LDS_PAD(tid + 256 * j)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = lds0[LDS_PAD(d3 * 256 + 32 * j + x5)];
        fwd_rows_pre<AR, 3>(v, wb, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) lds1[LDS_PAD(d3 * 256 + 32 * j + x5)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = lds1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)];
        fwd_rows_pre<AR, 3>(v, wc, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) lds0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = lds0[LDS_PAD(8 * tid + j)];
        fwd_rows_pre<AR, 2>(v, wd, P.mc);
        fwd_rows_pre<AR, 2>(v + 4, wd + 3, P.mc);
        A::fwd_round_end(v, P.mc);
        // back through LDS so that a wave stores 512 contiguous bytes per instruction
#pragma unroll
        for (int j = 0; j < 8; j++) lds1[LDS_PAD(8 * tid + j)] = v[j];
        __syncthreads();
        u64* dst = item_dst(args, pl, b, tile.a) + off;
#pragma unroll
        for (int j = 0; j < 8; j++) dst[tid + 256 * j] = A::store_fwd_final(lds1[LDS_PAD(tid + 256 * j)], P.mc);
        // (no barrier between items: the next item's first exchange writes lds0, whose last read is behind the barrier above,
        // and its first barrier stands between these reads of lds1 and the next writes to it)
    }
}

// the lo pass as the last kernel of a division by dropped moduli
template <class A, int IT, int EM>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_lo_div_kernel(NttArgs args, PolyList pl, FwdEpilogue ep) {
    fwd_lo_body<A, IT, true, EM>(args, pl, ep);
}

// The lo pass of ModUp's forward transforms with the inner product with the switching key in place of its stores.
// A workgroup owns one 2^11-point slice of one position e of the extended basis of one batch item: it transforms that
// slice of every digit whose limb e went through the converting hi pass (all live digits but the one e belongs to; the
// slice's twiddles are fetched once for all of them), multiplies each result by the two key words of (digit, e) as it
// comes out, adds the product of the digit that owns e (its limb is the decomposed polynomial's own, never transformed)
// and stores the two components of the inner product: the extended
// digits are never written in evaluation form nor read back.  All sums are exact integers in doubles (at most
// beta + 1 terms below 0.75 q each).
struct MacEpilogue {
    DigitSrc D;           // D.digits: rows (j*E + e) hold the hi pass' output (doubles); D.own: the decomposed polynomials
    PtrList8 key;         // per batch item: [dnum][2][M][N] (the same pointer for a shared key)
    OutList8 out;         // per batch item: [2][E][N]
    const u64* negp;      // [num_q]: -P mod q_i
    u32 level, M, E, beta;
    // prod != 0: the decomposed polynomial is d2 = a1 (.) b1 of the ciphertext product (a0, a1) x (b0, b1), which exists
    // nowhere in evaluation form: the own-limb term is formed from a1, b1 ([level+1][N] each, per batch item), and the
    // addends are d0 = a0 (.) b0 and d1 = a0 (.) b1 + a1 (.) b0 (D.own is not read)
    PtrList8 a0, a1, b0, b1;
    u32 prod, lin;
    // lin != 0 (with prod): the addends are ka * x + kb * y of two more ciphertexts (component 1 at + x_cstride, y_cstride)
    PtrList8 lx, ly;
    size_t x_cstride, y_cstride;
    u64 ka[CKKS_MAX_MODULI], kb[CKKS_MAX_MODULI];
};

// PROD, LIN: ep.prod, ep.lin.  They are template arguments so that what follows the digits is straight-line code: with the
// operands behind conditions, even ones that are the same for the whole launch, the compiler keeps each request next to its
// use, one round trip to memory per point.
template <bool PROD, bool LIN>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_lo_mac_kernel(NttArgs args, PolyList pl, MacEpilogue ep) {
    typedef ArithF64 A;
    typedef double E;
    __shared__ E lds0[LDS_PADDED_WORDS];
    __shared__ E lds1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(args.log_hi, args.lo_group);
    const u32 blk = tile.blk, e = tile.a, m_idx = pl_at(pl.mod, e);
    // the batch items of this workgroup: tile.b, tile.b + (the grid's extent over items), ...: a workgroup that takes several
    // fetches the slice's twiddles (half as many bytes as an item's points) once for all of them and requests an item's first
    // points before it is done with the previous item
    const u32 b_step = args.lo_group ? gridDim.y : gridDim.x;
    const size_t N = (size_t)1 << args.log_n, off = (size_t)blk << 11;
    const double* tw = args.tw_val + ((size_t)m_idx << args.log_n);
    const ModConstF mc = ((const ModConstF*)args.mc)[m_idx];
    const u32 own = e <= ep.level ? e / ep.D.alpha : 0xffffffffu;  // the digit that limb e belongs to
    const u32 TA = (1u << args.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    const size_t kstride = (size_t)ep.M * N;  // between the b and the a part of a digit's key; two of them per digit
    const size_t dstride = (size_t)ep.E * N;
    typedef ArithF64W AW;
    double wa[7], wb[7], wc[7], wd[6];  // the slice's twiddles, fetched once for all digits of all items
    load_tw_w<3>(tw, TA, wa);
    load_tw_w<3>(tw, 8 * TA + d3, wb);
    load_tw_w<3>(tw, 64 * TA + 8 * d3 + d2, wc);
    load_tw_w<2>(tw, 512 * TA + 2 * tid, wd);
    load_tw_w<2>(tw, 512 * TA + 2 * tid + 1, wd + 3);
    const u32 j0 = own == 0 ? 1 : 0;  // first digit to transform
    E v[8], raw[8];
    if (j0 < ep.beta) {
        const double* hi0 = (const double*)(ep.D.digits + tile.b * ep.D.bstride) + (size_t)e * N + off;
#pragma unroll
        for (int i = 0; i < 8; i++) raw[i] = hi0[(size_t)j0 * dstride + tid + 256 * i];
    }
    for (u32 b = tile.b; b < args.batch; b += b_step) {
    const u64* key = ep.key.p[b] + (size_t)m_idx * N + off;
    const double* hi = (const double*)(ep.D.digits + b * ep.D.bstride) + (size_t)e * N + off;
    E acc0[8], acc1[8];
#pragma unroll
    for (int j = 0; j < 8; j++) acc0[j] = acc1[j] = 0.0;
    u32 j = j0;
    while (j < ep.beta) {
        u32 jn = j + 1;
        if (jn == own) jn++;
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = raw[i];
        if (jn < ep.beta) {  // the next digit's points, a tile ahead
#pragma unroll
            for (int i = 0; i < 8; i++) raw[i] = hi[(size_t)jn * dstride + tid + 256 * i];
        }
        fwd_rows_pre<AW, 3>(v, wa, mc);
        A::fwd_round_end(v, mc);
#pragma unroll
        for (int i = 0; i < 8; i++) lds0[LDS_PAD(tid + 256 * i)] = v[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = lds0[LDS_PAD(d3 * 256 + 32 * i + x5)];
        fwd_rows_pre<AW, 3>(v, wb, mc);
        A::fwd_round_end(v, mc);
#pragma unroll
        for (int i = 0; i < 8; i++) lds1[LDS_PAD(d3 * 256 + 32 * i + x5)] = v[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = lds1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * i + d0)];
        fwd_rows_pre<AW, 3>(v, wc, mc);
        A::fwd_round_end(v, mc);
#pragma unroll
        for (int i = 0; i < 8; i++) lds0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * i + d0)] = v[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = lds0[LDS_PAD(8 * tid + i)];
        // the key words of this digit at the points this thread ends up with: requested now, needed after the last round
        u64 k0[8], k1[8];
        {
            const u64* kj = key + (size_t)j * 2 * kstride;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                k0[i] = kj[tid + 256 * i];
                k1[i] = kj[kstride + tid + 256 * i];
            }
        }
        fwd_rows_pre<AW, 2>(v, wd, mc);
        fwd_rows_pre<AW, 2>(v + 4, wd + 3, mc);
        A::fwd_round_end(v, mc);
        // back through LDS: point tid + 256 i of the slice, where the key words were fetched
#pragma unroll
        for (int i = 0; i < 8; i++) lds1[LDS_PAD(8 * tid + i)] = v[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const double y = lds1[LDS_PAD(tid + 256 * i)];
            acc0[i] += A::mulmod_any(y, A::from_u64(k0[i]), mc.q, mc.qinv);
            acc1[i] += A::mulmod_any(y, A::from_u64(k1[i]), mc.q, mc.qinv);
        }
        j = jn;
    }
    // the next item's first points: requested before the operands of what follows, or, where those leave no registers (the
    // linear combination's twelve operands per point), after them
    auto request_next = [&]() {
        if (b + b_step < args.batch && j0 < ep.beta) {
            const double* hin = (const double*)(ep.D.digits + (b + b_step) * ep.D.bstride) + (size_t)e * N + off;
#pragma unroll
            for (int i = 0; i < 8; i++) raw[i] = hin[(size_t)j0 * dstride + tid + 256 * i];
        }
    };
    if (!LIN) request_next();
    if (PROD && e <= ep.level) {
        // the tensor product of this slice, formed here: d2 feeds the digit that owns the limb, P d0 and P d1 join the sums
        const u64* kj = key + (size_t)own * 2 * kstride;
        const size_t po = (size_t)e * N + off;
        const u64 *pa0 = ep.a0.p[b] + po, *pa1 = ep.a1.p[b] + po, *pb0 = ep.b0.p[b] + po, *pb1 = ep.b1.p[b] + po;
        const double pres = mc.q - A::from_u64(ep.negp[e]);  // P mod q_e
        const u64* lx = LIN ? ep.lx.p[b] + po : nullptr;
        const u64* ly = LIN ? ep.ly.p[b] + po : nullptr;
        const double ka = LIN ? A::from_u64(ep.ka[e]) : 0.0, kb = LIN ? A::from_u64(ep.kb[e]) : 0.0;
        // four points at a time (two with the linear combination: the twiddles stay in registers for the next item and leave
        // room for 24 operands): six to ten operands per point, requested before the first is used
        constexpr int HP = LIN ? 2 : 4;
#pragma unroll
        for (int h = 0; h < 8; h += HP) {
            u64 ra0[HP], ra1[HP], rb0[HP], rb1[HP], rk0[HP], rk1[HP], rx0[HP], rx1[HP], ry0[HP], ry1[HP];
#pragma unroll
            for (int i = 0; i < HP; i++) {
                const u32 x = tid + 256 * (h + i);
                ra0[i] = pa0[x], ra1[i] = pa1[x], rb0[i] = pb0[x], rb1[i] = pb1[x];
                rk0[i] = kj[x], rk1[i] = kj[kstride + x];
                if (LIN) rx0[i] = lx[x], rx1[i] = lx[ep.x_cstride + x], ry0[i] = ly[x], ry1[i] = ly[ep.y_cstride + x];
            }
#pragma unroll
            for (int i = 0; i < HP; i++) {
                const double A0 = A::from_u64(ra0[i]), A1 = A::from_u64(ra1[i]), B0 = A::from_u64(rb0[i]), B1 = A::from_u64(rb1[i]);
                const double dd2 = A::mulmod_any(A1, B1, mc.q, mc.qinv);
                double dd0 = A::mulmod_any(A0, B0, mc.q, mc.qinv);
                double dd1 = A::mulmod_any(A0, B1, mc.q, mc.qinv) + A::mulmod_any(A1, B0, mc.q, mc.qinv);
                if (LIN) {  // at most 0.75 q more per term: both sums stay below 2^53
                    dd0 += A::mulmod_any(A::from_u64(rx0[i]), ka, mc.q, mc.qinv) + A::mulmod_any(A::from_u64(ry0[i]), kb, mc.q, mc.qinv);
                    dd1 += A::mulmod_any(A::from_u64(rx1[i]), ka, mc.q, mc.qinv) + A::mulmod_any(A::from_u64(ry1[i]), kb, mc.q, mc.qinv);
                }
                dd0 = A::reduce(dd0, mc);  // back below q / 2 + 1 as multiplicands
                dd1 = A::reduce(dd1, mc);
                acc0[h + i] += A::mulmod_any(dd2, A::from_u64(rk0[i]), mc.q, mc.qinv) + A::mulmod_any(dd0, pres, mc.q, mc.qinv);
                acc1[h + i] += A::mulmod_any(dd2, A::from_u64(rk1[i]), mc.q, mc.qinv) + A::mulmod_any(dd1, pres, mc.q, mc.qinv);
            }
        }
    } else if (!PROD && e <= ep.level) {
        // the digit that owns this limb
        const u64* kj = key + (size_t)own * 2 * kstride;
        const u64* yo = ep.D.own.p[b] + (size_t)e * N + off;
        u64 ry[8], rk0[8], rk1[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const u32 x = tid + 256 * i;
            ry[i] = yo[x], rk0[i] = kj[x], rk1[i] = kj[kstride + x];
        }
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const double y = A::from_u64(ry[i]);
            acc0[i] += A::mulmod_any(y, A::from_u64(rk0[i]), mc.q, mc.qinv);
            acc1[i] += A::mulmod_any(y, A::from_u64(rk1[i]), mc.q, mc.qinv);
        }
    }
    if (LIN) request_next();
    u64* o0 = ep.out.p[b] + (size_t)e * N + off;
    u64* o1 = o0 + (size_t)ep.E * N;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        o0[tid + 256 * i] = A::canonical(A::reduce(acc0[i], mc), mc);
        o1[tid + 256 * i] = A::canonical(A::reduce(acc1[i], mc), mc);
    }
    // (no barrier between items: the next item's first exchange writes lds0, and its barrier stands between the last item's
    // reads of lds1 and the next writes to it)
    }
}

// MUL (double-precision arithmetic, first pass, source list): the transform's input is the pointwise product of two
// polynomials (the d2 = a1 (.) b1 of a ciphertext product), formed as the points are loaded: d2 itself is never stored.
template <class A, int IT, bool MUL = false>
__global__ __launch_bounds__(NTT_THREADS) __attribute__((amdgpu_waves_per_eu(3, 8))) void ntt_inv_lo_kernel(NttArgs args, PolyList pl) {
    typedef typename A::E E;
    __shared__ E lds0[LDS_PADDED_WORDS];
    __shared__ E lds1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(args.log_hi, args.lo_group);
    const u32 blk = tile.blk, b0 = tile.b * IT;
    const u32 cnt = args.batch - b0 < (u32)IT ? args.batch - b0 : (u32)IT;
    const PolyRef<A> P = poly_ref<A>(args, pl, b0, tile.a);
    const size_t off = (size_t)blk << 11;
    const u32 TA = (1u << args.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    typedef typename LoTw<A>::TW TW;
    typedef typename LoTw<A>::AR AR;
    E v[8];
    ulonglong2 raw[4], raw2[MUL ? 4 : 1];
    TW wa[7], wb[7], wc[7], wd[6];
    load_lo_tw<A, 2>(P, 512 * TA + 2 * tid, wd);
    load_lo_tw<A, 2>(P, 512 * TA + 2 * tid + 1, wd + 3);
    load_lo_tw<A, 3>(P, 64 * TA + 8 * d3 + d2, wc);
    const size_t moff = ((size_t)pl_at(pl.spos, tile.a) << args.log_n) + off + 8 * tid;  // MUL: the multiplier's point
    {
        const ulonglong2* in = reinterpret_cast<const ulonglong2*>(P.src + off + 8 * tid);
#pragma unroll
        for (int j = 0; j < 4; j++) raw[j] = in[j];
        if constexpr (MUL) {
            const ulonglong2* in2 = reinterpret_cast<const ulonglong2*>(args.mul_list.p[b0] + moff);
#pragma unroll
            for (int j = 0; j < 4; j++) raw2[j] = in2[j];
        }
    }
#pragma unroll
    for (int it = 0; it < IT; it++) {
        if ((u32)it >= cnt) break;
        E* buf0 = (it & 1) ? lds1 : lds0;  // three exchanges per item: the buffers swap roles from item to item
        E* buf1 = (it & 1) ? lds0 : lds1;
        if constexpr (MUL) {
            if (args.use_lin) {  // uniform
                const double ka = A::from_u64(args.lin_ka), kb = A::from_u64(args.lin_kb);
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    v[2 * j] = A::reduce(A::mulmod_any(A::from_u64(raw[j].x), ka, P.mc.q, P.mc.qinv) +
                                         A::mulmod_any(A::from_u64(raw2[j].x), kb, P.mc.q, P.mc.qinv), P.mc);
                    v[2 * j + 1] = A::reduce(A::mulmod_any(A::from_u64(raw[j].y), ka, P.mc.q, P.mc.qinv) +
                                             A::mulmod_any(A::from_u64(raw2[j].y), kb, P.mc.q, P.mc.qinv), P.mc);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    v[2 * j] = A::mulmod_any(A::from_u64(raw[j].x), A::from_u64(raw2[j].x), P.mc.q, P.mc.qinv);
                    v[2 * j + 1] = A::mulmod_any(A::from_u64(raw[j].y), A::from_u64(raw2[j].y), P.mc.q, P.mc.qinv);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[2 * j] = A::load_first(raw[j].x, P.mc, true);
                v[2 * j + 1] = A::load_first(raw[j].y, P.mc, true);
            }
        }
        if (it + 1 < IT && (u32)(it + 1) < cnt) {  // the next item's points, a tile ahead
            const ulonglong2* in = reinterpret_cast<const ulonglong2*>(item_src<A>(args, pl, b0 + it + 1, tile.a) + off + 8 * tid);
#pragma unroll
            for (int j = 0; j < 4; j++) raw[j] = in[j];
            if constexpr (MUL) {
                const ulonglong2* in2 = reinterpret_cast<const ulonglong2*>(args.mul_list.p[b0 + it + 1] + moff);
#pragma unroll
                for (int j = 0; j < 4; j++) raw2[j] = in2[j];
            }
        }
        inv_rows_pre<AR, 2>(v, wd, P.mc);
        inv_rows_pre<AR, 2>(v + 4, wd + 3, P.mc);
        if (it == 0) load_lo_tw<A, 3>(P, 8 * TA + d3, wb);
#pragma unroll
        for (int j = 0; j < 8; j++) buf0[LDS_PAD(8 * tid + j)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)];
        inv_rows_pre<AR, 3>(v, wc, P.mc);
        if (it == 0) load_lo_tw<A, 3>(P, TA, wa);
#pragma unroll
        for (int j = 0; j < 8; j++) buf1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf1[LDS_PAD(d3 * 256 + 32 * j + x5)];
        inv_rows_pre<AR, 3>(v, wb, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) buf0[LDS_PAD(d3 * 256 + 32 * j + x5)] = v[j];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(tid + 256 * j)];
        inv_rows_pre<AR, 3>(v, wa, P.mc);
        u64* dst = item_dst(args, pl, b0 + it, tile.a) + off;
        if (args.last) {
#pragma unroll
            for (int j = 0; j < 8; j++) dst[tid + 256 * j] = A::store_inv_final(v[j], P.mc);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) dst[tid + 256 * j] = A::store_mid(v[j]);  // the hi pass follows
        }
    }
}

// ============================ hi pass (rows 2^11 apart, adjacent columns) ============================
// tile = R = 2^LOG_HI rows x CC = 2048/R columns; element (row, col) lives at (row << 11) + col0 + col.
// LOG_HI <= 3: a thread holds all R rows of 8/R columns (no exchange).
// LOG_HI >= 4: round 1 = radix 8 over rows r0 + (R/8)*j of one column; exchange through LDS;
//              round 2 = the remaining LOG_HI-3 stages over R/8 consecutive rows of 64/R adjacent columns.
// The forward hi pass is the first pass of a transform (reads canonical residues, writes the
// intermediate form); the inverse hi pass is the last one.
template <class A, int LOG_HI>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_hi_kernel(NttArgs args, PolyList pl) {
    typedef typename A::E E;
    constexpr int R = 1 << LOG_HI, CC = NTT_TILE / R;
    const u32 tid = threadIdx.x;
    const PolyRef<A> P = poly_ref<A>(args, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    const u64* src = P.src + (size_t)blockIdx.x * CC;
    u64* dst = P.dst + (size_t)blockIdx.x * CC;
    E v[8];
    if constexpr (LOG_HI <= 3) {
        constexpr int KC = 8 / R;
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) v[rr * KC + kc] = A::load_first(src[((size_t)rr << 11) + kc * 256 + tid], P.mc, false);
        fwd_rows<A, LOG_HI, KC>(v, P.tw, 1, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) dst[((size_t)rr << 11) + kc * 256 + tid] = A::store_mid(v[rr * KC + kc]);
    } else {
        __shared__ __attribute__((aligned(16))) E lds[NTT_TILE];
        constexpr int R8 = R / 8, S2 = LOG_HI - 3, KC2 = 8 / R8;
        const u32 r0 = tid / CC, col = tid % CC;
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = A::load_first(src[((size_t)(r0 + R8 * j) << 11) + col], P.mc, false);
        fwd_rows<A, 3, 1>(v, P.tw, 1, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) lds[(r0 + R8 * j) * CC + col] = v[j];
        __syncthreads();
        const u32 G = tid >> 5, cg = tid & 31;
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) v[rr * KC2 + kc] = lds[(G * R8 + rr) * CC + cg * KC2 + kc];
        fwd_rows<A, S2, KC2>(v, P.tw, 8 + G, P.mc);
        A::fwd_round_end(v, P.mc);
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) dst[((size_t)(G * R8 + rr) << 11) + cg * KC2 + kc] = A::store_mid(v[rr * KC2 + kc]);
    }
}

// The forward hi pass with a basis conversion (ModUp's or ModDown's) in front of it: the points of the target limb at
// position e = pl.dpos[a] are
//   sum_i yhat_i * [B/b_i]_{q_e}  mod q_e
// evaluated from the source basis' centred residues yhat (doubles, nd limbs from position lo of each batch item of y)
// as the tile is loaded: the converted polynomial is never written in coefficient form.
// convf: [position][ap] (constant, constant / q_e), rows padded with zeros to ap = 4, 8, 12 or 16 entries.
struct ConvPrologue {
    const double* y;
    size_t y_bstride;  // elements
    const TwF* convf;
    u32 lo, nd;
    u32 ap, pad;
};

// the source residues of one point: no branch around the loads (entries beyond the nd source limbs re-read the last
// one against a zero constant)
// ND <= AP: the entries that are read and multiplied (a row of the constants has AP, the last AP - ND of them zero)
template <int AP, int ND>
__device__ __forceinline__ void conv_load(double (&yv)[AP], const double* __restrict__ yp, size_t N, u32 nd) {
#pragma unroll
    for (int a = 0; a < ND; a++) yv[a] = yp[(size_t)((u32)a < nd ? a : nd - 1) * N];
}
template <int AP, int ND>
__device__ __forceinline__ double conv_sum(const double (&yv)[AP], const double* cw, double q, double qinv) {
    static_assert(ND <= 8 || AP > 8, "rows of more than eight entries are padded to twelve or sixteen");
    return f64m_dot_w<ND>(yv, cw, q, qinv);
}

// One workgroup converts and transforms the same tile of T target limbs: the source residues are fetched once for all T
// (the fetch, from L2 after the first, is what bounds a one-target-per-workgroup version).
template <int LOG_HI, int AP, int T, int ND = AP>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_hi_conv_kernel(NttArgs args, PolyList pl, ConvPrologue cp) {
    typedef ArithF64 A;
    typedef double E;
    constexpr int R = 1 << LOG_HI, CC = NTT_TILE / R;
    const u32 groups = (pl.n + T - 1) / T;
    const u32 tid = threadIdx.x, tile = blockIdx.x, b = blockIdx.y / groups, a0 = (blockIdx.y % groups) * T;
    const size_t N = (size_t)1 << args.log_n;
    const double* y = cp.y + b * cp.y_bstride + (size_t)cp.lo * N + (size_t)tile * CC;
    PolyRef<A> P[T];
    double cw[T][ND];  // the centred constants (the tables' quotients by the modulus are not read)
#pragma unroll
    for (int t = 0; t < T; t++) {
        const u32 a_idx = a0 + t < pl.n ? a0 + t : pl.n - 1;  // a ragged last group repeats its last limb and skips the store
        P[t] = poly_ref<A, true>(args, pl, b, a_idx);
        const TwF* ce = cp.convf + (size_t)pl.dpos[a_idx] * AP;
#pragma unroll
        for (int a = 0; a < ND; a++) cw[t][a] = ce[a].w;
    }
    E v[T][8];
    if constexpr (LOG_HI <= 3) {
        constexpr int KC = 8 / R;
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) {
                double yv[AP];
                conv_load<AP, ND>(yv, y + ((size_t)rr << 11) + kc * 256 + tid, N, cp.nd);
#pragma unroll
                for (int t = 0; t < T; t++) v[t][rr * KC + kc] = conv_sum<AP, ND>(yv, cw[t], P[t].mc.q, P[t].mc.qinv);
            }
#pragma unroll
        for (int t = 0; t < T; t++) {
            if (a0 + t >= pl.n) break;
            u64* dst = P[t].dst + (size_t)tile * CC;
            fwd_rows<A, LOG_HI, KC>(v[t], P[t].tw, 1, P[t].mc);
            A::fwd_round_end(v[t], P[t].mc);
#pragma unroll
            for (int rr = 0; rr < R; rr++)
#pragma unroll
                for (int kc = 0; kc < KC; kc++) dst[((size_t)rr << 11) + kc * 256 + tid] = A::store_mid(v[t][rr * KC + kc]);
        }
    } else {
        __shared__ __attribute__((aligned(16))) E lds[NTT_TILE];
        constexpr int R8 = R / 8, S2 = LOG_HI - 3, KC2 = 8 / R8;
        const u32 r0 = tid / CC, col = tid % CC;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            double yv[AP];
            conv_load<AP, ND>(yv, y + ((size_t)(r0 + R8 * j) << 11) + col, N, cp.nd);
#pragma unroll
            for (int t = 0; t < T; t++) v[t][j] = conv_sum<AP, ND>(yv, cw[t], P[t].mc.q, P[t].mc.qinv);
        }
        const u32 G = tid >> 5, cg = tid & 31;
#pragma unroll
        for (int t = 0; t < T; t++) {
            if (a0 + t >= pl.n) break;  // uniform over the workgroup
            u64* dst = P[t].dst + (size_t)tile * CC;
            if (t) __syncthreads();  // the previous limb's exchange has been read
            fwd_rows<A, 3, 1>(v[t], P[t].tw, 1, P[t].mc);
            A::fwd_round_end(v[t], P[t].mc);
#pragma unroll
            for (int j = 0; j < 8; j++) lds[(r0 + R8 * j) * CC + col] = v[t][j];
            __syncthreads();
#pragma unroll
            for (int rr = 0; rr < R8; rr++)
#pragma unroll
                for (int kc = 0; kc < KC2; kc++) v[t][rr * KC2 + kc] = lds[(G * R8 + rr) * CC + cg * KC2 + kc];
            fwd_rows<A, S2, KC2>(v[t], P[t].tw, 8 + G, P[t].mc);
            A::fwd_round_end(v[t], P[t].mc);
#pragma unroll
            for (int rr = 0; rr < R8; rr++)
#pragma unroll
                for (int kc = 0; kc < KC2; kc++) dst[((size_t)(G * R8 + rr) << 11) + cg * KC2 + kc] = A::store_mid(v[t][rr * KC2 + kc]);
        }
    }
}

// The inverse transform's last store: times 1/N, canonical; or (double-precision arithmetic only) times *scale and centred,
// as a double: |t| < 0.75 q after the exact product, so the centred representative is t, t - q or t + q.
template <class A>
__device__ __forceinline__ u64 inv_last_store(typename A::E v, const typename A::MC& m, const TwF* scale) {
    if constexpr (std::is_same<A, ArithF64>::value) {
        if (scale) {
            const TwF k = *scale;
            const double t = f64m_centre(ArithF64::mulmod(v, k.w, k.wq, m.q), m.q);
            return (u64)__double_as_longlong(t);
        }
    }
    return A::store_inv_final(v, m);
}

template <class A, int LOG_HI>
__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_hi_kernel(NttArgs args, PolyList pl) {
    typedef typename A::E E;
    constexpr int R = 1 << LOG_HI, CC = NTT_TILE / R;
    const u32 tid = threadIdx.x;
    const PolyRef<A> P = poly_ref<A>(args, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    u64* dst = P.dst + (size_t)blockIdx.x * CC;  // the lo pass has already moved the data to dst
    const TwF* scale = args.inv_scale ? args.inv_scale + pl_at(pl.mod, blockIdx.y % pl.n) : nullptr;
    E v[8];
    if constexpr (LOG_HI <= 3) {
        constexpr int KC = 8 / R;
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) v[rr * KC + kc] = A::load_mid(dst[((size_t)rr << 11) + kc * 256 + tid]);
        inv_rows<A, LOG_HI, KC>(v, P.tw, 1, P.mc);
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) dst[((size_t)rr << 11) + kc * 256 + tid] = inv_last_store<A>(v[rr * KC + kc], P.mc, scale);
    } else {
        __shared__ __attribute__((aligned(16))) E lds[NTT_TILE];
        constexpr int R8 = R / 8, S2 = LOG_HI - 3, KC2 = 8 / R8;
        const u32 G = tid >> 5, cg = tid & 31;
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) v[rr * KC2 + kc] = A::load_mid(dst[((size_t)(G * R8 + rr) << 11) + cg * KC2 + kc]);
        inv_rows<A, S2, KC2>(v, P.tw, 8 + G, P.mc);
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) lds[(G * R8 + rr) * CC + cg * KC2 + kc] = v[rr * KC2 + kc];
        __syncthreads();
        const u32 r0 = tid / CC, col = tid % CC;
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = lds[(r0 + R8 * j) * CC + col];
        inv_rows<A, 3, 1>(v, P.tw, 1, P.mc);
#pragma unroll
        for (int j = 0; j < 8; j++) dst[((size_t)(r0 + R8 * j) << 11) + col] = inv_last_store<A>(v[j], P.mc, scale);
    }
}

// ================================= rings below 2^11: one tile per poly (integer arithmetic) ==============
template <bool INVERSE>
__global__ __launch_bounds__(NTT_THREADS) void ntt_small_kernel(NttArgs args, PolyList pl) {
    typedef ArithU64 A;
    __shared__ u64 lds[NTT_TILE];
    const u32 tid = threadIdx.x;
    const PolyRef<A> P = poly_ref<A>(args, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    const u32 n = 1u << args.log_n;
    for (u32 e = tid; e < n; e += NTT_THREADS) lds[e] = P.src[e];
    __syncthreads();
    for (u32 st = 0; st < args.log_n; st++) {
        const u32 r = INVERSE ? args.log_n - 1 - st : st;  // stage with 2^r groups
        const u32 lt = args.log_n - 1 - r;                 // log2 of the pair distance
        for (u32 bf = tid; bf < n / 2; bf += NTT_THREADS) {
            const u32 i = bf >> lt;
            const u32 i0 = (i << (lt + 1)) + (bf & ((1u << lt) - 1)), i1 = i0 + (1u << lt);
            u64 x = lds[i0], y = lds[i1];
            if (INVERSE) A::inv_bf(x, y, P.tw[(1u << r) + i], P.mc); else A::fwd_bf(x, y, P.tw[(1u << r) + i], P.mc);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    for (u32 e = tid; e < n; e += NTT_THREADS) P.dst[e] = INVERSE ? A::store_inv_final(lds[e], P.mc) : A::store_fwd_final(lds[e], P.mc);
}

template <class A, int LOG_HI>
static void launch_hi(bool inverse, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl) {
    if (inverse) hipLaunchKernelGGL((ntt_inv_hi_kernel<A, LOG_HI>), grid, dim3(NTT_THREADS), 0, st, args, pl);
    else hipLaunchKernelGGL((ntt_fwd_hi_kernel<A, LOG_HI>), grid, dim3(NTT_THREADS), 0, st, args, pl);
}

template <class A>
static void launch_hi_any(u32 log_hi, bool inverse, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl) {
    switch (log_hi) {
        case 1: launch_hi<A, 1>(inverse, grid, st, args, pl); break;
        case 2: launch_hi<A, 2>(inverse, grid, st, args, pl); break;
        case 3: launch_hi<A, 3>(inverse, grid, st, args, pl); break;
        case 4: launch_hi<A, 4>(inverse, grid, st, args, pl); break;
        case 5: launch_hi<A, 5>(inverse, grid, st, args, pl); break;
        default: launch_hi<A, 6>(inverse, grid, st, args, pl); break;
    }
}

template <class A, int IT>
static void launch_inv_lo_it(dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl, bool mul = false) {
    if constexpr (std::is_same<A, ArithF64>::value && IT == 1) {  // the product-forming variant takes one item
        if (mul) {
            hipLaunchKernelGGL((ntt_inv_lo_kernel<A, IT, true>), grid, dim3(NTT_THREADS), 0, st, args, pl);
            return;
        }
    }
    hipLaunchKernelGGL((ntt_inv_lo_kernel<A, IT>), grid, dim3(NTT_THREADS), 0, st, args, pl);
}
// The plain forward lo pass: workgroups that loop over their items, up to eight each (measured at N = 2^16: 2, 4, 8 and 16
// items give 2.04, 2.06, 2.08 and 2.10e6 limb transforms per second against 1.97e6 with one fetch of the twiddles per two
// items; eight still leaves the layer's batches of eight a grid of one workgroup per slice).  `grid` is a lo pass' grid,
// whose extent over items is set here.
template <class A>
static void launch_fwd_lo_loop(u32 batch, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl) {
    constexpr u32 per_wg = 8;
    const u32 ext = (batch + per_wg - 1) / per_wg;
    if (args.lo_group) grid.y = ext;
    else grid.x = ext;
    hipLaunchKernelGGL((ntt_fwd_lo_loop_kernel<A>), grid, dim3(NTT_THREADS), 0, st, args, pl);
}
template <class A>
static void launch_lo_div(dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl, const FwdEpilogue& ep) {
    // which optional operands the division's last step has is the same for the whole launch: one instantiation per case
    u32 n_add = 0, n_other = 0;
    const u32 n_ct = (args.batch + 1) / 2;
    for (u32 r = 0; r < n_ct; r++) {
        const FinalItem& fi = ep.B.it[r];
        n_add += (fi.add0 ? 1 : 0) + (fi.add1 ? 1 : 0);
        n_other += (fi.mask ? 1 : 0) + (fi.acc ? 1 : 0);
    }
    const int em = n_other ? 0 : (n_add == 2 * n_ct ? 1 : (n_add == 0 ? 2 : 0));
    // one batch item per workgroup (see lo_items in launch_ntt_any)
#define LO_DIV_LAUNCH(EM) hipLaunchKernelGGL((ntt_fwd_lo_div_kernel<A, 1, EM>), grid, dim3(NTT_THREADS), 0, st, args, pl, ep)
    if (em == 1) LO_DIV_LAUNCH(1);
    else if (em == 2) LO_DIV_LAUNCH(2);
    else LO_DIV_LAUNCH(0);
#undef LO_DIV_LAUNCH
}
template <class A>
static void launch_inv_lo(u32 items, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl, bool mul = false) {
    if (items == 2 && !mul) launch_inv_lo_it<A, 2>(grid, st, args, pl, false);
    else launch_inv_lo_it<A, 1>(grid, st, args, pl, mul);
}

// Target limbs per workgroup of the converting hi pass: four, or six where there are many of them and the ring is large (the
// source residues are fetched by four workgroups instead of six for 24 targets; the pass takes as long by itself and leaves
// more of the chip to the other stream's kernels: 0.5 ms per step of the block slice; with few targets or small launches the
// larger groups cost parallelism)
// (not for the one-term "conversion" of the rescale, which has no arithmetic to share: 36 us with four, 41 with six)
static u32 conv_targets(u32 log_hi, u32 n_targets, u32 nd) { return (log_hi >= 4 && n_targets >= 12 && nd > 1) ? 6 : 4; }
template <int LOG_HI, int T>
static void launch_hi_conv_ap(u32 ap, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl, const ConvPrologue& cp) {
    if (ap == 4 && cp.nd == 1)  // the rescale: one dropped limb
        hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 4, T, 1>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
    else if (ap == 4) hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 4, T>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
    else if (ap == 8) hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 8, T>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
    else if (ap == 12 && cp.nd == 9)  // eight special primes and the dropped limb: three of the twelve entries are padding
        hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 12, T, 9>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
    else if (ap == 12) hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 12, T>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
    else hipLaunchKernelGGL((ntt_fwd_hi_conv_kernel<LOG_HI, 16, T>), grid, dim3(NTT_THREADS), 0, st, args, pl, cp);
}
static void launch_hi_conv(u32 log_hi, u32 ap, dim3 grid, hipStream_t st, const NttArgs& args, const PolyList& pl, const ConvPrologue& cp) {
    const bool six = conv_targets(log_hi, pl.n, cp.nd) == 6;
    switch (log_hi) {
        case 1: launch_hi_conv_ap<1, 4>(ap, grid, st, args, pl, cp); break;
        case 2: launch_hi_conv_ap<2, 4>(ap, grid, st, args, pl, cp); break;
        case 3: launch_hi_conv_ap<3, 4>(ap, grid, st, args, pl, cp); break;
        case 4: six ? launch_hi_conv_ap<4, 6>(ap, grid, st, args, pl, cp) : launch_hi_conv_ap<4, 4>(ap, grid, st, args, pl, cp); break;
        case 5: six ? launch_hi_conv_ap<5, 6>(ap, grid, st, args, pl, cp) : launch_hi_conv_ap<5, 4>(ap, grid, st, args, pl, cp); break;
        default: six ? launch_hi_conv_ap<6, 6>(ap, grid, st, args, pl, cp) : launch_hi_conv_ap<6, 4>(ap, grid, st, args, pl, cp); break;
    }
}

static hipError_t launch_ntt_any(const ckks_ctx* c, bool inverse, const u64* src, size_t src_bstride, u64* dst,
                                 size_t dst_bstride, const PolyList& pl, u32 batch, hipStream_t st, const u64* const* src_ptrs,
                                 const FwdEpilogue* epilogue, const TwF* inv_scale, const ConvPrologue* conv, bool hi_only = false,
                                 const u64* const* mul_ptrs = nullptr, const u64* lin_k = nullptr) {
    if (pl.n == 0 || batch == 0) return hipSuccess;
    if (mul_ptrs && (!inverse || !src_ptrs || !ntt_has_modup(c))) return hipErrorInvalidValue;
    if (lin_k && (!mul_ptrs || pl.n != 1)) return hipErrorInvalidValue;
    if (epilogue && epilogue->use_vl == 2 && !c->ntt_f64) return hipErrorInvalidValue;
    if (hi_only && (!conv || epilogue)) return hipErrorInvalidValue;
    if (src_ptrs && batch > KS_MAX_BATCH) return hipErrorInvalidValue;
    if (epilogue && (inverse || !ntt_has_epilogue(c) || batch > 2 * KS_MAX_BATCH)) return hipErrorInvalidValue;
    if ((inv_scale && !inverse) || (conv && inverse) || ((inv_scale || conv) && !ntt_has_modup(c))) return hipErrorInvalidValue;
    if (conv && (conv->nd == 0 || conv->nd > conv->ap || (conv->ap != 4 && conv->ap != 8 && conv->ap != 12 && conv->ap != 16)))
        return hipErrorInvalidValue;
    const bool f64 = c->ntt_f64;
    NttArgs args;
    args.src = src;
    args.dst = dst;
    args.src_bstride = src_bstride;
    args.dst_bstride = dst_bstride;
    args.mc = f64 ? (const void*)c->d_mcf : (const void*)c->d_mc;
    args.tw = f64 ? (const void*)(inverse ? c->d_itwf : c->d_twf) : (const void*)(inverse ? c->d_itw : c->d_tw);
    args.tw_val = f64 ? (inverse ? c->d_itwf_val : c->d_twf_val) : nullptr;
    args.log_n = c->log_n;
    args.log_lo = c->log_lo;
    args.log_hi = c->log_hi;
    args.first = 1;
    args.last = 1;
    args.batch = batch;
    {
        const u32 slices = pl.n << c->log_hi;
        args.lo_group = 0;
        for (u32 g = 64; g >= 8; g >>= 1)
            if (slices % g == 0) { args.lo_group = g; break; }
    }
    args.use_src_list = src_ptrs ? 1 : 0;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) {
        args.src_list.p[b] = (src_ptrs && b < batch) ? src_ptrs[b] : nullptr;
        args.mul_list.p[b] = (mul_ptrs && b < batch) ? mul_ptrs[b] : nullptr;
    }
    args.inv_scale = inv_scale;
    args.use_lin = lin_k ? 1 : 0;
    args.lin_ka = lin_k ? lin_k[0] : 0;
    args.lin_kb = lin_k ? lin_k[1] : 0;
    args.pad2 = 0;
    const u32 polys = pl.n * batch;
    const dim3 block(NTT_THREADS);
    const double pass_bytes = 16.0 * polys * c->N;
    if (c->log_n < CKKS_TILE_LOG) {
        ProfScope ps__(c, inverse ? K_NTT_INV_LO : K_NTT_FWD_LO, st, pass_bytes, 0.5 * polys * c->N * c->log_n);
        if (inverse) hipLaunchKernelGGL(ntt_small_kernel<true>, dim3(1, polys), block, 0, st, args, pl);
        else hipLaunchKernelGGL(ntt_small_kernel<false>, dim3(1, polys), block, 0, st, args, pl);
        return hipGetLastError();
    }
    const dim3 grid(c->N >> CKKS_TILE_LOG, polys);  // hi pass: one workgroup per 2^11 points
    const u32 slices = pl.n << c->log_hi;
    // batch items per lo-pass workgroup: in the inverse pass two share one fetch of the twiddles (an unrolled four cost too many
    // registers, and a loop over the items as in the plain forward pass spills in the variant that forms a product as it
    // loads, 4.7 -> 6.3 ms per step of the block slice; that variant takes one item: with two it holds two operands' points a
    // tile ahead and spills at three waves per SIMD, 4.7 against 4.2 ms per step for the class); the pass that ends a division takes one (with its epilogue's operands
    // two items leave only two waves per SIMD, which costs more than the second fetch of the twiddles); the plain forward
    // pass sets its own extent (launch_fwd_lo_loop)
    const u32 lo_items = (batch >= 2 && !epilogue) ? 2 : 1;
    const u32 lo_wgs = (batch + lo_items - 1) / lo_items;
    const dim3 grid_lo = args.lo_group ? dim3(args.lo_group, lo_wgs, slices / args.lo_group) : dim3(lo_wgs, slices);  // see lo_tile()
    const double lo_ops = 0.5 * polys * c->N * c->log_lo, hi_ops = 0.5 * polys * c->N * c->log_hi;
    // the second pass of either direction continues in place on dst
    NttArgs second = args;
    second.src = dst;
    second.src_bstride = dst_bstride;
    second.use_src_list = 0;
    second.first = 0;
    PolyList pd = pl;
    for (u32 i = 0; i < pl.n; i++) pd.spos[i] = pl.dpos[i];
    auto hi = [&](const NttArgs& a, const PolyList& l) { if (f64) launch_hi_any<ArithF64>(c->log_hi, inverse, grid, st, a, l); else launch_hi_any<ArithU64>(c->log_hi, inverse, grid, st, a, l); };
    auto lo = [&](const NttArgs& a, const PolyList& l) {
        if (!inverse) {
            if (f64) launch_fwd_lo_loop<ArithF64>(batch, grid_lo, st, a, l);
            else launch_fwd_lo_loop<ArithU64>(batch, grid_lo, st, a, l);
        } else {
            if (f64) launch_inv_lo<ArithF64>(lo_items, grid_lo, st, a, l);
            else launch_inv_lo<ArithU64>(lo_items, grid_lo, st, a, l);
        }
    };
    if (!inverse) {
        if (c->log_hi > 0) {
            args.last = 0;
            if (conv) {  // reads the digit's nd limbs for every target limb (from cache after the first), writes the target limbs
                ProfScope ps__(c, K_NTT_FWD_HI, st, 8.0 * c->N * batch * ((double)conv->nd + pl.n), hi_ops);
                const u32 ct = conv_targets(c->log_hi, pl.n, conv->nd);
                launch_hi_conv(c->log_hi, conv->ap, dim3(grid.x, (pl.n + ct - 1) / ct * batch), st, args, pl, *conv);
            } else {
                ProfScope ps__(c, K_NTT_FWD_HI, st, pass_bytes, hi_ops);
                hi(args, pl);
            }
            if (hi_only) return hipGetLastError();  // the caller's own lo pass follows (launch_ntt_lo_mac)
            if (epilogue) {  // reads w and v, writes the quotients (plus the addends it reads)
                ProfScope ps__(c, K_NTT_FWD_LO, st, (epilogue->use_vl == 2 ? 2.0 : 1.5) * pass_bytes, lo_ops);
                if (f64) launch_lo_div<ArithF64>(grid_lo, st, second, pd, *epilogue);
                else launch_lo_div<ArithU64>(grid_lo, st, second, pd, *epilogue);
            } else {
                ProfScope ps__(c, K_NTT_FWD_LO, st, pass_bytes, lo_ops);
                lo(second, pd);
            }
        } else {
            ProfScope ps__(c, K_NTT_FWD_LO, st, pass_bytes, lo_ops);
            lo(args, pl);
        }
    } else {
        args.last = c->log_hi == 0;
        {
            ProfScope ps__(c, K_NTT_INV_LO, st, mul_ptrs ? 1.5 * pass_bytes : pass_bytes, lo_ops);
            if (mul_ptrs) {  // one item per workgroup (see lo_items)
                dim3 g1 = grid_lo;
                if (args.lo_group) g1.y = batch;
                else g1.x = batch;
                launch_inv_lo<ArithF64>(1, g1, st, args, pl, true);
            }
            else lo(args, pl);
        }
        if (c->log_hi > 0) { ProfScope ps__(c, K_NTT_INV_HI, st, pass_bytes, hi_ops); hi(second, pd); }
    }
    return hipGetLastError();
}

hipError_t launch_ntt(const ckks_ctx* c, bool inverse, const u64* src, size_t src_bstride, u64* dst, size_t dst_bstride,
                      const PolyList& pl, u32 batch, hipStream_t st, const u64* const* src_ptrs, const FwdEpilogue* epilogue,
                      const TwF* inv_scale, const u64* const* mul_ptrs, const u64* lin_k) {
    return launch_ntt_any(c, inverse, src, src_bstride, dst, dst_bstride, pl, batch, st, src_ptrs, epilogue, inv_scale, nullptr, false,
                          mul_ptrs, lin_k);
}

hipError_t launch_ntt_modup(const ckks_ctx* c, u32 level, u32 j, const double* y, size_t y_bstride, u64* dst, size_t dst_bstride,
                            const PolyList& pl, u32 batch, hipStream_t st, bool hi_only) {
    ConvPrologue cp;
    cp.y = y;
    cp.y_bstride = y_bstride;
    cp.convf = c->modup_table_f(level, j);
    cp.lo = c->digit_lo(j);
    cp.nd = c->digit_hi(j, level) - cp.lo;
    cp.ap = c->alpha_pad;
    cp.pad = 0;
    return launch_ntt_any(c, false, dst, dst_bstride, dst, dst_bstride, pl, batch, st, nullptr, nullptr, nullptr, &cp, hi_only);
}

hipError_t launch_ntt_rescale(const ckks_ctx* c, u32 level, const double* y, u64* dst, u32 batch, hipStream_t st,
                              const FwdEpilogue* epilogue) {
    if (level == 0 || !c->d_rescale_conv_f) return hipErrorInvalidValue;
    ConvPrologue cp;
    cp.y = y;
    cp.y_bstride = c->N;  // one limb per batch item
    cp.convf = c->d_rescale_conv_f;
    cp.lo = 0;
    cp.nd = 1;
    cp.ap = 4;
    cp.pad = 0;
    PolyList pl;
    for (u32 a = 0; a < CKKS_MAX_MODULI; a++) pl.spos[a] = pl.dpos[a] = pl.mod[a] = (unsigned char)(a < level ? a : 0);
    pl.n = level;
    return launch_ntt_any(c, false, dst, level, dst, level, pl, batch, st, nullptr, epilogue, nullptr, &cp);
}

hipError_t launch_ntt_lo_mac(const ckks_ctx* c, u32 level, const DigitSrc& digits, const u64* const* keys, u64* const* outs, u32 n,
                             hipStream_t st, const MacProduct* prod) {
    if (!ntt_has_modup(c) || c->log_hi == 0 || n == 0 || n > KS_MAX_BATCH) return hipErrorInvalidValue;
    const u32 E = c->ext_limbs(level), beta = c->live_digits(level);
    NttArgs args = {};
    args.mc = c->d_mcf;
    args.tw = c->d_twf;
    args.tw_val = c->d_twf_val;
    args.log_n = c->log_n;
    args.log_lo = c->log_lo;
    args.log_hi = c->log_hi;
    args.batch = n;
    const u32 slices = E << c->log_hi;
    args.lo_group = 0;
    for (u32 g = 64; g >= 8; g >>= 1)
        if (slices % g == 0) { args.lo_group = g; break; }
    PolyList pl;
    pl.n = E;
    for (u32 e = 0; e < CKKS_MAX_MODULI; e++) pl.spos[e] = pl.dpos[e] = pl.mod[e] = (unsigned char)(e < E ? c->ext_modulus(level, e) : 0);
    MacEpilogue ep;
    ep.D = digits;
    double n_add = 0.0, n_keys = 0.0;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) {
        ep.key.p[b] = b < n ? keys[b] : nullptr;
        ep.out.p[b] = b < n ? outs[b] : nullptr;
        if (b < n && !ep.key.p[b]) return hipErrorInvalidValue;
        ep.a0.p[b] = (prod && b < n) ? prod->a0[b] : nullptr;
        ep.a1.p[b] = (prod && b < n) ? prod->a1[b] : nullptr;
        ep.b0.p[b] = (prod && b < n) ? prod->b0[b] : nullptr;
        ep.b1.p[b] = (prod && b < n) ? prod->b1[b] : nullptr;
        if (prod && b < n && (!ep.a0.p[b] || !ep.a1.p[b] || !ep.b0.p[b] || !ep.b1.p[b])) return hipErrorInvalidValue;
        if (b < n && (b == 0 || keys[b] != keys[b - 1])) n_keys += 1.0;
    }
    ep.negp = c->d_moddown + 2 * c->k_pad + (size_t)c->k_pad * c->num_q + 2 * c->num_q;
    ep.level = level;
    ep.M = c->M;
    ep.E = E;
    ep.beta = beta;
    ep.prod = prod ? 1 : 0;
    ep.lin = (prod && prod->lin_x) ? 1 : 0;
    if (ep.lin && (!prod->lin_y || !prod->ka || !prod->kb)) return hipErrorInvalidValue;
    ep.x_cstride = ep.lin ? prod->x_cstride : 0;
    ep.y_cstride = ep.lin ? prod->y_cstride : 0;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) {
        ep.lx.p[b] = (ep.lin && b < n) ? prod->lin_x[b] : nullptr;
        ep.ly.p[b] = (ep.lin && b < n) ? prod->lin_y[b] : nullptr;
        if (ep.lin && b < n && (!ep.lx.p[b] || !ep.ly.p[b])) return hipErrorInvalidValue;
    }
    for (u32 i = 0; i < CKKS_MAX_MODULI; i++) {
        ep.ka[i] = (ep.lin && i <= level) ? prod->ka[i] : 0;
        ep.kb[i] = (ep.lin && i <= level) ? prod->kb[i] : 0;
    }
    // digits transformed per batch item: every (digit, position) pair but the digits' own limbs
    const double n_tr = (double)beta * E - (level + 1.0);
    // the grid's extent over the batch: two, i.e. four items per workgroup in a batch of eight (measured: 16.5 ms per step for
    // the lo-pass class with one item per workgroup, 16.35 with all eight, 16.15 with four, which still leave the chip's 256
    // CUs, two workgroups each, four rounds of workgroups)
    const u32 b_ext = n < 2 ? n : 2;
    const dim3 grid = args.lo_group ? dim3(args.lo_group, b_ext, slices / args.lo_group) : dim3(b_ext, slices);
    // in: the transformed rows, the own limbs, the addends, the keys (once per distinct key); out: two components
    if (ep.lin) n_add = 4.0 * n;  // two components of two ciphertexts
    ProfScope ps__(c, K_NTT_FWD_LO, st, 8.0 * c->N * (n * (n_tr + (prod ? 4.0 : 1.0) * (level + 1.0) + 2.0 * E) + n_add * (level + 1.0) + n_keys * 2.0 * beta * E),
                   0.5 * n * n_tr * c->N * c->log_lo);
    // which operands join after the digits is the same for the whole launch: one instantiation per case
#define LO_MAC_LAUNCH(PROD, LIN) hipLaunchKernelGGL((ntt_fwd_lo_mac_kernel<PROD, LIN>), grid, dim3(NTT_THREADS), 0, st, args, pl, ep)
    if (ep.lin) LO_MAC_LAUNCH(true, true);
    else if (ep.prod) LO_MAC_LAUNCH(true, false);
    else LO_MAC_LAUNCH(false, false);
#undef LO_MAC_LAUNCH
    return hipGetLastError();
}

hipError_t launch_ntt_moddown(const ckks_ctx* c, u32 level, bool merged, const double* y, u64* dst, u32 batch, hipStream_t st,
                              const FwdEpilogue* epilogue) {
    if (merged && level == 0) return hipErrorInvalidValue;
    const u32 n_out = merged ? level : level + 1;
    ConvPrologue cp;
    cp.y = y;
    cp.y_bstride = (size_t)c->ext_limbs(level) * c->N;
    cp.convf = merged ? c->moddown_rs_table_f(level) : c->d_moddown_f;
    cp.lo = merged ? level : level + 1;  // the dropped limbs sit at consecutive positions of the extended polynomial
    cp.nd = merged ? c->num_p + 1 : c->num_p;
    cp.ap = merged ? c->k2_pad : c->k_pad;
    cp.pad = 0;
    PolyList pl;
    for (u32 a = 0; a < CKKS_MAX_MODULI; a++) pl.spos[a] = pl.dpos[a] = pl.mod[a] = (unsigned char)(a < n_out ? a : 0);
    pl.n = n_out;
    return launch_ntt_any(c, false, dst, n_out, dst, n_out, pl, batch, st, nullptr, epilogue, nullptr, &cp);
}
