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
// Twiddles psi^bitrev(i) sit in one table per modulus, each with its Shoup companion in the same
// 16-byte word; the index of the twiddle of a butterfly group obeys T(next stage) = 2*T + bit, so a
// thread needs only the index of its group at the first stage of a round.
// Butterflies are lazy: forward values are never corrected on the way (they stay below 35q < 2^64),
// inverse values are kept in [0, 2q); the last pass stores canonical residues.  Rings below 2^11 use a plain one-tile kernel.
#include "ctx.h"

#define NTT_THREADS 256
#define NTT_TILE 2048
#define LDS_PAD(p) ((p) + ((p) >> 3))        // keeps all three exchange patterns (almost) conflict-free
#define LDS_PADDED_WORDS (NTT_TILE + NTT_TILE / 8)

// Forward butterfly with no correction at all: the Shoup product t is in [0, 2q) for ANY 64-bit y, so
// both outputs stay non-negative and grow by at most 2q per stage: below (1 + 2*17) q < 2^64 for every
// supported modulus (q < 2^58) over a whole transform.  One word reduction at the very end.
__device__ __forceinline__ void fwd_bf(u64& x, u64& y, const TwPair w, u64 q) {
    const u64 t = mul_shoup_lazy(y, w.w, w.s, q);
    y = x + 2 * q - t;
    x = x + t;
}

__device__ __forceinline__ void inv_bf(u64& x, u64& y, const TwPair w, u64 q) {
    const u64 two_q = 2 * q;
    u64 s = x + y;
    if (s >= two_q) s -= two_q;
    const u64 d = x + two_q - y;
    x = s;
    y = mul_shoup_lazy(d, w.w, w.s, q);
}


// S radix-2 stages on 2^S "rows" of KC independent columns held in registers, v[row*KC + col];
// row bit S-1 is the largest distance.  T = twiddle index of this group at the first stage.
template <int S, int KC>
__device__ __forceinline__ void fwd_rows(u64* v, const TwPair* __restrict__ tw, u32 T, u64 q) {
#pragma unroll
    for (int a = 0; a < S; a++) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            const TwPair w = tw[(T << a) + (rr >> (S - a))];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) fwd_bf(v[rr * KC + kc], v[(rr + half) * KC + kc], w, q);
        }
    }
}

template <int S, int KC>
__device__ __forceinline__ void inv_rows(u64* v, const TwPair* __restrict__ tw, u32 T, u64 q) {
#pragma unroll
    for (int a = S - 1; a >= 0; a--) {
        const int half = (1 << S) >> (a + 1);
#pragma unroll
        for (int rr = 0; rr < (1 << S); rr++) {
            if (rr & half) continue;
            const TwPair w = tw[(T << a) + (rr >> (S - a))];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) inv_bf(v[rr * KC + kc], v[(rr + half) * KC + kc], w, q);
        }
    }
}

struct NttArgs {
    const u64* src;
    u64* dst;
    size_t src_bstride;  // in limb-polys
    size_t dst_bstride;
    const ModConst* mc;
    const TwPair* tw;    // [M][N]
    u32 log_n, log_lo, log_hi;
    u32 last;            // this pass writes the final result (canonical; inverse: times 1/N)
    u32 batch;           // batch items (each pl.n limb-polys)
    u32 lo_group;        // slices per group of the lo-pass numbering (0: plain)
    u32 use_src_list;    // batch item b reads src_list.p[b] instead of src + b*src_bstride*N
    PtrList8 src_list;
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

struct PolyRef {
    const u64* src;
    u64* dst;
    const TwPair* tw;
    ModConst mc;
};

__device__ __forceinline__ PolyRef poly_ref(const NttArgs& A, const PolyList& pl, u32 b, u32 a) {
    const u32 m_idx = pl.mod[a];
    PolyRef r;
    r.src = (A.use_src_list ? A.src_list.p[b] : A.src + (((size_t)b * A.src_bstride) << A.log_n)) + ((size_t)pl.spos[a] << A.log_n);
    r.dst = A.dst + (((size_t)b * A.dst_bstride + pl.dpos[a]) << A.log_n);
    r.tw = A.tw + ((size_t)m_idx << A.log_n);
    r.mc = A.mc[m_idx];
    return r;
}

// ================================ lo pass (contiguous 2^11 blocks) ================================
// positions inside the block: pos = d3*256 + d2*32 + d1*4 + d0 (d3,d2,d1 < 8, d0 < 4)
//   round A: thread = pos % 256,           points over d3          (distances 1024, 512, 256)
//   round B: thread = (d3, pos % 32),      points over d2          (distances 128, 64, 32)
//   round C: thread = (d3, d2, d0),        points over d1          (distances 16, 8, 4)
//   round D: thread = pos / 8,             8 consecutive points    (distances 2, 1)
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_lo_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 buf0[LDS_PADDED_WORDS];
    __shared__ u64 buf1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(A.log_hi, A.lo_group);
    const u32 blk = tile.blk;
    const PolyRef P = poly_ref(A, pl, tile.b, tile.a);
    const u64 q = P.mc.q;
    const u64* src = P.src + ((size_t)blk << 11);
    u64* dst = P.dst + ((size_t)blk << 11);
    const u32 TA = (1u << A.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    u64 v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = src[tid + 256 * j];
    fwd_rows<3, 1>(v, P.tw, TA, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf0[LDS_PAD(tid + 256 * j)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(d3 * 256 + 32 * j + x5)];
    fwd_rows<3, 1>(v, P.tw, 8 * TA + d3, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf1[LDS_PAD(d3 * 256 + 32 * j + x5)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)];
    fwd_rows<3, 1>(v, P.tw, 64 * TA + 8 * d3 + d2, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(8 * tid + j)];
    fwd_rows<2, 1>(v, P.tw, 512 * TA + 2 * tid, q);
    fwd_rows<2, 1>(v + 4, P.tw, 512 * TA + 2 * tid + 1, q);
    ulonglong2* out = reinterpret_cast<ulonglong2*>(dst + 8 * tid);
#pragma unroll
    for (int j = 0; j < 4; j++) out[j] = make_ulonglong2(reduce_word(v[2 * j], P.mc), reduce_word(v[2 * j + 1], P.mc));
}

__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_lo_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 buf0[LDS_PADDED_WORDS];
    __shared__ u64 buf1[LDS_PADDED_WORDS];
    const u32 tid = threadIdx.x;
    const LoTile tile = lo_tile(A.log_hi, A.lo_group);
    const u32 blk = tile.blk;
    const PolyRef P = poly_ref(A, pl, tile.b, tile.a);
    const u64 q = P.mc.q;
    const u64* src = P.src + ((size_t)blk << 11);
    u64* dst = P.dst + ((size_t)blk << 11);
    const u32 TA = (1u << A.log_hi) + blk;
    const u32 d3 = tid >> 5, x5 = tid & 31, d2 = (tid >> 2) & 7, d0 = tid & 3;
    u64 v[8];
    const ulonglong2* in = reinterpret_cast<const ulonglong2*>(src + 8 * tid);
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const ulonglong2 t = in[j];
        v[2 * j] = t.x;
        v[2 * j + 1] = t.y;
    }
    inv_rows<2, 1>(v, P.tw, 512 * TA + 2 * tid, q);
    inv_rows<2, 1>(v + 4, P.tw, 512 * TA + 2 * tid + 1, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf0[LDS_PAD(8 * tid + j)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)];
    inv_rows<3, 1>(v, P.tw, 64 * TA + 8 * d3 + d2, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf1[LDS_PAD(d3 * 256 + d2 * 32 + 4 * j + d0)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf1[LDS_PAD(d3 * 256 + 32 * j + x5)];
    inv_rows<3, 1>(v, P.tw, 8 * TA + d3, q);
#pragma unroll
    for (int j = 0; j < 8; j++) buf0[LDS_PAD(d3 * 256 + 32 * j + x5)] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = buf0[LDS_PAD(tid + 256 * j)];
    inv_rows<3, 1>(v, P.tw, TA, q);
    if (A.last) {
#pragma unroll
        for (int j = 0; j < 8; j++) dst[tid + 256 * j] = mul_shoup(v[j], P.mc.n_inv, P.mc.n_inv_sh, q);
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++) dst[tid + 256 * j] = v[j];  // lazy [0,2q): the hi pass follows
    }
}

// ============================ hi pass (rows 2^11 apart, adjacent columns) ============================
// tile = R = 2^LOG_HI rows x CC = 2048/R columns; element (row, col) lives at (row << 11) + col0 + col.
// LOG_HI <= 3: a thread holds all R rows of 8/R columns (no exchange).
// LOG_HI >= 4: round 1 = radix 8 over rows r0 + (R/8)*j of one column; exchange through LDS;
//              round 2 = the remaining LOG_HI-3 stages over R/8 consecutive rows of 64/R adjacent columns.
template <int LOG_HI>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_hi_kernel(NttArgs A, PolyList pl) {
    constexpr int R = 1 << LOG_HI, CC = NTT_TILE / R;
    const u32 tid = threadIdx.x;
    const PolyRef P = poly_ref(A, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    const u64 q = P.mc.q;
    const u64* src = P.src + (size_t)blockIdx.x * CC;
    u64* dst = P.dst + (size_t)blockIdx.x * CC;
    u64 v[8];
    if constexpr (LOG_HI <= 3) {
        constexpr int KC = 8 / R;
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) v[rr * KC + kc] = src[((size_t)rr << 11) + kc * 256 + tid];
        fwd_rows<LOG_HI, KC>(v, P.tw, 1, q);
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) dst[((size_t)rr << 11) + kc * 256 + tid] = v[rr * KC + kc];
    } else {
        __shared__ __attribute__((aligned(16))) u64 lds[NTT_TILE];
        constexpr int R8 = R / 8, S2 = LOG_HI - 3, KC2 = 8 / R8;
        const u32 r0 = tid / CC, col = tid % CC;
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = src[((size_t)(r0 + R8 * j) << 11) + col];
        fwd_rows<3, 1>(v, P.tw, 1, q);
#pragma unroll
        for (int j = 0; j < 8; j++) lds[(r0 + R8 * j) * CC + col] = v[j];
        __syncthreads();
        const u32 G = tid >> 5, cg = tid & 31;
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) v[rr * KC2 + kc] = lds[(G * R8 + rr) * CC + cg * KC2 + kc];
        fwd_rows<S2, KC2>(v, P.tw, 8 + G, q);
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) dst[((size_t)(G * R8 + rr) << 11) + cg * KC2 + kc] = v[rr * KC2 + kc];
    }
}

template <int LOG_HI>
__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_hi_kernel(NttArgs A, PolyList pl) {
    constexpr int R = 1 << LOG_HI, CC = NTT_TILE / R;
    const u32 tid = threadIdx.x;
    const PolyRef P = poly_ref(A, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    const u64 q = P.mc.q;
    u64* dst = P.dst + (size_t)blockIdx.x * CC;  // the lo pass has already moved the data to dst
    u64 v[8];
    if constexpr (LOG_HI <= 3) {
        constexpr int KC = 8 / R;
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++) v[rr * KC + kc] = dst[((size_t)rr << 11) + kc * 256 + tid];
        inv_rows<LOG_HI, KC>(v, P.tw, 1, q);
#pragma unroll
        for (int rr = 0; rr < R; rr++)
#pragma unroll
            for (int kc = 0; kc < KC; kc++)
                dst[((size_t)rr << 11) + kc * 256 + tid] = mul_shoup(v[rr * KC + kc], P.mc.n_inv, P.mc.n_inv_sh, q);
    } else {
        __shared__ __attribute__((aligned(16))) u64 lds[NTT_TILE];
        constexpr int R8 = R / 8, S2 = LOG_HI - 3, KC2 = 8 / R8;
        const u32 G = tid >> 5, cg = tid & 31;
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) v[rr * KC2 + kc] = dst[((size_t)(G * R8 + rr) << 11) + cg * KC2 + kc];
        inv_rows<S2, KC2>(v, P.tw, 8 + G, q);
#pragma unroll
        for (int rr = 0; rr < R8; rr++)
#pragma unroll
            for (int kc = 0; kc < KC2; kc++) lds[(G * R8 + rr) * CC + cg * KC2 + kc] = v[rr * KC2 + kc];
        __syncthreads();
        const u32 r0 = tid / CC, col = tid % CC;
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = lds[(r0 + R8 * j) * CC + col];
        inv_rows<3, 1>(v, P.tw, 1, q);
#pragma unroll
        for (int j = 0; j < 8; j++)
            dst[((size_t)(r0 + R8 * j) << 11) + col] = mul_shoup(v[j], P.mc.n_inv, P.mc.n_inv_sh, q);
    }
}

// ================================= rings below 2^11: one tile per poly =================================
template <bool INVERSE>
__global__ __launch_bounds__(NTT_THREADS) void ntt_small_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 lds[NTT_TILE];
    const u32 tid = threadIdx.x;
    const PolyRef P = poly_ref(A, pl, blockIdx.y / pl.n, blockIdx.y % pl.n);
    const u64 q = P.mc.q;
    const u32 n = 1u << A.log_n;
    for (u32 e = tid; e < n; e += NTT_THREADS) lds[e] = P.src[e];
    __syncthreads();
    for (u32 st = 0; st < A.log_n; st++) {
        const u32 r = INVERSE ? A.log_n - 1 - st : st;  // stage with 2^r groups
        const u32 lt = A.log_n - 1 - r;                 // log2 of the pair distance
        for (u32 bf = tid; bf < n / 2; bf += NTT_THREADS) {
            const u32 i = bf >> lt;
            const u32 i0 = (i << (lt + 1)) + (bf & ((1u << lt) - 1)), i1 = i0 + (1u << lt);
            u64 x = lds[i0], y = lds[i1];
            if (INVERSE) inv_bf(x, y, P.tw[(1u << r) + i], q); else fwd_bf(x, y, P.tw[(1u << r) + i], q);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    for (u32 e = tid; e < n; e += NTT_THREADS)
        P.dst[e] = INVERSE ? mul_shoup(lds[e], P.mc.n_inv, P.mc.n_inv_sh, q) : reduce_word(lds[e], P.mc);
}

template <int LOG_HI>
static void launch_hi(bool inverse, dim3 grid, hipStream_t st, const NttArgs& A, const PolyList& pl) {
    if (inverse) hipLaunchKernelGGL(ntt_inv_hi_kernel<LOG_HI>, grid, dim3(NTT_THREADS), 0, st, A, pl);
    else hipLaunchKernelGGL(ntt_fwd_hi_kernel<LOG_HI>, grid, dim3(NTT_THREADS), 0, st, A, pl);
}

static void launch_hi_any(u32 log_hi, bool inverse, dim3 grid, hipStream_t st, const NttArgs& A, const PolyList& pl) {
    switch (log_hi) {
        case 1: launch_hi<1>(inverse, grid, st, A, pl); break;
        case 2: launch_hi<2>(inverse, grid, st, A, pl); break;
        case 3: launch_hi<3>(inverse, grid, st, A, pl); break;
        case 4: launch_hi<4>(inverse, grid, st, A, pl); break;
        case 5: launch_hi<5>(inverse, grid, st, A, pl); break;
        default: launch_hi<6>(inverse, grid, st, A, pl); break;
    }
}

hipError_t launch_ntt(const ckks_ctx* c, bool inverse, const u64* src, size_t src_bstride, u64* dst,
                      size_t dst_bstride, const PolyList& pl, u32 batch, hipStream_t st, const u64* const* src_ptrs) {
    if (pl.n == 0 || batch == 0) return hipSuccess;
    if (src_ptrs && batch > KS_MAX_BATCH) return hipErrorInvalidValue;
    NttArgs A;
    A.src = src;
    A.dst = dst;
    A.src_bstride = src_bstride;
    A.dst_bstride = dst_bstride;
    A.mc = c->d_mc;
    A.tw = inverse ? c->d_itw : c->d_tw;
    A.log_n = c->log_n;
    A.log_lo = c->log_lo;
    A.log_hi = c->log_hi;
    A.last = 1;
    A.batch = batch;
    {
        const u32 slices = pl.n << c->log_hi;
        A.lo_group = 0;
        for (u32 g = 64; g >= 8; g >>= 1)
            if (slices % g == 0) { A.lo_group = g; break; }
    }
    A.use_src_list = src_ptrs ? 1 : 0;
    for (u32 b = 0; b < KS_MAX_BATCH; b++) A.src_list.p[b] = (src_ptrs && b < batch) ? src_ptrs[b] : nullptr;
    const u32 polys = pl.n * batch;
    const dim3 block(NTT_THREADS);
    const double pass_bytes = 16.0 * polys * c->N;
    if (c->log_n < CKKS_TILE_LOG) {
        ProfScope ps__(c, inverse ? K_NTT_INV_LO : K_NTT_FWD_LO, st, pass_bytes, 0.5 * polys * c->N * c->log_n);
        if (inverse) hipLaunchKernelGGL(ntt_small_kernel<true>, dim3(1, polys), block, 0, st, A, pl);
        else hipLaunchKernelGGL(ntt_small_kernel<false>, dim3(1, polys), block, 0, st, A, pl);
        return hipGetLastError();
    }
    const dim3 grid(c->N >> CKKS_TILE_LOG, polys);  // hi pass: one workgroup per 2^11 points
    const u32 slices = pl.n << c->log_hi;
    const dim3 grid_lo = A.lo_group ? dim3(A.lo_group, batch, slices / A.lo_group) : dim3(batch, slices);  // see lo_tile()
    const double lo_ops = 0.5 * polys * c->N * c->log_lo, hi_ops = 0.5 * polys * c->N * c->log_hi;
    // the second pass of either direction continues in place on dst
    NttArgs B = A;
    B.src = dst;
    B.src_bstride = dst_bstride;
    B.use_src_list = 0;
    PolyList pd = pl;
    for (u32 i = 0; i < pl.n; i++) pd.spos[i] = pl.dpos[i];
    if (!inverse) {
        if (c->log_hi > 0) {
            { ProfScope ps__(c, K_NTT_FWD_HI, st, pass_bytes, hi_ops); launch_hi_any(c->log_hi, false, grid, st, A, pl); }
            { ProfScope ps__(c, K_NTT_FWD_LO, st, pass_bytes, lo_ops); hipLaunchKernelGGL(ntt_fwd_lo_kernel, grid_lo, block, 0, st, B, pd); }
        } else {
            ProfScope ps__(c, K_NTT_FWD_LO, st, pass_bytes, lo_ops);
            hipLaunchKernelGGL(ntt_fwd_lo_kernel, grid_lo, block, 0, st, A, pl);
        }
    } else {
        A.last = c->log_hi == 0;
        { ProfScope ps__(c, K_NTT_INV_LO, st, pass_bytes, lo_ops); hipLaunchKernelGGL(ntt_inv_lo_kernel, grid_lo, block, 0, st, A, pl); }
        if (c->log_hi > 0) { ProfScope ps__(c, K_NTT_INV_HI, st, pass_bytes, hi_ops); launch_hi_any(c->log_hi, true, grid, st, B, pd); }
    }
    return hipGetLastError();
}
