// Negacyclic NTT / inverse NTT over Z_q[X]/(X^N+1) for gfx950 (Background, "RNS Decomposition and
// NTT Optimization": the transform that makes ring multiplication quasi-linear).
//
// Forward: natural-order coefficients in, out[k] = a(psi^(2*bitrev(k)+1)).  The log2(N) radix-2
// stages are split into two passes so that each workgroup transforms a 2^11-point tile held in LDS:
//   hi pass : the first log_hi stages pair elements 2^log_lo or more apart; a tile is all 2^log_hi
//             rows of a group of adjacent columns (rows are 2^log_lo elements apart in memory, so
//             every row segment is a contiguous, coalesced run);
//   lo pass : the remaining log_lo stages act inside contiguous blocks of 2^log_lo elements.
// The bit-reversed output order falls out of this split with no transpose.  The inverse runs the
// lo pass first, then the hi pass, and folds the 1/N into its last store.
// Butterflies are Harvey's lazy ones on Shoup-precomputed twiddles: forward values stay in
// [0, 4q), inverse values in [0, 2q); the last pass stores canonical residues.
#include "ctx.h"

#define NTT_THREADS 256

__device__ __forceinline__ void fwd_butterfly(u64& x, u64& y, u64 w, u64 w_sh, u64 q) {
    u64 two_q = 2 * q;
    if (x >= two_q) x -= two_q;
    u64 t = mul_shoup_lazy(y, w, w_sh, q);
    y = x + two_q - t;
    x = x + t;
}

__device__ __forceinline__ void inv_butterfly(u64& x, u64& y, u64 w, u64 w_sh, u64 q) {
    u64 two_q = 2 * q;
    u64 s = x + y;
    if (s >= two_q) s -= two_q;
    u64 d = x + two_q - y;
    x = s;
    y = mul_shoup_lazy(d, w, w_sh, q);
}

__device__ __forceinline__ u64 canon4(u64 v, u64 q) {  // [0,4q) -> [0,q)
    if (v >= 2 * q) v -= 2 * q;
    if (v >= q) v -= q;
    return v;
}

struct NttArgs {
    const u64* src;
    u64* dst;
    size_t src_bstride;  // in limb-polys
    size_t dst_bstride;
    const ModConst* mc;
    const u64* tw;       // [M][N]
    const u64* tw_sh;
    u32 log_n, log_lo, log_hi;
    u32 last;            // this pass writes the final result (canonical; inverse: times 1/N)
};

// ---- forward, strided pass (stages 0 .. log_hi-1) ----------------------------------------------
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_hi_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 lds[1 << CKKS_TILE_LOG];
    const u32 tid = threadIdx.x;
    const u32 p = blockIdx.y, b = p / pl.n, a = p % pl.n;
    const u32 N = 1u << A.log_n, tile = 1u << CKKS_TILE_LOG;
    const u32 log_cc = CKKS_TILE_LOG - A.log_hi, cc = 1u << log_cc;  // columns per tile
    const u32 col0 = blockIdx.x << log_cc;
    const u32 m_idx = pl.mod[a];
    const u64 q = A.mc[m_idx].q;
    const u64* src = A.src + (b * A.src_bstride + pl.spos[a]) * (size_t)N;
    u64* dst = A.dst + (b * A.dst_bstride + pl.dpos[a]) * (size_t)N;
    const u64* tw = A.tw + (size_t)m_idx * N;
    const u64* tw_sh = A.tw_sh + (size_t)m_idx * N;

    for (u32 e = tid; e < tile; e += NTT_THREADS) {
        u32 row = e >> log_cc, c = e & (cc - 1);
        lds[e] = src[((size_t)row << A.log_lo) + col0 + c];
    }
    __syncthreads();
    for (u32 s = 0; s < A.log_hi; s++) {
        const u32 lt = A.log_hi - 1 - s;  // log2 of the row distance of a pair
        for (u32 bf = tid; bf < tile / 2; bf += NTT_THREADS) {
            u32 rp = bf >> log_cc, c = bf & (cc - 1);
            u32 i = rp >> lt;
            u32 row = (i << (lt + 1)) + (rp & ((1u << lt) - 1));
            u32 i0 = (row << log_cc) + c, i1 = i0 + (1u << (lt + log_cc));
            u64 x = lds[i0], y = lds[i1];
            fwd_butterfly(x, y, tw[(1u << s) + i], tw_sh[(1u << s) + i], q);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    for (u32 e = tid; e < tile; e += NTT_THREADS) {
        u32 row = e >> log_cc, c = e & (cc - 1);
        dst[((size_t)row << A.log_lo) + col0 + c] = lds[e];  // lazy [0,4q): the lo pass follows
    }
}

// ---- forward, contiguous pass (stages log_hi .. log_n-1) ---------------------------------------
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_lo_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 lds[1 << CKKS_TILE_LOG];
    const u32 tid = threadIdx.x;
    const u32 p = blockIdx.y, b = p / pl.n, a = p % pl.n;
    const u32 N = 1u << A.log_n, tile = 1u << A.log_lo;
    const u32 blk = blockIdx.x;
    const u32 m_idx = pl.mod[a];
    const u64 q = A.mc[m_idx].q;
    const u64* src = A.src + (b * A.src_bstride + pl.spos[a]) * (size_t)N + ((size_t)blk << A.log_lo);
    u64* dst = A.dst + (b * A.dst_bstride + pl.dpos[a]) * (size_t)N + ((size_t)blk << A.log_lo);
    const u64* tw = A.tw + (size_t)m_idx * N;
    const u64* tw_sh = A.tw_sh + (size_t)m_idx * N;

    for (u32 e = tid; e < tile; e += NTT_THREADS) lds[e] = src[e];
    __syncthreads();
    for (u32 r = 0; r < A.log_lo; r++) {
        const u32 lt = A.log_lo - 1 - r;
        const u32 tw_base = (1u << (A.log_hi + r)) + (blk << r);
        for (u32 bf = tid; bf < tile / 2; bf += NTT_THREADS) {
            u32 i = bf >> lt;
            u32 i0 = (i << (lt + 1)) + (bf & ((1u << lt) - 1)), i1 = i0 + (1u << lt);
            u64 x = lds[i0], y = lds[i1];
            fwd_butterfly(x, y, tw[tw_base + i], tw_sh[tw_base + i], q);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    for (u32 e = tid; e < tile; e += NTT_THREADS) dst[e] = canon4(lds[e], q);
}

// ---- inverse, contiguous pass (pair distances 1 .. 2^(log_lo-1)) -------------------------------
__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_lo_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 lds[1 << CKKS_TILE_LOG];
    const u32 tid = threadIdx.x;
    const u32 p = blockIdx.y, b = p / pl.n, a = p % pl.n;
    const u32 N = 1u << A.log_n, tile = 1u << A.log_lo;
    const u32 blk = blockIdx.x;
    const u32 m_idx = pl.mod[a];
    const ModConst mc = A.mc[m_idx];
    const u64 q = mc.q;
    const u64* src = A.src + (b * A.src_bstride + pl.spos[a]) * (size_t)N + ((size_t)blk << A.log_lo);
    u64* dst = A.dst + (b * A.dst_bstride + pl.dpos[a]) * (size_t)N + ((size_t)blk << A.log_lo);
    const u64* tw = A.tw + (size_t)m_idx * N;
    const u64* tw_sh = A.tw_sh + (size_t)m_idx * N;

    for (u32 e = tid; e < tile; e += NTT_THREADS) lds[e] = src[e];
    __syncthreads();
    for (u32 lt = 0; lt < A.log_lo; lt++) {
        const u32 r = A.log_lo - 1 - lt;
        const u32 tw_base = (1u << (A.log_hi + r)) + (blk << r);
        for (u32 bf = tid; bf < tile / 2; bf += NTT_THREADS) {
            u32 i = bf >> lt;
            u32 i0 = (i << (lt + 1)) + (bf & ((1u << lt) - 1)), i1 = i0 + (1u << lt);
            u64 x = lds[i0], y = lds[i1];
            inv_butterfly(x, y, tw[tw_base + i], tw_sh[tw_base + i], q);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    if (A.last) {
        for (u32 e = tid; e < tile; e += NTT_THREADS) dst[e] = mul_shoup(lds[e], mc.n_inv, mc.n_inv_sh, q);
    } else {
        for (u32 e = tid; e < tile; e += NTT_THREADS) dst[e] = lds[e];  // lazy [0,2q)
    }
}

// ---- inverse, strided pass (row distances 1 .. 2^(log_hi-1)), scales by 1/N --------------------
__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_hi_kernel(NttArgs A, PolyList pl) {
    __shared__ u64 lds[1 << CKKS_TILE_LOG];
    const u32 tid = threadIdx.x;
    const u32 p = blockIdx.y, b = p / pl.n, a = p % pl.n;
    const u32 N = 1u << A.log_n, tile = 1u << CKKS_TILE_LOG;
    const u32 log_cc = CKKS_TILE_LOG - A.log_hi, cc = 1u << log_cc;
    const u32 col0 = blockIdx.x << log_cc;
    const u32 m_idx = pl.mod[a];
    const ModConst mc = A.mc[m_idx];
    const u64 q = mc.q;
    // the lo pass has already moved the data to dst
    u64* dst = A.dst + (b * A.dst_bstride + pl.dpos[a]) * (size_t)N;
    const u64* tw = A.tw + (size_t)m_idx * N;
    const u64* tw_sh = A.tw_sh + (size_t)m_idx * N;

    for (u32 e = tid; e < tile; e += NTT_THREADS) {
        u32 row = e >> log_cc, c = e & (cc - 1);
        lds[e] = dst[((size_t)row << A.log_lo) + col0 + c];
    }
    __syncthreads();
    for (u32 lt = 0; lt < A.log_hi; lt++) {
        const u32 s = A.log_hi - 1 - lt;
        for (u32 bf = tid; bf < tile / 2; bf += NTT_THREADS) {
            u32 rp = bf >> log_cc, c = bf & (cc - 1);
            u32 i = rp >> lt;
            u32 row = (i << (lt + 1)) + (rp & ((1u << lt) - 1));
            u32 i0 = (row << log_cc) + c, i1 = i0 + (1u << (lt + log_cc));
            u64 x = lds[i0], y = lds[i1];
            inv_butterfly(x, y, tw[(1u << s) + i], tw_sh[(1u << s) + i], q);
            lds[i0] = x;
            lds[i1] = y;
        }
        __syncthreads();
    }
    for (u32 e = tid; e < tile; e += NTT_THREADS) {
        u32 row = e >> log_cc, c = e & (cc - 1);
        dst[((size_t)row << A.log_lo) + col0 + c] = mul_shoup(lds[e], mc.n_inv, mc.n_inv_sh, q);
    }
}

hipError_t launch_ntt(const ckks_ctx* c, bool inverse, const u64* src, size_t src_bstride, u64* dst,
                      size_t dst_bstride, const PolyList& pl, u32 batch, hipStream_t st) {
    if (pl.n == 0 || batch == 0) return hipSuccess;
    NttArgs A;
    A.src = src;
    A.dst = dst;
    A.src_bstride = src_bstride;
    A.dst_bstride = dst_bstride;
    A.mc = c->d_mc;
    A.log_n = c->log_n;
    A.log_lo = c->log_lo;
    A.log_hi = c->log_hi;
    const u32 polys = pl.n * batch;
    const dim3 block(NTT_THREADS);
    const dim3 grid_lo(1u << c->log_hi, polys);
    const dim3 grid_hi(c->N >> CKKS_TILE_LOG, polys);
    if (!inverse) {
        A.tw = c->d_tw;
        A.tw_sh = c->d_tw_sh;
        A.last = 1;
        if (c->log_hi > 0) {
            { ProfScope ps__(c, K_NTT_FWD_HI, st, 16.0 * polys * c->N, 0.5 * polys * c->N * c->log_hi); hipLaunchKernelGGL(ntt_fwd_hi_kernel, grid_hi, block, 0, st, A, pl); }
            // the lo pass continues in place on dst
            NttArgs B = A;
            B.src = dst;
            B.src_bstride = dst_bstride;
            PolyList pd = pl;
            for (u32 i = 0; i < pl.n; i++) pd.spos[i] = pl.dpos[i];
            { ProfScope ps__(c, K_NTT_FWD_LO, st, 16.0 * polys * c->N, 0.5 * polys * c->N * c->log_lo); hipLaunchKernelGGL(ntt_fwd_lo_kernel, grid_lo, block, 0, st, B, pd); }
        } else {
            { ProfScope ps__(c, K_NTT_FWD_LO, st, 16.0 * polys * c->N, 0.5 * polys * c->N * c->log_lo); hipLaunchKernelGGL(ntt_fwd_lo_kernel, grid_lo, block, 0, st, A, pl); }
        }
    } else {
        A.tw = c->d_itw;
        A.tw_sh = c->d_itw_sh;
        A.last = c->log_hi == 0;
        { ProfScope ps__(c, K_NTT_INV_LO, st, 16.0 * polys * c->N, 0.5 * polys * c->N * c->log_lo); hipLaunchKernelGGL(ntt_inv_lo_kernel, grid_lo, block, 0, st, A, pl); }
        if (c->log_hi > 0) { ProfScope ps__(c, K_NTT_INV_HI, st, 16.0 * polys * c->N, 0.5 * polys * c->N * c->log_hi); hipLaunchKernelGGL(ntt_inv_hi_kernel, grid_hi, block, 0, st, A, pl); }
    }
    return hipGetLastError();
}
