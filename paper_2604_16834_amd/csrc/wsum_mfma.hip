// The multiply-accumulate over (input channel, tap) of the batched convolution (Methodology,
// "Convolution Evaluation", Eq. 11 and the rotation-free channel sum after it) on the matrix cores.
//
// With the integer weight factored out of the plaintext the layer's sum is, for every limb e, a dense
// modular matrix product
//     acc[o][x] = sum_k W_e[o][k] * X_e[k][x]  mod q_e,      o < C_out, k < 9*C_in, x < 2N,
// of a small weight matrix with the aligned, masked ciphertexts.  Residues below 2^50 are written in
// seven signed base-256 digits (v + bias with bias = 0x80 in each of the seven low bytes has the
// digits + 128 as its bytes, so two 64-bit operations give all seven); the 49 digit-by-digit products
// are exact 8-bit integer matrix products with 32-bit sums (v_mfma_i32_32x32x32_i8, the shape that
// runs at the full 8-bit rate: measured 4.3 POP/s against 2.5 for the 16x16x64 shape), summed by
// diagonal (digit positions adding up to s) in 13 accumulators; sum_s D_s 2^(8s) is the exact integer
// sum of products, reduced once in exact double-precision arithmetic.  Nothing is approximated: the result is the same
// canonical residue the scalar kernels give.
//
// One 256-thread workgroup = 64 columns x of one (component, limb) times 64 output channels.  Wave w
// owns output tile w&1 (32 channels) and column tile w>>1 (32 columns): every lane loads its own 32 X
// values of a 64-term block of k straight from HBM (32 lanes = one 256-byte run per term), splits them
// into digits and transposes bytes in registers (v_perm_b32) into the B operands.  The digit planes
// of the weights are prepared once per call in the A-operand lane layout and staged through LDS
// (double-buffered) so that the waves share them.  X streams from HBM exactly once.
//
// The weights are small integers (a real weight times the weight scale, rounded), not arbitrary residues: when the
// caller states a bound |w| < 2^(bits-1), the centred representative of each weight residue is written in DW = 3 (24
// bits) or 4 (32 bits) signed digits instead of 7, which leaves 7*DW digit products (21 or 28 instead of 49) and
// 7+DW-1 diagonals.  Same exact integer sum, same canonical residues.
#include "ctx.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define WM_THREADS 256
#define WM_DIGITS 7                                     // digits of an X value
#define WM_BIAS 0x0080808080808080ull
#define WM_TILES_PER_WG 16                              // 64-column tiles a workgroup streams one after the other
#define WM_OT_PER_WG 2                                  // output tiles of 32 channels per workgroup
#define WM_B_STAGE (WM_OT_PER_WG * WM_DIGITS * 2 * 64)  // uint4 words of one 64-term block of X digits (28 KiB)

// bytes 0..6 = the seven signed base-256 digits of v < 2^55 (two's complement bytes)
__host__ __device__ __forceinline__ u64 signed_digits(u64 v) { return (v + WM_BIAS) ^ WM_BIAS; }

// ---- weights: w_res [c_out][n_terms][nl] -> digit planes in A-operand layout ---------------------
// wa[(((e*KB + kb)*OT + ot)*7 + dw)*2 + ks][lane] = 16 bytes: digit dw of
//   W[32*ot + lane%32][64*kb + 32*ks + 16*(lane/32) + j], j < 16
// (zero beyond c_out / n_terms; OT = number of 32-channel tiles rounded up to a multiple of 2)
// DW < 7: the weights are centred first (v > q/2 -> v - q), DW digits hold them when |w| < 2^(8 DW - 1)
__global__ __launch_bounds__(WM_THREADS) void wsum_prep_kernel(const u64* __restrict__ w_res, uint4* __restrict__ wa,
                                                               const ModConst* __restrict__ mc, u32 level, u32 num_q, u32 c_out,
                                                               u32 n_terms, u32 nl, u32 KB, u32 OT, u32 DW) {
    const size_t idx = (size_t)blockIdx.x * WM_THREADS + threadIdx.x;
    if (idx >= (size_t)nl * KB * OT * DW * 2 * 64) return;
    const u32 lane = (u32)(idx & 63);
    size_t r = idx >> 6;
    const u32 ks = (u32)(r & 1);
    r >>= 1;
    const u32 dw = (u32)(r % DW);
    r /= DW;
    const u32 ot = (u32)(r % OT);
    r /= OT;
    const u32 kb = (u32)(r % KB), e = (u32)(r / KB);
    const u32 o = 32 * ot + (lane & 31), k0 = 64 * kb + 32 * ks + 16 * (lane >> 5);
    const u64 q = mc[e <= level ? e : num_q + (e - level - 1)].q;
    u32 words[4];
#pragma unroll
    for (u32 m = 0; m < 4; m++) {
        u32 wv = 0;
#pragma unroll
        for (u32 j = 0; j < 4; j++) {
            const u32 k = k0 + 4 * m + j;
            u64 v = (o < c_out && k < n_terms) ? w_res[((size_t)o * n_terms + k) * nl + e] : 0;
            if (DW < WM_DIGITS && v > (q >> 1)) v -= q;  // two's complement of the negative representative
            wv |= (u32)((signed_digits(v) >> (8 * dw)) & 0xffu) << (8 * j);
        }
        words[m] = wv;
    }
    wa[idx] = make_uint4(words[0], words[1], words[2], words[3]);
}

// {a.b[i], b.b[i], c.b[i], d.b[i]} for i = 0..3 from four dwords (a 4x4 byte transpose)
__device__ __forceinline__ void transpose4(u32 a, u32 b, u32 c, u32 d, u32& o0, u32& o1, u32& o2, u32& o3) {
    const u32 ab_lo = __builtin_amdgcn_perm(b, a, 0x05010400u);  // a0 b0 a1 b1
    const u32 ab_hi = __builtin_amdgcn_perm(b, a, 0x07030602u);  // a2 b2 a3 b3
    const u32 cd_lo = __builtin_amdgcn_perm(d, c, 0x05010400u);
    const u32 cd_hi = __builtin_amdgcn_perm(d, c, 0x07030602u);
    o0 = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x05040100u);       // a0 b0 c0 d0
    o1 = __builtin_amdgcn_perm(cd_lo, ab_lo, 0x07060302u);
    o2 = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x05040100u);
    o3 = __builtin_amdgcn_perm(cd_hi, ab_hi, 0x07060302u);
}

// Digits of 16 values (one per term) -> the seven 16-byte B-operand words of this lane.
__device__ __forceinline__ void digits_to_b(const u64* v, uint4* bw) {
    u32 w[7][4];
#pragma unroll
    for (u32 m = 0; m < 4; m++) {
        const u64 s0 = signed_digits(v[4 * m]), s1 = signed_digits(v[4 * m + 1]), s2 = signed_digits(v[4 * m + 2]),
                  s3 = signed_digits(v[4 * m + 3]);
        u32 unused;
        transpose4((u32)s0, (u32)s1, (u32)s2, (u32)s3, w[0][m], w[1][m], w[2][m], w[3][m]);
        transpose4((u32)(s0 >> 32), (u32)(s1 >> 32), (u32)(s2 >> 32), (u32)(s3 >> 32), w[4][m], w[5][m], w[6][m], unused);
    }
#pragma unroll
    for (u32 dx = 0; dx < 7; dx++) bw[dx] = make_uint4(w[dx][0], w[dx][1], w[dx][2], w[dx][3]);
}

// xs: the n_terms operands in layout xl, wa as above, acc [c_out][2][nl][N];  grid = (column groups, 2*nl, OT/2); a
// workgroup takes the `tiles_per_wg` consecutive 64-column tiles of its group, one after the other.
// RAGGED: n_terms is not a multiple of 64 or N is not a multiple of 64 (addresses are clamped and
// the values behind them masked to zero); the regular case carries none of that.
//
// Per 64-term block kb the workgroup needs 28 KiB of weight digits (A operands, shared) and the
// digits of its 64 x 64 values of X (B operands; thread (wave, lane) converts 16 of them: column
// tile wave>>1, terms 32*(wave&1) + 16*(lane>>5) + j, and shares them through LDS with the wave that
// owns the other output tile).  Both live in double-buffered LDS.  The blocks of all the workgroup's tiles form one
// stream: the iteration that multiplies block b stores the weights of block b+1 to LDS, requests the weights and X of
// block b+3, and runs the matrix instructions of block b out of LDS while the vector ALU turns X of block b+1 into
// digits for the other LDS buffer; what it waits for was requested two iterations ago.  The stream does not stop at a
// tile's last block: its reduction and stores run with the next tile's blocks already on their way.
template <int DW, bool RAGGED>
__global__ __launch_bounds__(WM_THREADS) void wsum_mfma_kernel(const u64* __restrict__ xs, XLayout xl, const uint4* __restrict__ wa,
                                                               u64* __restrict__ acc, const ModConstF* __restrict__ mcf,
                                                               const double* __restrict__ pow256, u32 N, u32 level, u32 nl, u32 num_q,
                                                               u32 n_terms, u32 c_out, u32 KB, u32 OT, u32 tiles_per_wg) {
    constexpr int DIAGS = WM_DIGITS + DW - 1;
    constexpr int A_STAGE = WM_OT_PER_WG * DW * 2 * 64;  // uint4 words of one 64-term block of weight digits
    // vector instructions of the digit conversion issued per matrix instruction (about 200 per block in all)
    constexpr int VALU_PER_MFMA = (2 * WM_DIGITS * 2 * WM_DIGITS + DW * 2 * WM_DIGITS - 1) / (DW * 2 * WM_DIGITS);
    __shared__ uint4 lds_a[2][A_STAGE];
    __shared__ uint4 lds_b[2][WM_B_STAGE];  // [column tile 2][32-term step 2][digit 7][lane 64]
    const u32 tid = threadIdx.x, lane = tid & 63;
    const u32 wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u32 g = lane >> 5;                 // which 16 terms of a 32-term step this lane holds
    const u32 wt = wave & 1;                 // output tile this wave owns; also the 32-term step whose X it converts
    const u32 xt = wave >> 1;                // column tile
    const u32 n_tiles = (N + 63) >> 6;
    const u32 tile_first = blockIdx.x * tiles_per_wg;
    if (tile_first >= n_tiles) return;       // whole workgroup
    const u32 tile_last = min(tile_first + tiles_per_wg, n_tiles) - 1;
    const u32 xin = xt * 32 + (lane & 31);   // column inside a tile
    const u32 e = blockIdx.y % nl, comp = blockIdx.y / nl;
    const u32 ot0 = blockIdx.z * WM_OT_PER_WG;
    const size_t ct_stride = (size_t)2 * nl * N;

    v16i d[DIAGS];
#pragma unroll
    for (int s = 0; s < DIAGS; s++)
#pragma unroll
        for (int r = 0; r < 16; r++) d[s][r] = 0;

    // term 64*kb + 32*wt + j + 16*g of column 64*tile + xin: a wave-uniform row pointer plus a 32-bit lane offset
    const u64* xbase = xs + comp * xl.s_comp + e * xl.s_e + (size_t)(32 * wt) * xl.s_k;
    const u32 lane_off = (u32)(16 * g * xl.s_k + xin);
    const u32 tile_step = (u32)xl.s_xt;
    const uint4* wsrc = wa + ((size_t)e * KB * OT + ot0) * (DW * 2 * 64) + tid;  // block kb: + kb * wstep
    const size_t wstep = (size_t)OT * (DW * 2 * 64);
    u64 raw0[16], raw1[16], raw2[16];
    // named, not arrays: they live across the loop's back edge in registers.  Two sets: the weights of two blocks are on
    // their way at any time
    uint4 apA0, apA1, apA2, apA3, apA4, apA5, apA6, apB0, apB1, apB2, apB3, apB4, apB5, apB6;
// no memory operation moves across this point, in any pass of the compiler
#define WM_KEEP_ORDER asm volatile("" ::: "memory"); __builtin_amdgcn_sched_barrier(0);
#define WM_LOAD_X(RAW, TILE, KBLK)                                                                    \
    if (RAGGED) {                                                                                     \
        _Pragma("unroll") for (u32 j = 0; j < 16; j++) {                                              \
            const u32 k = 64 * (KBLK) + 32 * wt + 16 * g + j;                                         \
            const u32 xx = 64 * (TILE) + xin;                                                         \
            RAW[j] = xs[xl.at(k < n_terms ? k : n_terms - 1, comp, e, xx < N ? xx : N - 1)];            \
        }                                                                                             \
    } else { /* one 64-bit address per block, then one addition per term */                           \
        const u64* p__ = xbase + ((size_t)(64 * (KBLK)) * xl.s_k + (size_t)(TILE) * tile_step) + lane_off; \
        _Pragma("unroll") for (u32 j = 0; j < 16; j++) {                                              \
            RAW[j] = *p__;                                                                            \
            p__ += xl.s_k;                                                                            \
        }                                                                                             \
    }
#define WM_MASK_X(RAW, TILE, KBLK)                                                                    \
    if (RAGGED) {                                                                                     \
        _Pragma("unroll") for (u32 j = 0; j < 16; j++)                                                \
            RAW[j] &= (64 * (TILE) + xin < N && 64 * (KBLK) + 32 * wt + 16 * g + j < n_terms) ? ~0ull : 0ull; \
    }
#define WM_A_EACH(OP, S)                                                                             \
    {                                                                                                 \
        if (DW > 0) OP(0, ap##S##0)                                                                   \
        if (DW > 1) OP(1, ap##S##1)                                                                   \
        if (DW > 2) OP(2, ap##S##2)                                                                   \
        if (DW > 3) OP(3, ap##S##3)                                                                   \
        if (DW > 4) OP(4, ap##S##4)                                                                   \
        if (DW > 5) OP(5, ap##S##5)                                                                   \
        if (DW > 6) OP(6, ap##S##6)                                                                   \
    }
#define WM_A_LD(I, V) { V = wsrc[kblk__ * wstep + I * WM_THREADS]; }
#define WM_A_ST(I, V) { lds_a[buf__][tid + I * WM_THREADS] = V; }
#define WM_LOAD_A(S, KBLK) { const size_t kblk__ = (KBLK); WM_A_EACH(WM_A_LD, S) }
#define WM_STORE_A(S, BUF) { const u32 buf__ = (BUF); WM_A_EACH(WM_A_ST, S) }
#define WM_STORE_B(RAW, BUF)                                                                          \
    {                                                                                                 \
        uint4 bw__[7];                                                                                \
        digits_to_b(RAW, bw__);                                                                       \
        _Pragma("unroll") for (u32 dx = 0; dx < 7; dx++) lds_b[BUF][((xt * 2 + wt) * 7 + dx) * 64 + lane] = bw__[dx]; \
    }
// the block after (TILE, KBLK) in the workgroup's stream; the stream's last block follows itself
#define WM_ADVANCE(TILE, KBLK)                                                                        \
    {                                                                                                 \
        if ((KBLK) + 1 < KB) (KBLK)++;                                                                \
        else if ((TILE) < tile_last) { (TILE)++; (KBLK) = 0; }                                        \
    }
// One iteration on LDS buffer CUR: multiplies block b = (tile_c, kb_c).  On entry the requests of two iterations are
// outstanding, oldest first: [weights of b+1 (register set S), X of b+1 (RAW_OLD)], [weights of b+2, X of b+2].  The
// iteration waits for the first pair only (loads return in order), stores those weights to LDS, requests
// [weights of b+3 (set S again), X of b+3 (RAW_NEW, whose block b was converted an iteration ago)], and runs the matrix
// instructions of block b while the vector ALU turns X of b+1 into digits: two blocks stay on their way throughout,
// the tile's last fold and stores included.
#define WM_ITER(CUR, S, RAW_NEW, RAW_OLD)                                                             \
    {                                                                                                 \
        constexpr u32 cur = (CUR);                                                                    \
        __syncthreads(); /* this block of both operands is in LDS[cur]; everyone is done with LDS[cur ^ 1] */ \
        const uint4* la = &lds_a[cur][wt * (DW * 2 * 64) + lane];                                     \
        const uint4* lb = &lds_b[cur][xt * (2 * WM_DIGITS * 64) + lane];                              \
        /* first the 32-term step ks = 0 with every weight digit, then ks = 1: seven B operands are held at a time; */ \
        /* the A operand of the next group of seven and, in the last group of ks = 0, the B operands of ks = 1 are */ \
        /* read from LDS a group (more than the LDS latency) ahead of their use */                     \
        v4i b[WM_DIGITS], bn[WM_DIGITS];                                                              \
        uint4 av = la[0], avn = av; /* first: the four waves read at once, and the first instruction needs this one */ \
        __builtin_amdgcn_sched_barrier(0);                                                            \
        _Pragma("unroll") for (u32 dx = 0; dx < WM_DIGITS; dx++) {                                    \
            const uint4 t = lb[dx * 64];                                                              \
            b[dx] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};                                    \
        }                                                                                             \
        _Pragma("unroll") for (u32 grp = 0; grp < 2 * DW; grp++) {                                    \
            const u32 dw = grp % DW;                                                                  \
            if (grp + 1 < 2 * DW) avn = la[(((grp + 1) % DW) * 2 + (grp + 1) / DW) * 64];             \
            if (grp == DW - 1) {                                                                      \
                _Pragma("unroll") for (u32 dx = 0; dx < WM_DIGITS; dx++) {                            \
                    const uint4 t = lb[(WM_DIGITS + dx) * 64];                                        \
                    bn[dx] = (v4i){(int)t.x, (int)t.y, (int)t.z, (int)t.w};                           \
                }                                                                                     \
            }                                                                                         \
            const v4i a = (v4i){(int)av.x, (int)av.y, (int)av.z, (int)av.w};                          \
            _Pragma("unroll") for (u32 dx = 0; dx < WM_DIGITS; dx++)                                  \
                d[dx + dw] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[dx], d[dx + dw], 0, 0, 0);    \
            av = avn;                                                                                 \
            if (grp == DW - 1) { _Pragma("unroll") for (u32 dx = 0; dx < WM_DIGITS; dx++) b[dx] = bn[dx]; } \
        }                                                                                             \
        /* everything else of the iteration rides between the matrix instructions (see the issue order below) */ \
        WM_STORE_A(S, cur ^ 1)                                                                        \
        WM_LOAD_A(S, kb_x)                                                                            \
        WM_LOAD_X(RAW_NEW, tile_x, kb_x)                                                              \
        WM_MASK_X(RAW_OLD, tile_n, kb_n)                                                              \
        WM_STORE_B(RAW_OLD, cur ^ 1)                                                                  \
        /* issue order: the LDS reads that start the block; then per matrix instruction a few vector instructions */ \
        /* (digit conversion, addresses) and one memory instruction: the stores of the weights to LDS during the */ \
        /* first group, then the requests of the block three ahead, the stores of the converted digits at the end; */ \
        /* each group starts with the LDS reads of the next group's operands */                        \
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);                                            \
        _Pragma("unroll") for (u32 grp = 0; grp < 2 * DW; grp++) {                                    \
            if (grp == DW - 1) __builtin_amdgcn_sched_group_barrier(0x100, 1 + WM_DIGITS, 0);         \
            else if (grp + 1 < 2 * DW) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);             \
            _Pragma("unroll") for (u32 q = 0; q < WM_DIGITS; q++) {                                   \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
                if (grp < DW) __builtin_amdgcn_sched_group_barrier(0x002, 2 * VALU_PER_MFMA - 2, 0); \
                else __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);                               \
                if (grp == 0 && q < DW) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);            \
                else if (grp * WM_DIGITS + q < DW + 4 + 16) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0); \
                else if (grp * WM_DIGITS + q >= DW * WM_DIGITS + 4 && grp * WM_DIGITS + q < DW * WM_DIGITS + 4 + 2 * WM_DIGITS && ((q & 1) == 0)) \
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                \
            }                                                                                         \
        }                                                                                             \
        __builtin_amdgcn_sched_group_barrier(0x200, 7, 0);                                            \
        __builtin_amdgcn_sched_barrier(0);                                                            \
        if (kb_c + 1 == KB && gb < n_blocks) fold_and_store(tile_c);                                  \
        gb++;                                                                                         \
        tile_c = tile_n, kb_c = kb_n;                                                                 \
        tile_n = tile_l, kb_n = kb_l;                                                                 \
        tile_l = tile_x, kb_l = kb_x;                                                                 \
        WM_ADVANCE(tile_x, kb_x)                                                                      \
    }

    // sum_s D_s 2^(8s) is the exact sum of products; modulo q it equals sum_s D_s c_s with c_s = 2^(8s) mod q, taken in
    // exact double-precision sums (f64m_fold_diagonals).  Leaves the accumulators at zero.
    const u32 mi = e <= level ? e : num_q + (e - level - 1);
    auto fold_and_store = [&](u32 tile) {
        const u32 x = 64 * tile + xin;
        const ModConstF m = mcf[mi];
        const double* __restrict__ pw = pow256 + (size_t)mi * POW256_ROW;
        double cp[3 * DIAGS];
#pragma unroll
        for (u32 s = 0; s < 3 * DIAGS; s++) cp[s] = pw[s];
        const double w17 = pw[39], w17q = pw[40];
        const size_t off = ((size_t)comp * nl + e) * N + x;
#pragma unroll
        for (u32 r = 0; r < 16; r++) {
            const u32 o = 32 * (ot0 + wt) + 8 * (r >> 2) + 4 * g + (r & 3);
            int ds[DIAGS];
#pragma unroll
            for (u32 s = 0; s < DIAGS; s++) {
                // the sums stay in the accumulator registers across the loop; read one, clear it
                int zero;
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(ds[s]) : "a"(d[s][r]));
                asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(zero));
                d[s][r] = zero;
            }
            const double v = f64m_fold_diagonals<DIAGS>(ds, cp, w17, w17q, m.q, m.qinv);
            if (o < c_out && (!RAGGED || x < N)) acc[(size_t)o * ct_stride + off] = f64m_canonical(v, m.q);
            __builtin_amdgcn_sched_barrier(0);  // one output at a time: the loads in flight own most of the registers
        }
    };

    u32 tile_c = tile_first, kb_c = 0;
    u32 tile_n = tile_c, kb_n = kb_c;
    WM_ADVANCE(tile_n, kb_n)
    u32 tile_l = tile_n, kb_l = kb_n;
    WM_ADVANCE(tile_l, kb_l)
    u32 tile_x = tile_l, kb_x = kb_l;
    WM_ADVANCE(tile_x, kb_x)
    WM_LOAD_A(A, 0)
    WM_STORE_A(A, 0)
    WM_LOAD_X(raw0, tile_c, kb_c)
    WM_MASK_X(raw0, tile_c, kb_c)
    WM_STORE_B(raw0, 0)
    // the two pairs of requests the loop expects, in its order
    WM_KEEP_ORDER
    WM_LOAD_A(B, kb_n)
    WM_KEEP_ORDER
    WM_LOAD_X(raw1, tile_n, kb_n)
    WM_KEEP_ORDER
    WM_LOAD_A(A, kb_l)
    WM_KEEP_ORDER
    WM_LOAD_X(raw2, tile_l, kb_l)
    WM_KEEP_ORDER
    // three register buffers of X, two sets of weights and two LDS buffers: the pattern repeats every six blocks
    const u32 n_blocks = (tile_last - tile_first + 1) * KB;
    // No way out of the loop but its end (an early exit would be one more way into its head for the compiler's account of
    // outstanding requests, and every wait in the loop would be set for the worst of them): the stream is run to a
    // multiple of six blocks; the extra iterations repeat the last block into accumulators that are not read again.
    u32 gb = 0;
    do {  // at least one block: no branch between the requests above and the loop, so their order stands
        WM_ITER(0, B, raw0, raw1)
        WM_ITER(1, A, raw1, raw2)
        WM_ITER(0, B, raw2, raw0)
        WM_ITER(1, A, raw0, raw1)
        WM_ITER(0, B, raw1, raw2)
        WM_ITER(1, A, raw2, raw0)
    } while (gb < n_blocks);
#undef WM_LOAD_X
#undef WM_KEEP_ORDER
#undef WM_MASK_X
#undef WM_LOAD_A
#undef WM_STORE_A
#undef WM_STORE_B
#undef WM_ITER
#undef WM_ADVANCE
#undef WM_A_EACH
#undef WM_A_LD
#undef WM_A_ST
}

bool wsum_mfma_applies(const ckks_ctx* c, u32 n_terms) { return c->small_q && n_terms <= c->lazy_terms && n_terms <= 4096; }

// digits the weights are written in, from the caller's bound |w| < 2^(weight_bits - 1) (0 = none: any residue)
static u32 weight_digits(u32 weight_bits) { return weight_bits == 0 || weight_bits > 32 ? WM_DIGITS : (weight_bits <= 24 ? 3 : 4); }

// scratch words (u64) for the weight digit planes (sized for the widest weights)
size_t wsum_mfma_scratch_elems(u32 n_limbs, u32 n_terms, u32 c_out) {
    const size_t KB = (n_terms + 63) / 64, OT = (c_out + 63) / 64 * WM_OT_PER_WG;
    return (size_t)n_limbs * KB * OT * WM_DIGITS * 2 * 64 * 2;  // 16 bytes per lane
}

template <int DW>
static void launch_wsum_dw(bool ragged, dim3 grid, hipStream_t st, const u64* xs, XLayout xl, const uint4* wa, u64* acc, const ckks_ctx* c,
                           u32 level, u32 nl, u32 n_terms, u32 c_out, u32 KB, u32 OT, u32 tiles_per_wg) {
    if (ragged)
        hipLaunchKernelGGL((wsum_mfma_kernel<DW, true>), grid, dim3(WM_THREADS), 0, st, xs, xl, wa, acc, c->d_mcf, c->d_pow256, c->N, level, nl,
                           c->num_q, n_terms, c_out, KB, OT, tiles_per_wg);
    else
        hipLaunchKernelGGL((wsum_mfma_kernel<DW, false>), grid, dim3(WM_THREADS), 0, st, xs, xl, wa, acc, c->d_mcf, c->d_pow256, c->N, level, nl,
                           c->num_q, n_terms, c_out, KB, OT, tiles_per_wg);
}

hipError_t launch_wsum_mfma(const ckks_ctx* c, u32 level, u32 nl, const u64* xs, XLayout xl, u32 n_terms, const u64* w_res, u32 c_out,
                            u64* acc, u64* scratch, u32 weight_bits, hipStream_t st) {
    const u32 KB = (n_terms + 63) / 64, OT = (c_out + 63) / 64 * WM_OT_PER_WG, DW = weight_digits(weight_bits);
    const size_t prep = (size_t)nl * KB * OT * DW * 2 * 64;
    hipLaunchKernelGGL(wsum_prep_kernel, dim3((u32)((prep + WM_THREADS - 1) / WM_THREADS)), dim3(WM_THREADS), 0, st, w_res,
                       (uint4*)scratch, c->d_mc, level, c->num_q, c_out, n_terms, nl, KB, OT, DW);
    // tiles of one workgroup: enough that the start and the end of its stream are a small part of it, few enough that the
    // chip's 256 CUs still get many workgroups each (16 tiles: 4096 workgroups at N = 2^16 and 32 limbs)
    const u32 n_tiles = (c->N + 63) / 64, tiles_per_wg = n_tiles < WM_TILES_PER_WG ? n_tiles : WM_TILES_PER_WG;
    dim3 grid((n_tiles + tiles_per_wg - 1) / tiles_per_wg, 2 * nl, OT / WM_OT_PER_WG);
    // the 32-bit lane offset of the regular kernel spans 16 terms: 16 * (2 * nl * N) words must fit
    const bool ragged = (n_terms & 63) || (c->N & 63) || 16 * xl.s_k + (size_t)(c->N >> 6) * xl.s_xt + 64 > 0xffffffffull;
    if (DW == 3) launch_wsum_dw<3>(ragged, grid, st, xs, xl, (const uint4*)scratch, acc, c, level, nl, n_terms, c_out, KB, OT, tiles_per_wg);
    else if (DW == 4) launch_wsum_dw<4>(ragged, grid, st, xs, xl, (const uint4*)scratch, acc, c, level, nl, n_terms, c_out, KB, OT, tiles_per_wg);
    else launch_wsum_dw<WM_DIGITS>(ragged, grid, st, xs, xl, (const uint4*)scratch, acc, c, level, nl, n_terms, c_out, KB, OT, tiles_per_wg);
    return hipGetLastError();
}
