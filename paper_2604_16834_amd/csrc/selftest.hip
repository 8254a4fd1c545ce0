// Self-test hook: the double-precision modular routines (f64mod.h) evaluated by the GPU on caller-given operands, so
// that a test can judge the device's results with 128-bit integers as it judges the host's.
#include "ctx.h"
#include "f64mod.h"

__global__ __launch_bounds__(256) void f64mod_probe_kernel(int op, const long long* __restrict__ y, const u64* __restrict__ w,
                                                          const double* __restrict__ wq, double q, double qinv, double* __restrict__ out,
                                                          size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const double yd = (double)y[i];
    double r;
    switch (op) {
        case CKKS_F64_MULMOD: r = f64m_mulmod(yd, f64m_from_u64(w[i]), wq[i], q); break;
        case CKKS_F64_MULMOD_ANY: r = f64m_mulmod_any(yd, f64m_from_u64(w[i]), q, qinv); break;
        case CKKS_F64_REDUCE: r = f64m_reduce(yd, q, qinv); break;
        case CKKS_F64_CANONICAL: r = (double)f64m_canonical(f64m_reduce(yd, q, qinv), q); break;
        default: r = f64m_centre(f64m_mulmod(yd, f64m_from_u64(w[i]), wq[i], q), q); break;  // CKKS_F64_CENTRE
    }
    out[i] = r;
}

// the conversion sum of ND terms: row i of y ([n][ND] centred residues) against the ND constants w (in [0, q); their centred
// representatives are formed here as the library's tables hold them)
template <int ND>
__global__ __launch_bounds__(256) void f64mod_dot_probe_kernel(const long long* __restrict__ y, const u64* __restrict__ w, u64 qi, double q,
                                                              double qinv, double* __restrict__ out, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double yv[ND], wv[ND];
#pragma unroll
    for (int a = 0; a < ND; a++) {
        yv[a] = (double)y[i * ND + a];
        wv[a] = w[a] > (qi >> 1) ? -f64m_from_u64(qi - w[a]) : f64m_from_u64(w[a]);
    }
    out[i] = f64m_dot_w<ND>(yv, wv, q, qinv);
}

extern "C" int ckks_f64mod_probe(int op, const int64_t* d_y, const uint64_t* d_w, const double* d_wq, uint64_t q, double* d_out, size_t n,
                                 void* stream) {
    if (op < CKKS_F64_MULMOD || op > CKKS_F64_DOT9 || !d_y || !d_out || q < 2 || q >= (1ull << 50)) return CKKS_ERR_INVALID_ARG;
    if (op == CKKS_F64_DOT8 || op == CKKS_F64_DOT9) {
        if (!d_w) return CKKS_ERR_INVALID_ARG;
        if (n == 0) return CKKS_OK;
        const size_t nb = (n + 255) / 256;
        if (nb > 0x7fffffffull) return CKKS_ERR_INVALID_ARG;
        if (op == CKKS_F64_DOT8)
            hipLaunchKernelGGL(f64mod_dot_probe_kernel<8>, dim3((unsigned)nb), dim3(256), 0, (hipStream_t)stream, (const long long*)d_y,
                               (const u64*)d_w, (u64)q, (double)q, 1.0 / (double)q, d_out, n);
        else
            hipLaunchKernelGGL(f64mod_dot_probe_kernel<9>, dim3((unsigned)nb), dim3(256), 0, (hipStream_t)stream, (const long long*)d_y,
                               (const u64*)d_w, (u64)q, (double)q, 1.0 / (double)q, d_out, n);
        return hipGetLastError() == hipSuccess ? CKKS_OK : CKKS_ERR_HIP;
    }
    const bool needs_w = op == CKKS_F64_MULMOD || op == CKKS_F64_MULMOD_ANY || op == CKKS_F64_CENTRE;
    if (needs_w && (!d_w || (op != CKKS_F64_MULMOD_ANY && !d_wq))) return CKKS_ERR_INVALID_ARG;
    if (n == 0) return CKKS_OK;
    const size_t blocks = (n + 255) / 256;
    if (blocks > 0x7fffffffull) return CKKS_ERR_INVALID_ARG;
    hipLaunchKernelGGL(f64mod_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, op, (const long long*)d_y,
                       (const u64*)d_w, d_wq, (double)q, 1.0 / (double)q, d_out, n);
    return hipGetLastError() == hipSuccess ? CKKS_OK : CKKS_ERR_HIP;
}
