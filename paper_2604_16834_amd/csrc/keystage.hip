// Staged switching keys ("Optimized Inference Pipeline", Evaluation Keys Reuse: only the keys of the current block
// group are resident, sets are offloaded and loaded between groups).  A key is [digit][b|a][limb][N]; its public
// halves a_j are uniform residues and carry no information, so they are a function of a 64-bit seed: the host
// keeps and moves only the b_j halves (half the bytes over the host link) and the a_j are written on the device.
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace {

// Output number `index` of the stream that a seed expands to.  This is the one function to replace for deployment: the
// stream here is the SplitMix64 sequence started at `seed` (Steele, Lea, Flood 2014; the state advances by a constant, so
// every output can be computed on its own), which is a benchmarking stand-in, not a cryptographic expansion: seeded
// public key halves need a PRF / XOF keyed with at least 128 bits.
__device__ __forceinline__ u64 seed_stream_at(u64 seed, u64 index) {
    u64 z = seed + (index + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// a[j][t][x] of the key: element e = (j*M + t)*N + x takes outputs 64e, 64e+1, ...; the top bitlength(q) bits of
// the first one below q are the value (exactly uniform); after 64 rejections the last output is reduced.
__global__ __launch_bounds__(256) void key_expand_a_kernel(u64* __restrict__ key, u64 seed, const ModConst* __restrict__ mc, u32 N,
                                                           u32 M) {
    const u32 x = blockIdx.x * 256 + threadIdx.x;
    if (x >= N) return;
    const u32 t = blockIdx.y, j = blockIdx.z;
    const u64 q = mc[t].q;
    const u32 shift = (u32)__builtin_clzll(q);  // 64 - bitlength(q)
    const u64 e = ((u64)j * M + t) * N + x;
    u64 z = 0, v = 0;
    bool found = false;
    for (u32 attempt = 0; attempt < 64 && !found; attempt++) {
        z = seed_stream_at(seed, e * 64 + attempt);
        v = z >> shift;
        found = v < q;
    }
    if (!found) v = z % q;
    key[(((size_t)j * 2 + 1) * M + t) * N + x] = v;
}

}  // namespace

hipError_t launch_key_expand_a(const ckks_ctx* c, u64 seed, u64* key, hipStream_t st) {
    dim3 grid((c->N + 255) / 256, c->M, c->dnum);
    hipLaunchKernelGGL(key_expand_a_kernel, grid, dim3(256), 0, st, key, seed, c->d_mc, c->N, c->M);
    return hipGetLastError();
}
