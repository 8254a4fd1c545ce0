// The slot automorphism sigma_g in evaluation (bit-reversed) order, as a gather index (device code only).
#pragma once
#include "ctx.h"

__device__ __forceinline__ u32 galois_gather_index(u32 k, u32 g, u32 log_n) {
    // evaluation point of entry k is psi^(2*brv(k)+1); sigma_g reads the entry whose point is that
    // power times g
    u32 e = ((2u * (__brev(k) >> (32 - log_n)) + 1u) * g) & ((2u << log_n) - 1u);
    return __brev((e - 1u) >> 1) >> (32 - log_n);
}
