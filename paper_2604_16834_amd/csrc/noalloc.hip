// Rescale for callers that cannot allocate or hand over a workspace (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): the same kernels as ckks_rescale, with their scratch (the dropped limb in coefficient
// form and the first-pass output of the forward transforms) in a device array that is part of the library's image.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process ends.  The array's
// name is only a host-side handle: the device address comes from hipGetSymbolAddress, once per device, with that device
// current (at context creation, else at the first call), and only that address is ever handed to kernels.
// All calls on one GPU share the array: calls that overlap in time on one GPU race.  Nothing has to be cleared between
// calls: every word of the scratch that a call reads was written earlier in the same call.
#include <mutex>

#include "ctx.h"

static __device__ __align__(256) unsigned char scratch[CKKS_NOALLOC_SCRATCH_BYTES];

#define NOALLOC_MAX_DEVICES 64
static void* g_scratch_ptr[NOALLOC_MAX_DEVICES];  // device address of `scratch` on each device, null until looked up
static std::mutex g_scratch_lock;

// The device address of the scratch array on the current device (looked up on first use).
hipError_t noalloc_scratch_current_device(int* device, void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    if (device) *device = dev;
    if (ptr) *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

extern "C" int ckks_rescale_noalloc(const ckks_ctx* c, const uint64_t* d_ct, uint32_t level, uint64_t* d_out, void* stream) {
    if (!c) return CKKS_ERR_INVALID_ARG;
    const size_t need = ckks_workspace_bytes(c, CKKS_OP_RESCALE, level, 1);  // 0: level out of range (ckks_rescale reports it)
    if (need > (size_t)CKKS_NOALLOC_SCRATCH_BYTES) {
        c->err = "ckks_rescale_noalloc: this ring size and level need " + std::to_string(need) + " bytes of scratch, the built-in buffer has " +
                 std::to_string((size_t)CKKS_NOALLOC_SCRATCH_BYTES) + "; use ckks_rescale with a workspace";
        return CKKS_ERR_UNSUPPORTED_PARAMS;
    }
    int dev = -1;
    void* ptr = nullptr;
    const hipError_t e = noalloc_scratch_current_device(&dev, &ptr);
    if (e != hipSuccess) {
        c->err = std::string("ckks_rescale_noalloc: ") + hipGetErrorString(e);
        return CKKS_ERR_HIP;
    }
    if (dev != c->device) {
        c->err = "ckks_rescale_noalloc: the context was created on another device than the current one";
        return CKKS_ERR_INVALID_ARG;
    }
    return ckks_rescale(c, d_ct, level, d_out, ptr, (size_t)CKKS_NOALLOC_SCRATCH_BYTES, stream);
}
