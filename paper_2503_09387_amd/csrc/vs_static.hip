// vs_decode_attn_static: vs_decode_attn for callers that cannot hand over a workspace of device
// memory they allocated (code under HIP graph capture, tight serving loops, harnesses that
// forbid allocation).  The partial results of the row shares live in an array that is part of
// the library's own code object on every device; nothing is allocated, here or in any routine
// this file calls.
#include "vs_internal.h"

namespace {

constexpr size_t kScratchBytes = size_t(16) << 20;  // per device, held until the process ends

// (In host code this name is only a handle for hipGetSymbolAddress: it is not a device address.
// Each device has its own copy of the array at its own address.)
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

unsigned char* g_scratch_ptr[16] = {};  // device address of `scratch` on device d, once asked for

// The device address of this device's array; asked for once per device, with that device current.
hipError_t scratch_of_current_device(unsigned char** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" {

size_t vs_decode_static_scratch_bytes(void) { return kScratchBytes; }

vs_status vs_decode_attn_static(const vs_shape* shape, int32_t n_streams, void* k_slab, void* v_slab,
                                int32_t capacity, int32_t* lens, const void* q, const void* k_new,
                                const void* v_new, void* out, void* hip_stream) {
    if (!shape) return VS_ERR_NULL;
    // what vs_decode_attn would ask of a workspace for this call must fit the array
    const size_t need = vs_workspace_bytes(shape, 0, capacity > 0 ? capacity : 0, n_streams > 0 ? n_streams : 0);
    if (need == 0) return vs::decode_entry(shape, n_streams, k_slab, v_slab, capacity, lens, q, k_new, v_new, out,
                                           nullptr, 0, hip_stream);  // (reports what is wrong with the arguments)
    if (need > kScratchBytes) return VS_ERR_WORKSPACE;
    (void)hipGetLastError();
    unsigned char* ptr = nullptr;
    if (scratch_of_current_device(&ptr) != hipSuccess) return VS_ERR_HIP;
    // Nothing in the array has to be zero for a decode call: every partial result that the merge
    // reads is written earlier in the same call.
    return vs::decode_entry(shape, n_streams, k_slab, v_slab, capacity, lens, q, k_new, v_new, out, ptr,
                            kScratchBytes, hip_stream);
}

}  // extern "C"
