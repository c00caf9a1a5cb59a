// kunlun_gdpa_fwd_static: the forward entry point for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and so cannot size and provide the
// workspace that kunlun_gdpa_fwd asks for.  The work lists of the call (issue order of the examples, or the
// query-tile tables) go into a fixed array in device memory that is part of the library image instead.
#include <mutex>

#include "common.h"

namespace {

// The scratch array.  Every GPU the library runs on holds its own copy, at its own address, until the process
// ends.  In host code the NAME of the array is only a stand-in (not a device address): the address on the
// current device comes from hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[KUNLUN_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_ptr[MAX_DEVICES];  // per device; null = not looked up yet

// Device address of `scratch` on the current device (looked up on the first call on that device).
hipError_t scratch_on_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int kunlun_gdpa_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                                      const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                                      int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* stream) {
    // every check of kunlun_gdpa_fwd first, against a stand-in workspace of the full size (host only) ...
    int rc = kunlun::gdpa_fwd_checked(q, k, v, o, lse, q_offsets, kv_offsets, B, H, d, max_q, max_kv, total_q, total_kv, scale,
                                      act, head_act, dtype, (void*)(uintptr_t)256, (size_t)-1, stream, false, false);
    if (rc != KUNLUN_OK) return rc;
    if (B == 0 || total_q == 0) return KUNLUN_OK;
    // ... then the one limit of this entry point: the work lists must fit the fixed array
    const size_t need = kunlun_workspace_bytes(KUNLUN_OP_GDPA_FWD, B, H, d, max_q, max_kv, total_q, total_kv);
    if (need == 0 || need > (size_t)KUNLUN_STATIC_SCRATCH_BYTES) return KUNLUN_ERR_WORKSPACE;
    void* ws = nullptr;
    if (scratch_on_current_device(&ws) != hipSuccess) return KUNLUN_ERR_LAUNCH;
    // The kernels overwrite every entry of the work lists they read, so nothing in the array has to start at
    // zero and no fill is enqueued; whatever the previous call left behind is dead.
    return kunlun::gdpa_fwd_checked(q, k, v, o, lse, q_offsets, kv_offsets, B, H, d, max_q, max_kv, total_q, total_kv, scale, act,
                                    head_act, dtype, ws, (size_t)KUNLUN_STATIC_SCRATCH_BYTES, stream, true, false);
}
