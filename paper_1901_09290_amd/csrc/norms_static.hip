// Group norms of one layer for callers that cannot allocate device memory: the scratch the two kernels need (row
// sums and per-chunk column partials) lives in an array the library holds on every device it runs on.
#include <atomic>

#include "norms.h"

namespace pt {

constexpr size_t kStaticScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code the array's name is only a handle for hipGetSymbolAddress: each device has its own copy at its own
// address.  That address is resolved once per device, with the device current, and is what the kernels receive.
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int32_t static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_hip_error(e);
        return PT_ERR_LAUNCH;
    }
    if (dev < 0 || dev >= kMaxDevices) return PT_ERR_UNSUPPORTED;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return PT_ERR_LAUNCH;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing first calls resolve the same address
    }
    *out = p;
    return PT_OK;
}

}  // namespace pt

using namespace pt;

extern "C" int32_t pt_group_norms_static(const float* w, int32_t K, int32_t RS, int32_t C, int32_t w_cpitch,
                                         float* out_norm, float* in_norm, uint16_t* w_shadow, void* stream) {
    const NormLayer L{w, out_norm, in_norm, w_shadow, nullptr, nullptr, K, RS, C, w_cpitch};
    int32_t rc = check_norm_layer(L);
    if (rc != PT_OK) return rc;
    if (norm_layer_ws_bytes(K, RS, C) > kStaticScratchBytes) return PT_ERR_WORKSPACE;  // layer too large for the held scratch
    void* p = nullptr;
    rc = static_scratch(&p);
    if (rc != PT_OK) return rc;
    return launch_norms(&L, 1, p, kStaticScratchBytes, 0.f, (hipStream_t)stream);
}
