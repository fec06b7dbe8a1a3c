// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "prunetrain.h"

namespace pt {

constexpr int kWave = 64;

// Records the last failing HIP error for pt_last_hip_error().
void set_hip_error(hipError_t e);

inline int32_t launch_status() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e);
        return PT_ERR_LAUNCH;
    }
    return PT_OK;
}

// One-time opt-in of a kernel to `lds` bytes of dynamic LDS (needed above 64 KiB), kept per device: bit d of `done`
// says the attribute is set on device d.  Safe from any host thread: the attribute call is idempotent, so two
// threads racing through the first call both succeed.
struct LdsOptIn {
    std::atomic<uint64_t> done{0};
    hipError_t ensure(const void* kernel, size_t lds, size_t always_above = 65536) {
        if (lds <= always_above) return hipSuccess;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const uint64_t bit = 1ull << (dev & 63);
        if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        done.fetch_or(bit, std::memory_order_release);
        return hipSuccess;
    }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// fp32 -> bf16 bits, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Two fp32 -> packed bf16x2 (lo in bits 15:0) with the hardware converter (round to nearest even).
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    f32x2_t f = {lo, hi};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

// Exact floor(m / d) for m*d < 2^32 with magic = floor(2^32 / d) + 1 (computed on the host).
__device__ __forceinline__ uint32_t fast_div(uint32_t m, uint32_t magic) { return __umulhi(m, magic); }
inline uint32_t make_magic(uint32_t d) { return (uint32_t)((((uint64_t)1) << 32) / d + 1); }

}  // namespace pt
