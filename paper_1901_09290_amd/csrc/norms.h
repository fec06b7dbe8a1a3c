// Group-norm launcher shared by the entry points of lasso.hip and norms_static.hip.
#pragma once

#include "common.h"

namespace pt {

// One layer of a norms launch (the public descriptors are mapped onto this).
struct NormLayer {
    const float* w;
    float* out_norm;
    float* in_norm;
    uint16_t* shadow;   // nullptr: no bf16 copy
    uint8_t* zero_out;  // nullptr, or [K]: also write (out_norm < thr)
    uint8_t* zero_in;   // nullptr, or [C]
    int32_t K, RS, C, cpitch;
};

int32_t check_norm_layer(const NormLayer& L);
size_t norm_layer_ws_bytes(int32_t K, int32_t RS, int32_t C);
// Group norms (and zero masks where asked for) of n layers; `ws` is device memory of at least the layers' summed
// norm_layer_ws_bytes, 16-byte aligned, fully written before it is read (nothing in it needs clearing).
int32_t launch_norms(const NormLayer* layers, int n, void* ws, size_t ws_bytes, float thr, hipStream_t st);

}  // namespace pt
