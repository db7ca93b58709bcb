// Device-side helpers shared by the kernels: bf16 conversion, activations, 16-byte row chunks.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "dgi.h"

namespace dgi {

__device__ __forceinline__ float bf16_to_float(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// round to nearest even (v_cvt_pk_bf16_f32 on gfx950); NaN stays NaN
__device__ __forceinline__ uint16_t float_to_bf16(float f) {
    const __bf16 h = static_cast<__bf16>(f);
    uint16_t u;
    __builtin_memcpy(&u, &h, 2);
    return u;
}

__device__ __forceinline__ float activate(float x, int act, float slope) {
    switch (act) {
        case DGI_ACT_RELU: return x > 0.f ? x : 0.f;
        case DGI_ACT_ELU: return x > 0.f ? x : slope * expm1f(x);
        case DGI_ACT_LEAKY_RELU: return x > 0.f ? x : slope * x;
        default: return x;
    }
}

__device__ __forceinline__ void store_element(void* out, int64_t offset, float v, int out_bf16) {
    if (out_bf16) static_cast<uint16_t*>(out)[offset] = float_to_bf16(v);
    else static_cast<float*>(out)[offset] = v;
}

}  // namespace dgi
