// Small device-side math shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>

// sigmoid(z) with exp2 on the hardware unit; the product z * log2(e) is
// carried in two parts so the relative error stays ~1e-7 for |z| up to ~80.
__device__ __forceinline__ float sigmoid_f32(float z)
{
    const float nz = -z;
    const float l2e_hi = 1.44269502162933349609375f, l2e_lo = 1.92596299e-8f;
    const float t = nz * l2e_hi;
    const float tl = fmaf(nz, l2e_hi, -t) + nz * l2e_lo;
    const float e = __builtin_amdgcn_exp2f(t) * fmaf(tl, 0.693147182f, 1.0f);
    return __builtin_amdgcn_rcpf(1.0f + e);
}

// g = sigmoid(z) and d = g (1 - g) = sigmoid(z) sigmoid(-z), both to about 1e-7 relative. With e = exp(-|z|) and
// r = 1 / (1 + e): sigmoid(|z|) = r, sigmoid(-|z|) = e r, and the slope is e r r. The difference 1 - g is never
// formed, so a saturated gate keeps its (tiny) slope's relative accuracy.
__device__ __forceinline__ void sigmoid_and_slope_f32(float z, float& g, float& d)
{
    const float nz = -fabsf(z);
    const float l2e_hi = 1.44269502162933349609375f, l2e_lo = 1.92596299e-8f;
    const float t = nz * l2e_hi;
    const float tl = fmaf(nz, l2e_hi, -t) + nz * l2e_lo;
    const float e = __builtin_amdgcn_exp2f(t) * fmaf(tl, 0.693147182f, 1.0f);
    const float r = __builtin_amdgcn_rcpf(1.0f + e);
    const float small = e * r;  // sigmoid(-|z|)
    g = z >= 0.0f ? r : small;
    d = small * r;
}
