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
