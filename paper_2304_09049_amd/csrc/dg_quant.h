// The activation quantiser (Sec. 2.1, Eq. 1) as the kernels apply it, operation by operation in binary32:
// multiply, add (never fused), round half to even, clip.  NaN fails every comparison and therefore yields code 0.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ uint32_t dg_quantize_code(float x, float s, float z, float lo_f, float hi_f, int lo)
{
    const float r = rintf(__fadd_rn(__fmul_rn(s, x), z));
    int q = lo;
    if (r > lo_f) q = r >= hi_f ? lo + 3 : (int)r;
    return (uint32_t)(q - lo);
}
