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

// The same code by clamping in binary32 (fewer instructions; for epilogues that quantise many values per lane):
// max(r, lo) keeps lo when r is NaN (IEEE maxNum), min(., lo + 3) bounds it above, and the difference to lo -- an
// integer between 0 and 3 -- is exact.  Equal to dg_quantize_code for every input.
__device__ __forceinline__ uint32_t dg_quantize_code_clamped(float x, float s, float z, float lo_f, float hi_f)
{
    const float r = rintf(__fadd_rn(__fmul_rn(s, x), z));
    return (uint32_t)(int)(fminf(fmaxf(r, lo_f), hi_f) - lo_f);
}
