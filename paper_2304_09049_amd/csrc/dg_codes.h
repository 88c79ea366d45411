// Packing in registers: for kernels that read activation codes still one per byte and do the run-time packing stage in
// their own load stage.
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>

// 16 codes, one per byte, into one packed word, code i at bits 2i; bits above a code's two are dropped, as the packing
// kernel drops them.  The four dwords are transposed bytewise (8 permutes), so that dword b holds codes b, 4+b, 8+b, 12+b,
// one per byte; shifted left by 2b and merged bit-field-wise they are the word (every bit of it has exactly one source:
// 14 instructions).
__device__ __forceinline__ uint32_t dg_pack_codes16(uint4 t)
{
    const uint32_t a0 = __builtin_amdgcn_perm(t.y, t.x, 0x05010400u), a1 = __builtin_amdgcn_perm(t.y, t.x, 0x07030602u);
    const uint32_t b0 = __builtin_amdgcn_perm(t.w, t.z, 0x05010400u), b1 = __builtin_amdgcn_perm(t.w, t.z, 0x07030602u);
    const uint32_t z0 = __builtin_amdgcn_perm(b0, a0, 0x05040100u), z1 = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
    const uint32_t z2 = __builtin_amdgcn_perm(b1, a1, 0x05040100u), z3 = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
    auto merge = [](uint32_t mask, uint32_t x, uint32_t rest) { return (x & mask) | (rest & ~mask); };
    uint32_t w = merge(0x0C0C0C0Cu, z1 << 2, z0);
    w = merge(0x30303030u, z2 << 4, w);
    return merge(0xC0C0C0C0u, z3 << 6, w);
}
